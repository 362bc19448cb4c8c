/*
 * unetglue.h - C ABI of the network glue around the rotation convolution: the ordinary
 * layers of the UNet-shaped stack the benchmark's training step is made of (paper Sec. V-A,
 * Fig. 9: ReLU, 2x2 max-pool, 2x2 stride-2 transposed-convolution up-sampling, skip
 * concatenation, 1x1 head, soft-max cross-entropy), each with its backward pass.
 *
 * Same conventions as rotconv.h: plain C; every tensor pointer is DEVICE memory owned by the
 * caller, dense row-major fp32 NCHW (labels int32, max-pool indices uint8); `stream` is a
 * hipStream_t passed as void*; calls only enqueue; outputs are overwritten unless said
 * otherwise; results are bitwise reproducible.  Return value: a rotconv_status
 * (ROTCONV_ERR_NULL, ROTCONV_ERR_SHAPE, ROTCONV_ERR_WORKSPACE, ROTCONV_ERR_LAUNCH).
 */
#ifndef UNETGLUE_H
#define UNETGLUE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* y = max(x, 0); n elements.  In place (y == x) is allowed. */
int glue_relu_fwd(const float* x, float* y, size_t n, void* stream);
/* dx = dy where y > 0 else 0 (y = the forward OUTPUT).  dx may alias dy. */
int glue_relu_bwd(const float* y, const float* dy, float* dx, size_t n, void* stream);

/* 2x2 max-pool, stride 2; H and W even.  x [N,C,H,W] -> y [N,C,H/2,W/2]; idx (uint8, same shape
 * as y) = 2*a + b of the winning element (first maximum in row-major order wins ties). */
int glue_maxpool2_fwd(const float* x, float* y, uint8_t* idx, int N, int C, int H, int W, void* stream);
/* dx [N,C,H,W]: dy goes to the winner of each window, zeros elsewhere.  accumulate != 0 adds the routed
 * gradient to what dx already holds (a skip connection's gradient) instead of overwriting it. */
int glue_maxpool2_bwd(const float* dy, const uint8_t* idx, float* dx, int N, int C, int H, int W, int accumulate,
                      void* stream);

/* 2x2 stride-2 transposed convolution, no bias: y[n,co,2h+a,2w+b] = sum_ci x[n,ci,h,w] * w[ci,co,a,b].
 * x [N,Cin,H,W], w [Cin,Cout,2,2], y / dy [N,Cout,2H,2W].  ws: scratch of
 * glue_upconv2_workspace_bytes() bytes (used by the weight gradient only). */
size_t glue_upconv2_workspace_bytes(int N, int Cin, int Cout, int H, int W);
int glue_upconv2_fwd(const float* x, const float* w, float* y, int N, int Cin, int Cout, int H, int W, void* stream);
int glue_upconv2_bwd_data(const float* dy, const float* w, float* dx, int N, int Cin, int Cout, int H, int W,
                          void* stream);
int glue_upconv2_bwd_weight(const float* x, const float* dy, float* dw, int N, int Cin, int Cout, int H, int W,
                            void* ws, size_t ws_bytes, void* stream);

/* out[n] = concat(a[n], b[n]) along channels: a [N,Ca,P], b [N,Cb,P], out [N,Ca+Cb,P] (P = H*W). */
int glue_concat2(const float* a, const float* b, float* out, int N, int Ca, int Cb, size_t P, void* stream);
/* The reverse for gradients: da (+)= dcat[:, :Ca], db = dcat[:, Ca:].  accumulate_a != 0 adds into da. */
int glue_split2(const float* dcat, float* da, float* db, int N, int Ca, int Cb, size_t P, int accumulate_a,
                void* stream);

/* 1x1 convolution, no bias: y[n,co,p] = sum_ci w[co,ci] * x[n,ci,p].  x [N,Cin,P], w [Cout,Cin]. */
size_t glue_conv1x1_workspace_bytes(int N, int Cin, int Cout, size_t P);
int glue_conv1x1_fwd(const float* x, const float* w, float* y, int N, int Cin, int Cout, size_t P, void* stream);
int glue_conv1x1_bwd_data(const float* dy, const float* w, float* dx, int N, int Cin, int Cout, size_t P,
                          void* stream);
int glue_conv1x1_bwd_weight(const float* x, const float* dy, float* dw, int N, int Cin, int Cout, size_t P, void* ws,
                            size_t ws_bytes, void* stream);

/* Mean soft-max cross-entropy over all N*P pixels.  logits [N,K,P], labels int32 [N,P] in 0..K-1.
 * loss: one float; dlogits [N,K,P] = (softmax - onehot) / (N*P).  ws: N*P floats.  A pixel whose label
 * lies outside 0..K-1 adds nothing to the loss and gets a zero gradient (the divisor stays N*P). */
int glue_softmax_ce(const float* logits, const int32_t* labels, float* loss, float* dlogits, int N, int K, size_t P,
                    void* ws, size_t ws_bytes, void* stream);

/* ---- bfloat16 twins ------------------------------------------------------------------------------
 * Same operations and argument meanings with activations, their gradients and the weights handed to
 * the forward / input-gradient calls stored as bfloat16 (uint16_t holding the upper half of the fp32
 * bit pattern): configuration "bf16 weights / activations, fp32 accumulation".  Every value is widened
 * exactly, all arithmetic and accumulation is fp32, and each bf16 output element is rounded once, to
 * nearest-even.  Weight gradients (dw) and the loss stay fp32; workspace sizes are those of the fp32
 * calls. */
int glue_relu_fwd_bf16(const uint16_t* x, uint16_t* y, size_t n, void* stream);
int glue_relu_bwd_bf16(const uint16_t* y, const uint16_t* dy, uint16_t* dx, size_t n, void* stream);
int glue_maxpool2_fwd_bf16(const uint16_t* x, uint16_t* y, uint8_t* idx, int N, int C, int H, int W, void* stream);
int glue_maxpool2_bwd_bf16(const uint16_t* dy, const uint8_t* idx, uint16_t* dx, int N, int C, int H, int W,
                           int accumulate, void* stream);
int glue_upconv2_fwd_bf16(const uint16_t* x, const uint16_t* w, uint16_t* y, int N, int Cin, int Cout, int H, int W,
                          void* stream);
int glue_upconv2_bwd_data_bf16(const uint16_t* dy, const uint16_t* w, uint16_t* dx, int N, int Cin, int Cout, int H,
                               int W, void* stream);
int glue_upconv2_bwd_weight_bf16(const uint16_t* x, const uint16_t* dy, float* dw, int N, int Cin, int Cout, int H,
                                 int W, void* ws, size_t ws_bytes, void* stream);
int glue_concat2_bf16(const uint16_t* a, const uint16_t* b, uint16_t* out, int N, int Ca, int Cb, size_t P,
                      void* stream);
int glue_split2_bf16(const uint16_t* dcat, uint16_t* da, uint16_t* db, int N, int Ca, int Cb, size_t P,
                     int accumulate_a, void* stream);
int glue_conv1x1_fwd_bf16(const uint16_t* x, const uint16_t* w, uint16_t* y, int N, int Cin, int Cout, size_t P,
                          void* stream);
int glue_conv1x1_bwd_data_bf16(const uint16_t* dy, const uint16_t* w, uint16_t* dx, int N, int Cin, int Cout, size_t P,
                               void* stream);
int glue_conv1x1_bwd_weight_bf16(const uint16_t* x, const uint16_t* dy, float* dw, int N, int Cin, int Cout, size_t P,
                                 void* ws, size_t ws_bytes, void* stream);
int glue_softmax_ce_bf16(const uint16_t* logits, const int32_t* labels, float* loss, uint16_t* dlogits, int N, int K,
                         size_t P, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* UNETGLUE_H */
