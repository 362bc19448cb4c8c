/*
 * rotconv.h - C ABI of the MI355X (gfx950) multi-orientation convolution library.
 *
 * One base filter bank is expanded to R orientations; every orientation is a
 * 2-D cross-correlation of the same input (paper Sec. III-B, Eq. 5 and 7), the
 * R responses of a filter are max-pooled over orientation groups with the
 * arg-max kept (Eq. 10), and the backward passes route the upstream gradient
 * through the arg-max (Eq. 12) into the input gradient (Eq. 13, 15) and the
 * base-weight gradient (Eq. 14, 16).  Point-wise average pooling over the
 * orientation groups (Eq. 9, gradient shared equally: Eq. 11) is the other
 * pooling the paper names; a plan selects it with pool_op.  Orientations whose angles differ by
 * multiples of 90 degrees share their per-tap channel contractions (Eq. 8);
 * other angles get one first-quadrant filter each plus its three quarter-turn
 * copies (Sec. III-D).
 *
 * Conventions common to every call
 *   - Plain C, no C++ types, no exceptions cross this boundary.
 *   - Pointers marked DEVICE point to memory of the current HIP device, owned by
 *     the caller; the library never allocates, frees or keeps them.  Pointers
 *     marked HOST are ordinary host memory.  The plan owns only its small
 *     tables (host copies, and device copies uploaded on first use).
 *   - All tensors are dense, contiguous, row-major, fp32 unless said otherwise:
 *       x      [N][Cin][H][W]
 *       w      [B][Cout][Cin][k][k]   B = 2 (f_x then f_y, Eq. 17) in STEERABLE mode, else 1
 *       y, dy  [N][Cout*R][Ho][Wo]    channel = co*R + r
 *       ypool, gpool [N][Cout*(R/G)][Ho][Wo]  channel = co*(R/G) + g
 *       idx    same shape as ypool, uint8: the orientation index r (0..R-1) that won
 *       dw     [B][Cout][Cin][k][k]   fp32
 *     Ho = (H + 2*pad - k)/stride + 1, likewise Wo.
 *   - Orientation r has angle theta_r (degrees, counter-clockwise when row 0 is
 *     drawn on top).  theta_r = 90*s_r + phi_r, phi_r in [0,90): its filter is
 *     the first-quadrant filter F_phi_r turned by s_r exact quarter turns,
 *     rot90(A)[i][j] = A[j][k-1-i].
 *   - Pool group g of a filter holds the orientations r with r mod (R/G) == g
 *     (for evenly spaced angles and G = 4: the four symmetric rotations of one
 *     first-quadrant angle, Sec. V-A).  Ties: the smallest r wins.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     only enqueue work; nothing synchronises with the host.  Outputs are
 *     overwritten, never accumulated into.  Same inputs give bitwise the same
 *     outputs on every run (no floating-point atomics anywhere).  A plan's first
 *     call on a device uploads its tables (the only allocation and host-to-device
 *     copy the library makes); every later call launches kernels only, so it can
 *     be recorded into a HIP graph and replayed.
 *   - Kernel choices are made when a plan is created, from the descriptor and the
 *     optional rotconv_plan_options (below); the process environment is never read.
 *   - Host threads: a plan is immutable except for the table upload of its first
 *     call on a device, and is bound to that device afterwards (a call on another
 *     device returns ROTCONV_ERR_UNSUPPORTED).  Make that first call from one
 *     thread; later calls may come from any thread, each with its own workspace.
 *   - `ws` is a DEVICE scratch buffer of at least rotconv_workspace_bytes(plan)
 *     bytes, 256-byte aligned; its contents are undefined between calls, and
 *     two calls sharing one ws must not overlap in time.
 *   - Return value: a rotconv_status.  Argument errors are found on the host
 *     before anything is launched and leave the outputs untouched.
 */
#ifndef ROTCONV_H
#define ROTCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ROTCONV_OK = 0,
  ROTCONV_ERR_NULL = -1,        /* a required pointer is NULL                                  */
  ROTCONV_ERR_SHAPE = -2,       /* a size is < 1, the output would be empty, G does not divide R */
  ROTCONV_ERR_ANGLES = -3,      /* angles not ascending in [0,360), or not multiples of 90 in EXACT90 */
  ROTCONV_ERR_UNSUPPORTED = -4, /* valid request this build has no kernel for                  */
  ROTCONV_ERR_WORKSPACE = -5,   /* ws is NULL or ws_bytes too small                            */
  ROTCONV_ERR_LAUNCH = -6       /* the HIP runtime reported an error                           */
} rotconv_status;

typedef enum { ROTCONV_F32 = 0, ROTCONV_BF16 = 1 } rotconv_dtype;
typedef enum { ROTCONV_EXACT90 = 0, ROTCONV_STEERABLE = 1, ROTCONV_BILINEAR = 2, ROTCONV_P4M = 3 } rotconv_mode;
typedef enum { ROTCONV_POOL_MAX = 0, ROTCONV_POOL_AVG = 1 } rotconv_pool_op;
typedef enum { ROTCONV_ACT_NONE = 0, ROTCONV_ACT_RELU = 1 } rotconv_activation;

/* Problem statement of Sec. III (input C_in x H x W, filters C_out x C_in x K x K),
 * with a batch dimension, an orientation set, stride and zero padding. */
typedef struct {
  int32_t N, Cin, H, W;
  int32_t Cout, k;          /* square kernels only: quarter turns need them            */
  int32_t R;                /* number of orientations, 1..255; Cout * R, Cin and N at most 65535 each
                               (ROTCONV_ERR_UNSUPPORTED beyond)                         */
  const double* angles_deg; /* HOST, R strictly ascending angles in [0,360); NULL means
                               r*360/R (evenly spaced, Sec. III-D).  Copied by plan_create. */
  int32_t mode;             /* rotconv_mode: how first-quadrant filters are built.
                               EXACT90: angles must be multiples of 90 (Eq. 5).
                               STEERABLE: F_phi = sin(phi) f_x + cos(phi) f_y (Eq. 17).
                               BILINEAR: F_phi = base filter resampled bilinearly about the
                               tap-grid centre, zero outside the k x k support (not the
                               paper's rule; the benchmark configurations ask for it).
                               P4M: rotations and reflection (the p4m group of Sec. II /
                               Sec. III-B): R is even, angles_deg must be NULL; orientation
                               r < R/2 is the base filter turned by r*360/(R/2) degrees
                               (multiples of 90, so R is 2, 4 or 8), orientation R/2 + a is
                               the left-right mirrored base filter, M[i][j] = W[i][k-1-j],
                               turned by the same angle a*360/(R/2). */
  int32_t stride, pad;      /* stride >= 1, pad >= 0.  3x3 / stride 1 / pad 1 layers run on the matrix
                               cores whatever N, Cin, Cout, H, W are (row widths the kernels do not take
                               directly are staged in the workspace on zero-padded rows, same result);
                               other k, stride, pad run slower general kernels. */
  int32_t pool_group;       /* G, must divide R; 0 means R (one pooled map per filter) */
  int32_t dtype;            /* rotconv_dtype of x, w, y, ypool, gpool, dy, dx.
                               ROTCONV_BF16: those tensors hold bfloat16; products are
                               accumulated in fp32, the arg-max is taken on the fp32
                               values before y / ypool are rounded (nearest even) to
                               bf16; dw stays fp32; idx stays uint8.  The rotated banks a
                               bf16 plan multiplies with are bf16 too (the first-quadrant
                               combination is formed in fp64 from fp64 coefficients and
                               rounded to fp32, then to bf16, nearest even).  3x3 /
                               stride 1 / pad 1 layers run on the bf16 matrix cores; other
                               shapes are widened to fp32 in the workspace and run the
                               fp32 kernels. */
  int32_t pool_op;          /* rotconv_pool_op.  ROTCONV_POOL_MAX (0): Eq. 10 / Eq. 12.
                               ROTCONV_POOL_AVG: ypool = mean over the pool group (Eq. 9),
                               every member receives gpool / G (Eq. 11); `idx` arguments are
                               ignored and may be NULL.  bf16 plans: the fused calls run on fp32 copies
                               in the workspace (the rotated banks rounded to bf16 first, as for every bf16
                               plan), results rounded once. */
  int32_t activation;       /* rotconv_activation, applied by rotconv_pool_fwd only (max-pooling plans).
                               ROTCONV_ACT_RELU: ypool = max(pooled value, 0), and idx = 255 (no
                               orientation) wherever the pooled value is not positive.  Because an idx
                               outside its pool group routes nothing (Eq. 12), rotconv_pool_bwd_data and
                               rotconv_pool_bwd_weight fed that idx and the gradient of the ReLU OUTPUT
                               return the gradients through ReLU, pooling and convolution: the block
                               "rotation convolution + ReLU" of Sec. V-A without a pass of its own. */
} rotconv_desc;

typedef struct rotconv_plan rotconv_plan; /* opaque */

/* Tuning switches of a plan's kernel choice (results are the same for every setting, up to summation order).
 * All zero = automatic, which is what rotconv_plan_create uses. */
typedef struct {
  int32_t fwd_csplit;   /* channel split of the 3x3 forward on small maps with deep inputs: 0 automatic,
                           1 never (where an unsplit kernel exists), n >= 2: n parts                        */
  int32_t gs;           /* shapes outside the 3x3 / stride 1 / pad 1 kernels on the matrix multiply + scatter
                           family: 0 automatic (from about a megaflop), 1 always, -1 never (generic kernels)   */
  int32_t gs_chunk_mb;  /* MiB of products that family keeps in the workspace at once: 0 = 512, n > 0 = n,
                           -1 = one image at a time (at least one image's worth is always taken)               */
  int32_t bwd_lut;      /* fp32 gradients of layers whose pool group spans several first-quadrant banks:
                           0 automatic (routed gradients folded into the base taps, one contraction),
                           -1 never (one contraction per bank)                                                 */
  int32_t fwd_base;     /* fp32 forward of such layers: 0 automatic (products of the base bank only, combined
                           into the banks' products on the vector ALU), -1 never (one contraction per bank)    */
  int32_t direct;       /* layers with at most four input channels (a network's first layer): 0 automatic (the
                           pooled forward on the vector-ALU kernel, no matrix instructions), -1 never             */
  int32_t direct_ty;    /* rows per band of that kernel: 0 automatic, n > 0 = n                                   */
  int32_t px_fwd;       /* bf16 pooled forward of layers with 8 to 128 input channels pooled over all orientations:
                           0 automatic (filters on the matrix instruction's M side, a lane per pixel column, for
                           layers with four banks and at most 64 input channels), 1 wherever that kernel can run,
                           -1 never (pixels on the M side, eight pixels per lane)                                   */
  int32_t reserved[4];  /* must be 0 */
} rotconv_plan_options;

/* Validates the descriptor, builds the orientation tables on the host and
 * returns a plan.  Touches no GPU.  `*out` is set only on ROTCONV_OK. */
int rotconv_plan_create(const rotconv_desc* desc, rotconv_plan** out);
/* The same with tuning switches; `opts` HOST, copied, NULL = all automatic.  ROTCONV_ERR_UNSUPPORTED for a
 * non-zero reserved field. */
int rotconv_plan_create_opt(const rotconv_desc* desc, const rotconv_plan_options* opts, rotconv_plan** out);
/* Frees the plan and its device tables (if any were uploaded). NULL is allowed. */
int rotconv_plan_destroy(rotconv_plan* plan);

/* Bytes of scratch the largest call on this plan needs (may be 0). */
size_t rotconv_workspace_bytes(const rotconv_plan* plan);
/* Bytes of scratch with which rotconv_bwd_data and rotconv_bwd_weight (the unfused gradient calls, dense dy) run on
 * the matrix cores as well: the routed products of a few images at a time, k*k*Q*Cout*H*W floats per image.  With the
 * smaller rotconv_workspace_bytes they run slower general kernels (same result); never less than that value. */
size_t rotconv_workspace_bytes_unfused(const rotconv_plan* plan);
/* Output extents; any pointer may be NULL. Cunpooled = Cout*R, Cpooled = Cout*R/G. */
int rotconv_out_shape(const rotconv_plan* plan, int32_t* Ho, int32_t* Wo, int32_t* Cunpooled, int32_t* Cpooled);

/* Host-side views of the plan's tables (for inspection and tests; no GPU).
 * rotconv_plan_orientations: Q = number of distinct first-quadrant angles;
 *   bank_of_r[r] in 0..Q-1 and quarter_of_r[r] in 0..3 (HOST arrays of R ints, may be NULL).
 * rotconv_plan_expansion: the linear map base bank(s) -> rotated banks of one
 *   (co,ci) slice, dense, HOST array E[R][k*k][B][k*k] of floats:
 *   W^(r)[t] = sum_{b,u} E[r][t][b][u] * w[b][u]   (Eq. 5 / Sec. III-D / Eq. 17). */
int rotconv_plan_orientations(const rotconv_plan* plan, int32_t* Q, int32_t* bank_of_r, int32_t* quarter_of_r);
int rotconv_plan_expansion(const rotconv_plan* plan, float* E);
/* The routed-gradient table of 3x3 plans with one base bank (B = 1), HOST array T[9][R + 1][9] of floats: with
 * Delta_r = G [idx == r] (Eq. 12), the gradient that reaches base tap u of a filter at pixel p (the D of
 * dX = sum_co,u w[co,ci,u] D[u], dw[co,ci,u] = sum_p D[u][p] x[ci,p]; Eq. 13-16 with the expansion folded in) is
 * D[u][p] = sum over dy, dx in {-1,0,1} of G[p + (dy,dx)] * T[(dy+1)*3 + (dx+1)][idx[p + (dy,dx)]][u]; row R (no
 * orientation) is zero.  ROTCONV_ERR_UNSUPPORTED for other plans. */
int rotconv_plan_routed_table(const rotconv_plan* plan, float* T);

/* ---- the five calls of the unfused chain ------------------------------------- */

/* Eq. 7: y[n,co*R+r] = W^(r) (cross-correlated with) x.  x, w, y DEVICE. */
int rotconv_fwd(const rotconv_plan* plan, const void* x, const void* w, void* y, void* ws, size_t ws_bytes,
                void* stream);
/* Eq. 13 + 15: dx = sum_r (transposed correlation of dy_r with W^(r)).  dy, w, dx DEVICE. */
int rotconv_bwd_data(const rotconv_plan* plan, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes,
                     void* stream);
/* Eq. 14 + 16: dw = sum_r expansion^T( correlation of x with dy_r ), summed over the batch.
 * x, dy, dw DEVICE; dw is fp32. */
int rotconv_bwd_weight(const rotconv_plan* plan, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes,
                       void* stream);
/* Eq. 10 over pool groups, with arg-max (ROTCONV_POOL_AVG plans: Eq. 9, the mean; idx untouched).
 * y, ypool, idx DEVICE. */
int orient_maxpool_fwd(const rotconv_plan* plan, const void* y, void* ypool, uint8_t* idx, void* stream);
/* Eq. 12: dy[n,co*R+r] = gpool[n,co*(R/G)+g] if idx == r else 0.  gpool, idx, dy DEVICE.
 * idx values that are not members of their pool group give zeros.
 * ROTCONV_POOL_AVG plans: Eq. 11, dy[n,co*R+r] = gpool[n,co*(R/G)+g] / G. */
int orient_maxpool_bwd(const rotconv_plan* plan, const void* gpool, const uint8_t* idx, void* dy, void* stream);

/* ---- the fused hot path: the R-fold tensors y / dy are never materialised ------ */

/* Eq. 8 + Eq. 10 in one pass: the input tile is read once and shared by all rotated copies.
 * ROTCONV_POOL_AVG plans: the mean over a pool group is linear in the bank, so the three fused calls
 * run ONE ordinary convolution with the group-averaged bank (1/G) sum_r W^(r) (and its adjoints). */
int rotconv_pool_fwd(const rotconv_plan* plan, const void* x, const void* w, void* ypool, uint8_t* idx, void* ws,
                     size_t ws_bytes, void* stream);
/* rotconv_pool_fwd for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels as
 * rotconv_pool_fwd, but the scratch (the re-laid banks and, for some plans, per-bank candidates or channel-split
 * parts) lives in a file-scope device array of ROTCONV_STATIC_SCRATCH_BYTES that each GPU the library runs on
 * holds until the process ends.  The call makes no hipMalloc / hipFree and uploads nothing:
 *   - ROTCONV_ERR_UNSUPPORTED if the plan's tables are not on the current device yet (run any ordinary call
 *     of the plan there first; that first call is the one that allocates);
 *   - ROTCONV_ERR_WORKSPACE if this call's scratch need exceeds ROTCONV_STATIC_SCRATCH_BYTES (e.g. layers deeper
 *     than about 512 x 512 channels at R = 4, plans that stage padded rows or widened copies of large tensors);
 *   - the first call on a device resolves the array's device address (no allocation; make it outside a capture).
 * All calls on one GPU share that GPU's array, which keeps the last call's contents; every region a call reads
 * it has written first, so nothing needs clearing.  Two calls that overlap in time on one GPU (two streams, two
 * host threads) race on it: serialise them. */
#define ROTCONV_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
int rotconv_pool_fwd_static(const rotconv_plan* plan, const void* x, const void* w, void* ypool, uint8_t* idx,
                            void* stream);
/* Eq. 12 + Eq. 13 + Eq. 15. */
int rotconv_pool_bwd_data(const rotconv_plan* plan, const void* gpool, const uint8_t* idx, const void* w, void* dx,
                          void* ws, size_t ws_bytes, void* stream);
/* Eq. 12 + Eq. 14 + Eq. 16. */
int rotconv_pool_bwd_weight(const rotconv_plan* plan, const void* x, const void* gpool, const uint8_t* idx, float* dw,
                            void* ws, size_t ws_bytes, void* stream);

/* ---- regularisers of the steerable pair (Sec. III-D, Eq. 18-20) ------------------------------------
 * w DEVICE fp32 [2][Cout][per]: the two base banks f_x then f_y of a STEERABLE layer, per = Cin*k*k; "filter b"
 * of Eq. 19 / Eq. 20 is output filter b flattened over (Cin, k, k) (B = Cout).
 *   L_mag  = 1/B sum_b (||wx_b|| - ||wy_b||)^2                               (Eq. 19)
 *   L_orth = 1/B sum_b ( <wx_b, wy_b> / (||wx_b|| ||wy_b|| + eps) )^2       (Eq. 20)
 * losses DEVICE fp32 [2] receives (L_mag, L_orth).  dw DEVICE fp32 [2][Cout][per] (may be NULL) receives
 * lambda_mag dL_mag/dw + lambda_orth dL_orth/dw, the regularisers' share of Eq. 18's gradient; accumulate != 0
 * adds it to what dw holds (the layer's dw from rotconv_pool_bwd_weight) instead of overwriting.  A filter of
 * zero norm gets a zero gradient for the terms that divide by that norm.  ws: Cout * 2 floats.  Fixed
 * reduction order: bitwise reproducible. */
int rotconv_steerable_reg(const float* w, int32_t Cout, int32_t per, float lambda_mag, float lambda_orth, float eps,
                          float* losses, float* dw, int32_t accumulate, void* ws, size_t ws_bytes, void* stream);

/* ---- measuring kernels (for the benchmark's measured-peak figures; not on the hot path) ------------------
 * rotconv_diag_mfma: 2048 workgroups of four waves, each wave n_iter rounds of eight independent matrix
 *   instructions on registers only (dtype ROTCONV_F32: 16x16x4 fp32; ROTCONV_BF16: 16x16x32 bf16 with fp32
 *   accumulation).  sink DEVICE, rotconv_diag_mfma_sink_bytes() bytes, receives one float per lane.  *flops (HOST,
 *   may be NULL) receives the floating-point operations the launch executes; time it with events on `stream`.
 * rotconv_diag_copy: dst[i] = src[i] for bytes / 16 float4 elements (dst, src DEVICE, 16-byte aligned, bytes a
 *   multiple of 16): 2 * bytes of HBM traffic. */
size_t rotconv_diag_mfma_sink_bytes(void);
int rotconv_diag_mfma(int dtype, int n_iter, float* sink, void* stream, double* flops);
int rotconv_diag_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Static, never NULL. */
const char* rotconv_status_string(int status);
/* Matrix work a fused call executes, in conv-equivalents (one conv-equivalent = N*Ho*Wo*Cin*Cout*k*k multiply-adds,
 * an ordinary convolution of the layer's shape): pass 0 rotconv_pool_fwd, 1 rotconv_pool_bwd_data, 2
 * rotconv_pool_bwd_weight.  The method's count (Eq. 8) is Q, the number of first-quadrant banks; kernels that fold
 * the banks into the base bank execute fewer (1 per base bank), kernels that multiply every quarter turn on its own
 * execute more (up to R); the structured-sparse bf16 instances count at the dense rate they issue at (R / 2).
 * For reporting (the benchmark's executed-work roofline). */
double rotconv_plan_conv_equivalents(const rotconv_plan* plan, int pass);
/* Name of the kernel family a call of the given kind on this plan uses ("generic", "mfma_p4", "mfma_p4_base" (the
 * pooled forward on products of the base bank), "mfma_p4_bf16", "mfma_p4_bf16_lut" (a bf16 gradient whose routed
 * gradients are folded into the base taps in fp32 and rounded to bf16 once, the matrix operand), "mfma_gemm_scatter",
 * "valu_direct" (layers with at most four input channels: vector ALU only), "mfma_px_bf16" (the bf16 pooled forward with
 * a lane per pixel column)).  pass: 0 / 1 / 2 = the fused calls rotconv_pool_fwd / _bwd_data / _bwd_weight (and
 * rotconv_fwd); 3 / 4 = the unfused gradient calls rotconv_bwd_data / rotconv_bwd_weight when given
 * rotconv_workspace_bytes_unfused of scratch (with less they run "generic"). */
const char* rotconv_plan_kernel_name(const rotconv_plan* plan, int pass);

#ifdef __cplusplus
}
#endif
#endif /* ROTCONV_H */
