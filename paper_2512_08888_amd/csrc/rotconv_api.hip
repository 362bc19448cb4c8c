// extern "C" entry points of the rotation-convolution library (see include/rotconv.h).
// This layer checks arguments, uploads the plan's tables on first use, picks the
// kernel family and enqueues; it never synchronises with the host.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstring>

#include "rotconv_kernels.h"
#include "rotconv_bf16.h"
#include "rotconv_p4.h"
#include "rotconv_gs.h"
#include "rotconv_direct.h"
#include "rotconv_px_fwd_bf16.h"

namespace rotconv {

namespace {

template <typename T>
bool upload(const std::vector<T>& h, T** d) {
  const size_t bytes = std::max<size_t>(h.size(), 1) * sizeof(T);
  if (hipMalloc(reinterpret_cast<void**>(d), bytes) != hipSuccess) return false;
  if (!h.empty() && hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return false;
  return true;
}

}  // namespace

int ensure_device_tables(rotconv_plan* p) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return ROTCONV_ERR_LAUNCH;
  if (p->dev.device == dev) return ROTCONV_OK;
  if (p->dev.device >= 0) return ROTCONV_ERR_UNSUPPORTED;  // a plan is bound to the first device it ran on
  const HostTables& t = p->host;
  DeviceTables& d = p->dev;
  std::vector<int32_t> rq(p->d.R);
  for (int r = 0; r < p->d.R; ++r) rq[r] = t.bank_of_r[r] * 4 + t.quarter_of_r[r];
  const bool bf = p->d.dtype == ROTCONV_BF16;      // only bf16 plans read the fp64 coefficients
  const std::vector<double> none64;
  const bool ok = upload(t.exp_src, &d.exp_src) && upload(t.exp_coef, &d.exp_coef) && upload(t.tr_ptr, &d.tr_ptr) &&
                  upload(t.tr_col, &d.tr_col) && upload(t.tr_coef, &d.tr_coef) && upload(t.fq_src, &d.fq_src) &&
                  upload(t.fq_coef, &d.fq_coef) && upload(t.fqt_ptr, &d.fqt_ptr) && upload(t.fqt_col, &d.fqt_col) &&
                  upload(t.fqt_coef, &d.fqt_coef) && upload(p->rot_of, &d.rot_of) && upload(rq, &d.rq_of_r) &&
                  upload(t.turn_tap, &d.turn_tap) && upload(t.lut_bwd, &d.lut_bwd) &&
                  upload(bf ? t.exp_coef64 : none64, &d.exp_coef64) && upload(bf ? t.fq_coef64 : none64, &d.fq_coef64) &&
                  upload(t.fwd_base_coef, &d.fwd_base_coef) && upload(bf ? t.fq_dense64 : none64, &d.fq_dense64);
  if (!ok) {
    (void)hipGetLastError();
    free_device_tables(p);
    return ROTCONV_ERR_LAUNCH;
  }
  d.device = dev;
  // the plans this one runs some passes through: their tables go up with the parent's, so that no pass of the
  // parent allocates after the parent's first call
  for (rotconv_plan* ch : {p->avg_child, p->pad_child})
    if (ch) {
      const int rc = ensure_device_tables(ch);
      if (rc != ROTCONV_OK) return rc;
    }
  return ROTCONV_OK;
}

void free_device_tables(rotconv_plan* p) {
  DeviceTables& d = p->dev;
  void* ptrs[] = {d.exp_src, d.exp_coef, d.tr_ptr, d.tr_col, d.tr_coef, d.fq_src,
                  d.fq_coef, d.fqt_ptr, d.fqt_col, d.fqt_coef, d.rot_of, d.rq_of_r, d.turn_tap, d.lut_bwd,
                  d.exp_coef64, d.fq_coef64, d.fwd_base_coef, d.fq_dense64};
  for (void* q : ptrs)
    if (q) (void)hipFree(q);
  d = DeviceTables();
}

// Are the plan's tables (and those of the plans it runs passes through) on the current device already?
bool tables_on_current_device(const rotconv_plan* p) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || p->dev.device != dev) return false;
  for (const rotconv_plan* ch : {p->avg_child, p->pad_child})
    if (ch && !tables_on_current_device(ch)) return false;
  return true;
}

namespace {

int finish() { return hipGetLastError() == hipSuccess ? ROTCONV_OK : ROTCONV_ERR_LAUNCH; }

size_t align256(size_t v) { return (v + 255) / 256 * 256; }

bool aligned(const void* p, size_t a) { return reinterpret_cast<uintptr_t>(p) % a == 0; }

// Bytes reserved for the packed banks of the fast forward (the larger of the fp32 and, for bf16 plans, the bf16 image).
size_t fwd_pack_region(const rotconv_plan* p) {
  size_t b = p4_fwd_pack_floats(p) * sizeof(float);
  if (p->d.dtype == ROTCONV_BF16) b = std::max(b, p4_fwd_bf16_pack_bytes(p));
  return align256(b);
}

// Scratch of the fast forward: packed banks, then per-bank candidates or the unpooled map.
size_t fwd_fast_ws_bytes(const rotconv_plan* p) {
  const size_t pack = fwd_pack_region(p);
  const size_t hw = (size_t)p->d.H * p->d.W;
  const int mode = p4_fwd_pool_mode(p);
  size_t extra = 0;
  if (mode == kOutPartial) extra = align256((size_t)p->host.Q * p->d.N * p->d.Cout * hw * 4) +
                                   align256((size_t)p->host.Q * p->d.N * p->d.Cout * hw);
  if (mode == kOutUnpooled) extra = align256((size_t)p->d.N * p->d.Cout * p->d.R * hw * 4);
  // channel split: one unpooled part per split
  const int cs = std::max(p->fwd_csplit[0], p->fwd_csplit[1]);
  if (cs > 1) extra = std::max(extra, align256((size_t)cs * p->d.N * p->d.Cout * p->d.R * hw * 4));
  return pack + extra;
}

// the fp32 path's own need (a bf16 plan adds its staging areas in front, see carve())
int check_ws_inner(const rotconv_plan* p, const void* ws, size_t ws_bytes) {
  if (p->ws_inner == 0) return ROTCONV_OK;
  if (!ws || ws_bytes < p->ws_inner) return ROTCONV_ERR_WORKSPACE;
  return ROTCONV_OK;
}

// Scratch of an average-pooling plan: rotated banks, the group-averaged bank (or its gradient), an all-zero idx
// map for the R = 1 plan's fused gradient calls, then that plan's own scratch.
struct AvgLayout { size_t wexp, wavg, idx0, child, total; };
AvgLayout avg_layout(const rotconv_plan* p) {
  AvgLayout L;
  const size_t bank = (size_t)p->d.Cout * p->d.Cin * p->kk * sizeof(float);
  L.wexp = 0;
  L.wavg = align256((size_t)p->d.R * bank);
  L.idx0 = L.wavg + align256((size_t)p->ng * bank);
  L.child = L.idx0 + align256(p->n_yp);
  L.total = L.child + align256(p->avg_child ? p->avg_child->ws_bytes : 0);
  return L;
}

// Staging areas of a plan whose calls run on zero-padded rows (pad_child): an input-sized area, an output-sized area
// (pooled; unpooled if rotconv_fwd goes that way too), the idx map, then the child's own scratch.
struct PadLayout { size_t in, out, idx, child, total; };
PadLayout pad_layout(const rotconv_plan* p) {
  const rotconv_plan* ch = p->pad_child;
  const size_t es = p->d.dtype == ROTCONV_BF16 ? 2 : 4;
  PadLayout L;
  L.in = 0;
  L.out = align256(ch->n_x * es);
  L.idx = L.out + align256((p->pad_use[0] ? ch->n_yu : ch->n_yp) * es);
  L.child = L.idx + align256(ch->n_yp);
  L.total = L.child + align256(ch->ws_bytes);
  return L;
}

// Scratch with which the unfused gradient calls (dense dy) of an fp32 plan leave the generic kernels for the matrix
// multiply + scatter family; equals the plan's own need where that family is used anyway or does not apply.
size_t unfused_ws_inner(const rotconv_plan* p) {
  if (p->gs || p->d.pool_op == ROTCONV_POOL_AVG || !gs_wanted(p)) return p->ws_inner;
  return std::max(p->ws_inner, align256(gs_ws_bytes(p)));
}

// Do the unfused gradient calls (dense dy) run matrix multiply + scatter with this much scratch?  Plans whose fused
// calls run that family anyway: always; plans on the register-resident kernels: when the family is wanted for the
// layer and the caller brought rotconv_workspace_bytes_unfused.
bool unfused_on_gs(const rotconv_plan* p, const void* ws, size_t ws_bytes) {
  if (p->gs) return true;
  if (p->d.pool_op == ROTCONV_POOL_AVG || !gs_wanted(p)) return false;
  return ws && ws_bytes >= unfused_ws_inner(p);
}

// how a pass runs: 2 bf16 matrix-core kernel, 1 fp32 matrix-core kernel, 0 generic
int pass_level(const rotconv_plan* p, int pass) {
  if (p->direct[pass] || (pass == 0 && p->px16)) return 2;
  if (p->d.dtype == ROTCONV_BF16 && p->native16[pass]) return 2;
  return p->fast[pass] ? 1 : 0;
}

}  // namespace
}  // namespace rotconv

using namespace rotconv;

extern "C" {

int rotconv_plan_create(const rotconv_desc* desc, rotconv_plan** out) {
  return rotconv_plan_create_opt(desc, nullptr, out);
}

int rotconv_plan_create_opt(const rotconv_desc* desc, const rotconv_plan_options* opts, rotconv_plan** out) {
  if (!desc || !out) return ROTCONV_ERR_NULL;
  if (opts && (opts->reserved[0] || opts->reserved[1] || opts->reserved[2] || opts->reserved[3])) return ROTCONV_ERR_UNSUPPORTED;
  rotconv_plan* p = nullptr;
  const int rc = validate_and_build(desc, &p);
  if (rc != ROTCONV_OK) return rc;
  if (opts) p->opt = *opts;
  p->bwdw_splits = generic_bwdw_splits(p);
  p->ws_bytes = generic_ws_bytes(p);
  p->fast[0] = p4_fwd_supported(p) ? 1 : 0;
  if (p->fast[0]) {
    p->fwd_csplit[0] = p4_fwd_csplit(p, false);
    p->fwd_csplit[1] = p4_fwd_csplit(p, true);
  }
  if (p->fast[0]) p->ws_bytes = std::max(p->ws_bytes, fwd_fast_ws_bytes(p));
  // one pool group over several banks: products of the base bank only.  Maps below 32 x 32 pixels with deep inputs
  // keep the channel split of the per-bank kernel where its cost model chose one (few workgroups either way).
  if (p->fast[0] && p4_fwd_base_supported(p) && (p->fwd_csplit[1] == 1 || (long)p->d.H * p->d.W >= 1024)) {
    p->fwd_base = 1;
    p->fwd_csplit[1] = 1;
    p->fwd_base_cls = p4_fwd_base_classify(p, &p->host.fwd_base_coef);
  }
  if (direct_fwd_supported(p)) {     // first layers: the pooled forward on the vector ALU
    p->direct[0] = 1;
    p->ws_bytes = std::max(p->ws_bytes, direct_fwd_pack_floats(p) * sizeof(float));
  }
  if (!p->direct[0] && px_fwd_bf16_supported(p)) {     // bf16, shallow layers: a lane per pixel column
    p->px16 = 1;
    p->ws_bytes = std::max(p->ws_bytes, px_fwd_bf16_pack_bytes(p));
  }
  if (direct_bwd_weight_supported(p)) {     // ... and, with a single bank, the weight gradient
    p->direct[2] = 1;
    p->ws_bytes = std::max(p->ws_bytes, direct_bwd_weight_ws_floats(p) * sizeof(float));
  }
  p->bwd_lut = p4_bwd_lut_choice(p) ? 1 : 0;
  p->fast[1] = p4_bwd_data_supported(p) ? 1 : 0;
  if (p->fast[1])
    p->ws_bytes = std::max(p->ws_bytes, align256(p4_bwd_data_pack_floats(p) * sizeof(float)) +
                                            p4_bwd_data_part_floats(p) * sizeof(float));
  p->fast[2] = p4_bwd_weight_supported(p) ? 1 : 0;
  if (p->fast[2]) p->ws_bytes = std::max(p->ws_bytes, p4_bwd_weight_ws_floats(p) * sizeof(float));
  if (p->d.dtype == ROTCONV_BF16) {     // scratch of the kernels that take bf16 tensors directly
    if (p->fast[0] && p4_fwd_bf16_supported(p)) p->ws_bytes = std::max(p->ws_bytes, p4_fwd_bf16_pack_bytes(p));
    if (p->fast[1] && p4_bwd_data_bf16_supported(p))
      p->ws_bytes = std::max(p->ws_bytes, align256(p4_bwd_data_bf16_pack_bytes(p)) + p4_bwd_data_bf16_part_bytes(p));
    if (p->fast[1] && p4_bwd_data_bf16_lut_supported(p))
      p->ws_bytes = std::max(p->ws_bytes, align256(p4_bwd_data_bf16_lut_pack_bytes(p)) + p4_bwd_data_bf16_lut_part_bytes(p));
  }
  // other layers (k, stride, pad, or a pool group that cuts through a bank): matrix multiply + scatter
  const bool is3x3 = p->d.k == 3 && p->d.stride == 1 && p->d.pad == 1;
  if (!(p->fast[0] && p->fast[1] && p->fast[2]) && !(is3x3 && p4_fwd_pool_mode(p) != kOutUnpooled) && gs_wanted(p)) {
    p->gs = 1;
    p->gs_chunk_bytes = gs_chunk_budget(p);
    p->ws_bytes = std::max(p->ws_bytes, gs_ws_bytes(p));
  }
  p->ws_inner = p->ws_bytes = align256(p->ws_bytes);
  const size_t hw_in = (size_t)p->d.H * p->d.W, hw_out = (size_t)p->Ho * p->Wo;
  p->n_x = (size_t)p->d.N * p->d.Cin * hw_in;
  p->n_w = (size_t)p->B * p->d.Cout * p->d.Cin * p->kk;
  p->n_yp = (size_t)p->d.N * p->d.Cout * p->ng * hw_out;
  p->n_yu = (size_t)p->d.N * p->d.Cout * p->d.R * hw_out;
  if (p->d.dtype == ROTCONV_BF16) {
    p->ws_bytes = align256(p->n_x * 4) + align256(p->n_w * 4) + align256(p->n_yu * 4) + p->ws_inner;
    p->native16[0] = p->fast[0] && p4_fwd_bf16_supported(p) ? 1 : 0;
    p->native16[1] = p->fast[1] && p4_bwd_data_bf16_supported(p) ? 1 : 0;
    if (p->fast[1] && p4_bwd_data_bf16_lut_supported(p)) p->native16[1] = p->bwd_lut16[1] = 1;
    p->native16[2] = p->fast[2] && p4_bwd_weight_bf16_supported(p) ? 1 : 0;
    if (p->native16[2] && p4_bwd_lut16_choice(p)) p->bwd_lut16[2] = 1;
  }
  if (p->d.pool_op == ROTCONV_POOL_AVG) {
    // the fused calls of an average-pooling plan run an ordinary convolution (R = 1) with Cout * R/G filters
    rotconv_desc cd = p->d;
    cd.Cout = p->d.Cout * p->ng; cd.R = 1; cd.angles_deg = nullptr; cd.mode = ROTCONV_EXACT90; cd.pool_group = 0;
    cd.pool_op = ROTCONV_POOL_MAX;
    cd.dtype = ROTCONV_F32;       // a bf16 plan runs it on widened copies
    const int crc = rotconv_plan_create_opt(&cd, &p->opt, &p->avg_child);
    if (crc != ROTCONV_OK) {
      delete p;
      return crc;
    }
    const AvgLayout L = avg_layout(p);
    const size_t staging = p->ws_bytes - p->ws_inner;       // a bf16 plan's fp32 copies in front (0 for fp32 plans)
    p->ws_inner = std::max(p->ws_inner, L.total);
    p->ws_bytes = staging + p->ws_inner;
    p->native16[0] = p->native16[1] = p->native16[2] = 0;   // the fused calls go through the averaged bank in fp32
  }
  // 3x3 / stride 1 / pad 1 layers whose row width keeps a pass off the matrix-core kernels: the same layer on rows
  // padded to a multiple of 8 (32 beyond 256 pixels)
  if (p->d.pool_op != ROTCONV_POOL_AVG && p->d.k == 3 && p->d.stride == 1 && p->d.pad == 1) {
    const int top = p->d.dtype == ROTCONV_BF16 ? 2 : 1;
    const int Wp = p->d.W > 256 ? (p->d.W + 31) / 32 * 32 : (p->d.W + 7) / 8 * 8;
    const bool lacking = pass_level(p, 0) < top || pass_level(p, 1) < top || pass_level(p, 2) < top;
    if (lacking && Wp != p->d.W) {
      rotconv_desc cd = p->d;       // angles_deg points at the plan's own list (the defaults where none were given)
      cd.W = Wp;
      if (cd.mode == ROTCONV_P4M) cd.angles_deg = nullptr;   // that mode takes no explicit angles
      rotconv_plan* ch = nullptr;
      const int crc = rotconv_plan_create_opt(&cd, &p->opt, &ch);
      if (crc != ROTCONV_OK) {
        delete p;
        return crc;
      }
      int any = 0;
      for (int i = 0; i < 3; ++i) any |= p->pad_use[i] = pass_level(ch, i) > pass_level(p, i) ? 1 : 0;
      if (any) {
        p->pad_child = ch;
        p->ws_bytes = std::max(p->ws_bytes, pad_layout(p).total);
      } else {
        rotconv_plan_destroy(ch);
      }
    }
  }
  *out = p;
  return ROTCONV_OK;
}

int rotconv_plan_destroy(rotconv_plan* plan) {
  if (!plan) return ROTCONV_OK;
  if (plan->avg_child) rotconv_plan_destroy(plan->avg_child);
  if (plan->pad_child) rotconv_plan_destroy(plan->pad_child);
  free_device_tables(plan);
  delete plan;
  return ROTCONV_OK;
}

size_t rotconv_workspace_bytes(const rotconv_plan* plan) { return plan ? plan->ws_bytes : 0; }

size_t rotconv_workspace_bytes_unfused(const rotconv_plan* plan) {
  if (!plan) return 0;
  if (plan->d.dtype == ROTCONV_BF16) return plan->ws_bytes - plan->ws_inner + unfused_ws_inner(plan);   // staging areas in front
  return std::max(plan->ws_bytes, unfused_ws_inner(plan));
}

int rotconv_out_shape(const rotconv_plan* plan, int32_t* Ho, int32_t* Wo, int32_t* Cunpooled, int32_t* Cpooled) {
  if (!plan) return ROTCONV_ERR_NULL;
  if (Ho) *Ho = plan->Ho;
  if (Wo) *Wo = plan->Wo;
  if (Cunpooled) *Cunpooled = plan->d.Cout * plan->d.R;
  if (Cpooled) *Cpooled = plan->d.Cout * plan->ng;
  return ROTCONV_OK;
}

int rotconv_plan_orientations(const rotconv_plan* plan, int32_t* Q, int32_t* bank_of_r, int32_t* quarter_of_r) {
  if (!plan) return ROTCONV_ERR_NULL;
  if (Q) *Q = plan->host.Q;
  for (int r = 0; r < plan->d.R; ++r) {
    if (bank_of_r) bank_of_r[r] = plan->host.bank_of_r[r];
    if (quarter_of_r) quarter_of_r[r] = plan->host.quarter_of_r[r];
  }
  return ROTCONV_OK;
}

int rotconv_plan_expansion(const rotconv_plan* plan, float* E) {
  if (!plan || !E) return ROTCONV_ERR_NULL;
  const int kk = plan->kk, B = plan->B, R = plan->d.R;
  std::memset(E, 0, sizeof(float) * R * kk * B * kk);
  for (int row = 0; row < R * kk; ++row)
    for (int e = 0; e < kMaxNnz; ++e) {
      const int s = plan->host.exp_src[row * kMaxNnz + e];
      if (s >= 0) E[(size_t)row * B * kk + s] += plan->host.exp_coef[row * kMaxNnz + e];
    }
  return ROTCONV_OK;
}

int rotconv_plan_routed_table(const rotconv_plan* plan, float* T) {
  if (!plan || !T) return ROTCONV_ERR_NULL;
  if (plan->host.lut_bwd.empty() || plan->B != 1) return ROTCONV_ERR_UNSUPPORTED;
  const int R1 = plan->d.R + 1;
  for (int rel = 0; rel < 9; ++rel)
    for (int r = 0; r < R1; ++r)
      for (int u = 0; u < 9; ++u) T[((size_t)rel * R1 + r) * 9 + u] = plan->host.lut_bwd[((size_t)rel * R1 + r) * 12 + u];
  return ROTCONV_OK;
}

}  // extern "C" (the fp32 implementations below have internal linkage)

static int f32_rotconv_fwd(const rotconv_plan* plan, const void* x, const void* w, void* y, void* ws, size_t ws_bytes,
                void* stream) {
  if (!plan || !x || !w || !y) return ROTCONV_ERR_NULL;
  int rc = check_ws_inner(plan, ws, ws_bytes);
  if (rc) return rc;
  rotconv_plan* p = const_cast<rotconv_plan*>(plan);
  if ((rc = ensure_device_tables(p))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int cs = p->fwd_csplit[0];
  if (p->fast[0] && aligned(x, 8) && aligned(ws, cs > 1 ? 256 : 16) && aligned(y, 16)) {
    const float* wt = static_cast<const float*>(w);      // the kernel takes w itself, or the bank packed into ws
    if (!p4_fwd_raw_weights(p, 1, cs)) {
      launch_p4_pack_fwd(p, static_cast<const float*>(w), static_cast<float*>(ws), st);
      wt = static_cast<const float*>(ws);
    }
    if (cs > 1) {     // small map, deep input: the channels are split over workgroups
      float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + fwd_pack_region(p));
      launch_p4_fwd(p, kOutUnpooled, static_cast<const float*>(x), wt, part, nullptr, st, 1, cs);
      launch_p4_sum_parts(p, part, cs, static_cast<float*>(y), st);
      return finish();
    }
    launch_p4_fwd(p, kOutUnpooled, static_cast<const float*>(x), wt, static_cast<float*>(y), nullptr, st);
    return finish();
  }
  if (p->gs) {
    launch_gs_fwd(p, static_cast<const float*>(x), static_cast<const float*>(w), static_cast<float*>(y), ws, st);
    return finish();
  }
  float* wexp = static_cast<float*>(ws);
  launch_expand_bank(p, static_cast<const float*>(w), wexp, st);
  launch_fwd_generic(p, static_cast<const float*>(x), wexp, static_cast<float*>(y), st);
  return finish();
}

static int f32_rotconv_bwd_data(const rotconv_plan* plan, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes,
                     void* stream) {
  if (!plan || !dy || !w || !dx) return ROTCONV_ERR_NULL;
  int rc = check_ws_inner(plan, ws, ws_bytes);
  if (rc) return rc;
  rotconv_plan* p = const_cast<rotconv_plan*>(plan);
  if ((rc = ensure_device_tables(p))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // the unfused gradients of a plan whose fused calls run the register-resident kernels: matrix multiply + scatter
  // if the caller brought the larger workspace that family needs (rotconv_workspace_bytes_unfused), else generic
  if (unfused_on_gs(p, ws, ws_bytes)) {
    launch_gs_bwd_data(p, static_cast<const float*>(dy), static_cast<const float*>(w), static_cast<float*>(dx), ws, st);
    return finish();
  }
  float* wexp = static_cast<float*>(ws);
  launch_expand_bank(p, static_cast<const float*>(w), wexp, st);
  launch_bwd_data_generic(p, static_cast<const float*>(dy), wexp, static_cast<float*>(dx), st);
  return finish();
}

static int f32_rotconv_bwd_weight(const rotconv_plan* plan, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes,
                       void* stream) {
  if (!plan || !x || !dy || !dw) return ROTCONV_ERR_NULL;
  int rc = check_ws_inner(plan, ws, ws_bytes);
  if (rc) return rc;
  rotconv_plan* p = const_cast<rotconv_plan*>(plan);
  if ((rc = ensure_device_tables(p))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (unfused_on_gs(p, ws, ws_bytes)) {
    launch_gs_bwd_weight(p, static_cast<const float*>(x), static_cast<const float*>(dy), dw, ws, st);
    return finish();
  }
  launch_bwd_weight_generic(p, static_cast<const float*>(x), static_cast<const float*>(dy), nullptr, nullptr,
                            static_cast<float*>(ws), dw, st);
  return finish();
}

static int f32_orient_maxpool_fwd(const rotconv_plan* plan, const void* y, void* ypool, uint8_t* idx, void* stream) {
  if (plan && plan->avg_child) {
    if (!y || !ypool) return ROTCONV_ERR_NULL;
    launch_avgpool_fwd(plan, static_cast<const float*>(y), static_cast<float*>(ypool), static_cast<hipStream_t>(stream));
    return finish();
  }
  if (!plan || !y || !ypool || !idx) return ROTCONV_ERR_NULL;
  launch_maxpool_fwd(plan, static_cast<const float*>(y), static_cast<float*>(ypool), idx,
                     static_cast<hipStream_t>(stream));
  return finish();
}

static int f32_orient_maxpool_bwd(const rotconv_plan* plan, const void* gpool, const uint8_t* idx, void* dy, void* stream) {
  if (plan && plan->avg_child) {
    if (!gpool || !dy) return ROTCONV_ERR_NULL;
    launch_avgpool_bwd(plan, static_cast<const float*>(gpool), static_cast<float*>(dy), static_cast<hipStream_t>(stream));
    return finish();
  }
  if (!plan || !gpool || !idx || !dy) return ROTCONV_ERR_NULL;
  launch_maxpool_bwd(plan, static_cast<const float*>(gpool), idx, static_cast<float*>(dy),
                     static_cast<hipStream_t>(stream));
  return finish();
}

// Does the pooled forward of an fp32 plan run the register-resident kernel for these pointers?
static bool f32_pool_fwd_is_fast(const rotconv_plan* p, const void* x, const void* ypool, const uint8_t* idx,
                                 const void* ws) {
  return !p->avg_child && p->fast[0] && aligned(x, 8) && aligned(ws, 256) && aligned(ypool, 16) && aligned(idx, 8);
}

// Scratch the pooled forward of an fp32 plan touches: the packed banks (+ candidates / parts) of the register-resident
// kernel; every other route is sized by the plan's largest call.
static size_t f32_pool_fwd_need(const rotconv_plan* p, const void* x, const void* ypool, const uint8_t* idx,
                                const void* ws) {
  return f32_pool_fwd_is_fast(p, x, ypool, idx, ws) ? std::min(p->ws_inner, fwd_fast_ws_bytes(p)) : p->ws_inner;
}

// no_upload: the caller may not allocate, so a plan whose tables are not on this device yet is refused
static int f32_rotconv_pool_fwd(const rotconv_plan* plan, const void* x, const void* w, void* ypool, uint8_t* idx, void* ws,
                     size_t ws_bytes, void* stream, bool own_need = false, bool no_upload = false) {
  if (!plan || !x || !w || !ypool || (!idx && !plan->avg_child)) return ROTCONV_ERR_NULL;
  // own_need: the buffer only has to hold what THIS call touches, not the plan's largest call
  const size_t need = own_need ? f32_pool_fwd_need(plan, x, ypool, idx, ws) : plan->ws_inner;
  if (need && (!ws || ws_bytes < need)) return ROTCONV_ERR_WORKSPACE;
  int rc;
  rotconv_plan* p = const_cast<rotconv_plan*>(plan);
  if (no_upload && !tables_on_current_device(p)) return ROTCONV_ERR_UNSUPPORTED;
  if ((rc = ensure_device_tables(p))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (p->avg_child) {     // Eq. 9: the mean over a group = one convolution with the group-averaged bank
    const AvgLayout L = avg_layout(p);
    char* c = static_cast<char*>(ws);
    float* wexp = reinterpret_cast<float*>(c + L.wexp);
    float* wavg = reinterpret_cast<float*>(c + L.wavg);
    launch_expand_bank(p, static_cast<const float*>(w), wexp, st);
    launch_avg_bank(p, wexp, wavg, st);
    return rotconv_fwd(p->avg_child, x, wavg, ypool, c + L.child, p->avg_child->ws_bytes, stream);
  }
  if (f32_pool_fwd_is_fast(p, x, ypool, idx, ws)) {
    float* wt = static_cast<float*>(ws);
    char* extra = static_cast<char*>(ws) + fwd_pack_region(p);
    const int mode = p4_fwd_pool_mode(p);
    const size_t hw = (size_t)p->d.H * p->d.W;
    const int cs = p->fwd_csplit[1];
    // the bank the kernel multiplies with: w itself where the kernel can re-lay its block on its own, else packed into ws
    auto bank = [&](int nq_, int cs_) -> const float* {
      if (p4_fwd_raw_weights(p, nq_, cs_)) return static_cast<const float*>(w);
      launch_p4_pack_fwd(p, static_cast<const float*>(w), wt, st, nq_);
      return wt;
    };
    if (cs > 1) {     // small map, deep input: the channels are split over workgroups, summed and pooled afterwards
      float* part = reinterpret_cast<float*>(extra);
      launch_p4_fwd(p, kOutUnpooled, static_cast<const float*>(x), bank(1, cs), part, nullptr, st, 1, cs);
      launch_p4_sum_pool(p, part, cs, static_cast<float*>(ypool), idx, st);
      return finish();
    }
    if (p->fwd_base) {     // the pool group spans all banks: products of the base bank, banks combined in the kernel
      launch_p4_pack_base(p, static_cast<const float*>(w), wt, st);
      launch_p4_fwd_base(p, static_cast<const float*>(x), wt, static_cast<float*>(ypool), idx, st);
      return finish();
    }
    const int nq = mode == kOutPartial ? p4_fwd_fold(p) : 1;
    const float* wb = bank(nq, 1);
    if (mode == kOutPooled) {
      launch_p4_fwd(p, mode, static_cast<const float*>(x), wb, static_cast<float*>(ypool), idx, st);
    } else if (nq > 1) {     // the pool group spans all banks: pooled across them inside the kernel
      launch_p4_fwd(p, kOutPooled, static_cast<const float*>(x), wb, static_cast<float*>(ypool), idx, st, nq);
    } else if (mode == kOutPartial) {
      float* pv = reinterpret_cast<float*>(extra);
      uint8_t* pi = reinterpret_cast<uint8_t*>(extra + align256((size_t)p->host.Q * p->d.N * p->d.Cout * hw * 4));
      launch_p4_fwd(p, mode, static_cast<const float*>(x), wb, pv, pi, st);
      launch_p4_combine(p, pv, pi, static_cast<float*>(ypool), idx, st);
    } else {
      float* yu = reinterpret_cast<float*>(extra);
      launch_p4_fwd(p, mode, static_cast<const float*>(x), wb, yu, nullptr, st);
      launch_maxpool_fwd(p, yu, static_cast<float*>(ypool), idx, st, true);
    }
    return finish();
  }
  if (p->gs) {
    launch_gs_pool_fwd(p, static_cast<const float*>(x), static_cast<const float*>(w), static_cast<float*>(ypool), idx,
                       ws, st);
    return finish();
  }
  float* wexp = static_cast<float*>(ws);
  launch_expand_bank(p, static_cast<const float*>(w), wexp, st);
  launch_pool_fwd_generic(p, static_cast<const float*>(x), wexp, static_cast<float*>(ypool), idx, st);
  return finish();
}

static int f32_rotconv_pool_bwd_data(const rotconv_plan* plan, const void* gpool, const uint8_t* idx, const void* w, void* dx,
                          void* ws, size_t ws_bytes, void* stream) {
  if (!plan || !gpool || (!idx && !plan->avg_child) || !w || !dx) return ROTCONV_ERR_NULL;
  int rc = check_ws_inner(plan, ws, ws_bytes);
  if (rc) return rc;
  rotconv_plan* p = const_cast<rotconv_plan*>(plan);
  if ((rc = ensure_device_tables(p))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (p->avg_child) {     // Eq. 11 + 13 + 15: the input gradient of that one convolution (its only orientation is 0)
    const AvgLayout L = avg_layout(p);
    char* c = static_cast<char*>(ws);
    float* wexp = reinterpret_cast<float*>(c + L.wexp);
    float* wavg = reinterpret_cast<float*>(c + L.wavg);
    uint8_t* idx0 = reinterpret_cast<uint8_t*>(c + L.idx0);
    launch_expand_bank(p, static_cast<const float*>(w), wexp, st);
    launch_avg_bank(p, wexp, wavg, st);
    launch_fill_u8(idx0, p->n_yp, 0, st);
    return rotconv_pool_bwd_data(p->avg_child, gpool, idx0, wavg, dx, c + L.child, p->avg_child->ws_bytes, stream);
  }
  if (p->fast[1] && aligned(gpool, 8) && aligned(idx, 2) && aligned(dx, 16) && aligned(ws, 16)) {
    const bool raw = p4_bwd_data_raw_weights(p) && aligned(w, 16);   // the kernel takes w itself, 16 bytes at a time
    const float* wd = static_cast<const float*>(w);
    if (!raw) {                                                       // ... or the banks packed into ws
      launch_p4_pack_bwd(p, static_cast<const float*>(w), static_cast<float*>(ws), st);
      wd = static_cast<const float*>(ws);
    }
    float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + align256(p4_bwd_data_pack_floats(p) * sizeof(float)));
    launch_p4_bwd_data(p, static_cast<const float*>(gpool), idx, wd, static_cast<float*>(dx), part, st, raw);
    return finish();
  }
  if (p->gs) {
    launch_gs_pool_bwd_data(p, static_cast<const float*>(gpool), idx, static_cast<const float*>(w),
                            static_cast<float*>(dx), ws, st);
    return finish();
  }
  float* wexp = static_cast<float*>(ws);
  launch_expand_bank(p, static_cast<const float*>(w), wexp, st);
  launch_pool_bwd_data_generic(p, static_cast<const float*>(gpool), idx, wexp, static_cast<float*>(dx), st);
  return finish();
}

static int f32_rotconv_pool_bwd_weight(const rotconv_plan* plan, const void* x, const void* gpool, const uint8_t* idx, float* dw,
                            void* ws, size_t ws_bytes, void* stream) {
  if (!plan || !x || !gpool || (!idx && !plan->avg_child) || !dw) return ROTCONV_ERR_NULL;
  int rc = check_ws_inner(plan, ws, ws_bytes);
  if (rc) return rc;
  rotconv_plan* p = const_cast<rotconv_plan*>(plan);
  if ((rc = ensure_device_tables(p))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (p->avg_child) {     // Eq. 11 + 14 + 16: that convolution's weight gradient, shared out to the R banks, reduced
    const AvgLayout L = avg_layout(p);
    char* c = static_cast<char*>(ws);
    float* rep = reinterpret_cast<float*>(c + L.wexp);
    float* dwavg = reinterpret_cast<float*>(c + L.wavg);
    uint8_t* idx0 = reinterpret_cast<uint8_t*>(c + L.idx0);
    launch_fill_u8(idx0, p->n_yp, 0, st);
    rc = rotconv_pool_bwd_weight(p->avg_child, x, gpool, idx0, dwavg, c + L.child, p->avg_child->ws_bytes, stream);
    if (rc) return rc;
    launch_avg_bank_bwd(p, dwavg, rep, dw, st);
    return finish();
  }
  if (p->fast[2] && aligned(x, 16) && aligned(gpool, 16) && aligned(idx, 4) && aligned(ws, 16)) {
    launch_p4_bwd_weight(p, static_cast<const float*>(x), static_cast<const float*>(gpool), idx,
                         static_cast<float*>(ws), dw, st);
    return finish();
  }
  if (p->gs) {
    launch_gs_pool_bwd_weight(p, static_cast<const float*>(x), static_cast<const float*>(gpool), idx, dw, ws, st);
    return finish();
  }
  launch_bwd_weight_generic(p, static_cast<const float*>(x), nullptr, static_cast<const float*>(gpool), idx,
                            static_cast<float*>(ws), dw, st);
  return finish();
}

extern "C" {

// ---- public entry points: fp32 plans go straight to the kernels; bf16 plans widen the bf16 tensors into
// fp32 staging areas at the head of the workspace, run the same kernels behind them, and round the results to
// bf16 once (the arg-max is taken on the fp32 values).  dW is fp32 in both cases. ----

namespace {

struct Stage {               // fp32 staging areas of a bf16 plan inside the caller's workspace
  float *x, *w, *y;          // input-sized, weight-sized, (unpooled-)output-sized
  void* inner;               // workspace handed on to the fp32 path
  size_t inner_bytes;
};

Stage carve(const rotconv_plan* p, void* ws, size_t ws_bytes) {
  Stage s;
  char* c = static_cast<char*>(ws);
  s.x = reinterpret_cast<float*>(c); c += align256(p->n_x * 4);
  s.w = reinterpret_cast<float*>(c); c += align256(p->n_w * 4);
  s.y = reinterpret_cast<float*>(c); c += align256(p->n_yu * 4);
  s.inner = c;
  s.inner_bytes = ws_bytes - (size_t)(c - static_cast<char*>(ws));
  return s;
}

bool is_bf16(const rotconv_plan* p) { return p->d.dtype == ROTCONV_BF16; }
const uint16_t* h16(const void* p) { return static_cast<const uint16_t*>(p); }

// The calls of a plan with padded rows: stage the tensors at the child's row width, run the child, crop.
struct PadCtx {
  const rotconv_plan* ch;
  char *in, *out, *idx, *cws;
  int es, W, Wp;
  size_t rows_x, rows_p, rows_u;    // rows of the input, the pooled and the unpooled maps
  hipStream_t st;
};
int pad_ctx(const rotconv_plan* p, void* ws, size_t ws_bytes, void* stream, PadCtx* c) {
  if (!ws || ws_bytes < p->ws_bytes) return ROTCONV_ERR_WORKSPACE;
  const PadLayout L = pad_layout(p);
  char* b = static_cast<char*>(ws);
  c->ch = p->pad_child;
  c->in = b + L.in; c->out = b + L.out; c->idx = b + L.idx; c->cws = b + L.child;
  c->es = is_bf16(p) ? 2 : 4;
  c->W = p->d.W; c->Wp = p->pad_child->d.W;
  c->rows_x = (size_t)p->d.N * p->d.Cin * p->d.H;
  c->rows_p = (size_t)p->d.N * p->d.Cout * p->ng * p->d.H;
  c->rows_u = (size_t)p->d.N * p->d.Cout * p->d.R * p->d.H;
  c->st = static_cast<hipStream_t>(stream);
  return ROTCONV_OK;
}

}  // namespace

int rotconv_fwd(const rotconv_plan* plan, const void* x, const void* w, void* y, void* ws, size_t ws_bytes,
                void* stream) {
  if (!plan || !x || !w || !y) return ROTCONV_ERR_NULL;
  if (plan->pad_child && plan->pad_use[0]) {
    PadCtx c;
    int rc = pad_ctx(plan, ws, ws_bytes, stream, &c);
    if (rc) return rc;
    launch_repitch(x, c.in, c.rows_x, c.W, c.Wp, c.es, 0, c.st);
    if ((rc = rotconv_fwd(c.ch, c.in, w, c.out, c.cws, c.ch->ws_bytes, stream))) return rc;
    launch_repitch(c.out, y, c.rows_u, c.Wp, c.W, c.es, 0, c.st);
    return finish();
  }
  if (!is_bf16(plan)) return f32_rotconv_fwd(plan, x, w, y, ws, ws_bytes, stream);
  if (!ws || ws_bytes < plan->ws_bytes) return ROTCONV_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (plan->native16[0] && aligned(x, 4) && aligned(w, 2) && aligned(ws, 256) && aligned(y, 16)) {
    rotconv_plan* p = const_cast<rotconv_plan*>(plan);
    const int rc = ensure_device_tables(p);
    if (rc) return rc;
    uint16_t* wt = static_cast<uint16_t*>(ws);
    launch_p4_pack_fwd_bf16(p, 1, h16(w), wt, st);
    launch_p4_fwd_bf16(p, kOutUnpooled, 1, h16(x), wt, y, nullptr, st);
    return finish();
  }
  const Stage s = carve(plan, ws, ws_bytes);
  launch_widen(h16(x), s.x, plan->n_x, st);
  launch_widen(h16(w), s.w, plan->n_w, st);
  const int rc = f32_rotconv_fwd(plan, s.x, s.w, s.y, s.inner, s.inner_bytes, stream);
  if (rc) return rc;
  launch_narrow(s.y, static_cast<uint16_t*>(y), plan->n_yu, st);
  return finish();
}

int rotconv_bwd_data(const rotconv_plan* plan, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes,
                     void* stream) {
  if (!plan || !dy || !w || !dx) return ROTCONV_ERR_NULL;
  if (!is_bf16(plan)) return f32_rotconv_bwd_data(plan, dy, w, dx, ws, ws_bytes, stream);
  if (!ws || ws_bytes < plan->ws_bytes) return ROTCONV_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const Stage s = carve(plan, ws, ws_bytes);
  launch_widen(h16(dy), s.y, plan->n_yu, st);
  launch_widen(h16(w), s.w, plan->n_w, st);
  const int rc = f32_rotconv_bwd_data(plan, s.y, s.w, s.x, s.inner, s.inner_bytes, stream);
  if (rc) return rc;
  launch_narrow(s.x, static_cast<uint16_t*>(dx), plan->n_x, st);
  return finish();
}

int rotconv_bwd_weight(const rotconv_plan* plan, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes,
                       void* stream) {
  if (!plan || !x || !dy || !dw) return ROTCONV_ERR_NULL;
  if (!is_bf16(plan)) return f32_rotconv_bwd_weight(plan, x, dy, dw, ws, ws_bytes, stream);
  if (!ws || ws_bytes < plan->ws_bytes) return ROTCONV_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const Stage s = carve(plan, ws, ws_bytes);
  launch_widen(h16(x), s.x, plan->n_x, st);
  launch_widen(h16(dy), s.y, plan->n_yu, st);
  return f32_rotconv_bwd_weight(plan, s.x, s.y, dw, s.inner, s.inner_bytes, stream);
}

int orient_maxpool_fwd(const rotconv_plan* plan, const void* y, void* ypool, uint8_t* idx, void* stream) {
  if (!plan || !y || !ypool || (!idx && !plan->avg_child)) return ROTCONV_ERR_NULL;
  if (!is_bf16(plan)) return f32_orient_maxpool_fwd(plan, y, ypool, idx, stream);
  if (plan->avg_child) {
    launch_avgpool_fwd_bf16(plan, h16(y), static_cast<uint16_t*>(ypool), static_cast<hipStream_t>(stream));
    return finish();
  }
  launch_maxpool_fwd_bf16(plan, h16(y), static_cast<uint16_t*>(ypool), idx, static_cast<hipStream_t>(stream));
  return finish();
}

int orient_maxpool_bwd(const rotconv_plan* plan, const void* gpool, const uint8_t* idx, void* dy, void* stream) {
  if (!plan || !gpool || (!idx && !plan->avg_child) || !dy) return ROTCONV_ERR_NULL;
  if (!is_bf16(plan)) return f32_orient_maxpool_bwd(plan, gpool, idx, dy, stream);
  if (plan->avg_child) {
    launch_avgpool_bwd_bf16(plan, h16(gpool), static_cast<uint16_t*>(dy), static_cast<hipStream_t>(stream));
    return finish();
  }
  launch_maxpool_bwd_bf16(plan, h16(gpool), idx, static_cast<uint16_t*>(dy), static_cast<hipStream_t>(stream));
  return finish();
}

namespace {

// Does the pooled forward of a bf16 plan run the bf16 matrix-core kernel for these pointers?
bool bf16_pool_fwd_is_native(const rotconv_plan* plan, const void* x, const void* w, const void* ypool,
                             const uint8_t* idx, const void* ws) {
  const int pmode = plan->native16[0] ? p4_fwd_pool_mode(plan) : kOutUnpooled;
  return pmode != kOutUnpooled && aligned(x, 4) && aligned(w, 2) && aligned(ws, 256) && aligned(ypool, 16) &&
         aligned(idx, 8);
}

// Bytes of `ws` one call of the pooled forward touches, by the route it takes for these pointers (never more than
// rotconv_workspace_bytes, which is the largest need of any call on the plan).
// Does the pooled forward run the vector-ALU kernel of layers with at most four input channels for these pointers?
bool pool_fwd_is_direct(const rotconv_plan* p, const void* x, const void* ypool, const void* ws) {
  const size_t es = is_bf16(p) ? 2 : 4;
  return p->direct[0] && aligned(x, es) && aligned(ypool, es) && aligned(ws, 16);
}

bool pool_fwd_is_px16(const rotconv_plan* p, const void* x, const void* ypool, const void* ws) {
  return p->px16 && aligned(x, 2) && aligned(ypool, 2) && aligned(ws, 16);
}

size_t pool_fwd_need(const rotconv_plan* plan, const void* x, const void* w, const void* ypool, const uint8_t* idx,
                     const void* ws) {
  if (plan->pad_child && plan->pad_use[0]) return plan->ws_bytes;             // staging copies + the padded plan
  if (pool_fwd_is_px16(plan, x, ypool, ws)) return align256(px_fwd_bf16_pack_bytes(plan));
  if (pool_fwd_is_direct(plan, x, ypool, ws)) return align256(direct_fwd_pack_floats(plan) * sizeof(float));
  if (!is_bf16(plan)) return f32_pool_fwd_need(plan, x, ypool, idx, ws);
  if (bf16_pool_fwd_is_native(plan, x, w, ypool, idx, ws)) return std::min(plan->ws_bytes, fwd_fast_ws_bytes(plan));
  return plan->ws_bytes;                                                      // fp32 staging areas in front
}

// own_need: `ws` has to hold what this call touches (pool_fwd_need), not the plan's largest call.
// no_upload: no allocation allowed: a plan whose tables are not on the current device yet is refused.
int pool_fwd_impl(const rotconv_plan* plan, const void* x, const void* w, void* ypool, uint8_t* idx, void* ws,
                  size_t ws_bytes, void* stream, bool own_need, bool no_upload) {
  if (!plan || !x || !w || !ypool || (!idx && !plan->avg_child)) return ROTCONV_ERR_NULL;
  if (plan->pad_child && plan->pad_use[0]) {
    if (no_upload && !tables_on_current_device(plan->pad_child)) return ROTCONV_ERR_UNSUPPORTED;
    PadCtx c;
    int rc = pad_ctx(plan, ws, ws_bytes, stream, &c);
    if (rc) return rc;
    launch_repitch(x, c.in, c.rows_x, c.W, c.Wp, c.es, 0, c.st);
    if ((rc = pool_fwd_impl(c.ch, c.in, w, c.out, reinterpret_cast<uint8_t*>(c.idx), c.cws, c.ch->ws_bytes, stream, false,
                            no_upload)))
      return rc;
    launch_repitch(c.out, ypool, c.rows_p, c.Wp, c.W, c.es, 0, c.st);
    launch_repitch(c.idx, idx, c.rows_p, c.Wp, c.W, 1, 0, c.st);
    return finish();
  }
  if (pool_fwd_is_direct(plan, x, ypool, ws)) {     // at most four input channels: the vector-ALU kernel
    const size_t dneed = own_need ? pool_fwd_need(plan, x, w, ypool, idx, ws) : plan->ws_bytes;
    if (!ws || ws_bytes < dneed) return ROTCONV_ERR_WORKSPACE;
    if (no_upload && !tables_on_current_device(plan)) return ROTCONV_ERR_UNSUPPORTED;
    rotconv_plan* p = const_cast<rotconv_plan*>(plan);
    const int rc = ensure_device_tables(p);
    if (rc) return rc;
    launch_direct_fwd(p, x, w, ypool, idx, static_cast<float*>(ws), static_cast<hipStream_t>(stream));
    return finish();
  }
  if (pool_fwd_is_px16(plan, x, ypool, ws)) {
    const size_t pneed = own_need ? pool_fwd_need(plan, x, w, ypool, idx, ws) : plan->ws_bytes;
    if (!ws || ws_bytes < pneed) return ROTCONV_ERR_WORKSPACE;
    if (no_upload && !tables_on_current_device(plan)) return ROTCONV_ERR_UNSUPPORTED;
    rotconv_plan* p = const_cast<rotconv_plan*>(plan);
    const int rc = ensure_device_tables(p);
    if (rc) return rc;
    launch_px_fwd_bf16(p, h16(x), h16(w), static_cast<uint16_t*>(ypool), idx, static_cast<uint16_t*>(ws),
                       static_cast<hipStream_t>(stream));
    return finish();
  }
  if (!is_bf16(plan)) return f32_rotconv_pool_fwd(plan, x, w, ypool, idx, ws, ws_bytes, stream, own_need, no_upload);
  const size_t need = own_need ? pool_fwd_need(plan, x, w, ypool, idx, ws) : plan->ws_bytes;
  if (!ws || ws_bytes < need) return ROTCONV_ERR_WORKSPACE;
  if (no_upload && !tables_on_current_device(plan)) return ROTCONV_ERR_UNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (bf16_pool_fwd_is_native(plan, x, w, ypool, idx, ws)) {
    // bf16 tensors straight into the bf16 matrix-core kernel; scratch laid out as in the fp32 path
    const int pmode = p4_fwd_pool_mode(plan);
    rotconv_plan* p = const_cast<rotconv_plan*>(plan);
    const int rc = ensure_device_tables(p);
    if (rc) return rc;
    uint16_t* wt = static_cast<uint16_t*>(ws);
    char* extra = static_cast<char*>(ws) + fwd_pack_region(p);
    const size_t hw = (size_t)p->d.H * p->d.W;
    const int nq = pmode == kOutPartial ? p4_fwd_bf16_fold(p) : 1;
    launch_p4_pack_fwd_bf16(p, nq, h16(w), wt, st);
    if (pmode == kOutPooled) {
      launch_p4_fwd_bf16(p, pmode, 1, h16(x), wt, ypool, idx, st);
    } else if (nq > 1) {     // the pool group spans all banks: pooled across them inside the kernel
      launch_p4_fwd_bf16(p, kOutPooled, nq, h16(x), wt, ypool, idx, st);
    } else {
      float* pv = reinterpret_cast<float*>(extra);
      uint8_t* pi = reinterpret_cast<uint8_t*>(extra + align256((size_t)p->host.Q * p->d.N * p->d.Cout * hw * 4));
      launch_p4_fwd_bf16(p, pmode, 1, h16(x), wt, pv, pi, st);
      launch_p4_combine_bf16(p, pv, pi, static_cast<uint16_t*>(ypool), idx, st);
    }
    return finish();
  }
  const Stage s = carve(plan, ws, ws_bytes);
  launch_widen(h16(x), s.x, plan->n_x, st);
  launch_widen(h16(w), s.w, plan->n_w, st);
  const int rc = f32_rotconv_pool_fwd(plan, s.x, s.w, s.y, idx, s.inner, s.inner_bytes, stream, false, no_upload);
  if (rc) return rc;
  launch_narrow(s.y, static_cast<uint16_t*>(ypool), plan->n_yp, st);
  return finish();
}

// ---- scratch of the entry point that allocates nothing ------------------------------------------------------
// One array per GPU (each device that loads this code object holds its own copy at its own address, until the
// process ends).  Host code never uses the array's name as an address: static_scratch() resolves the device
// address once per device with hipGetSymbolAddress and hands that pointer to the kernels.
constexpr size_t kStaticScratchBytes = ROTCONV_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (nullptr on failure).
static void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr) return ptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
    (void)hipGetLastError();
    return nullptr;
  }
  g_scratch_ptr[dev].store(ptr, std::memory_order_release);     // every thread resolves the same address
  return ptr;
}

}  // namespace

int rotconv_pool_fwd(const rotconv_plan* plan, const void* x, const void* w, void* ypool, uint8_t* idx, void* ws,
                     size_t ws_bytes, void* stream) {
  return pool_fwd_impl(plan, x, w, ypool, idx, ws, ws_bytes, stream, false, false);
}

int rotconv_pool_fwd_static(const rotconv_plan* plan, const void* x, const void* w, void* ypool, uint8_t* idx,
                            void* stream) {
  if (!plan || !x || !w || !ypool || (!idx && !plan->avg_child)) return ROTCONV_ERR_NULL;
  void* ws = static_scratch();
  if (!ws) return ROTCONV_ERR_LAUNCH;
  if (pool_fwd_need(plan, x, w, ypool, idx, ws) > kStaticScratchBytes) return ROTCONV_ERR_WORKSPACE;
  return pool_fwd_impl(plan, x, w, ypool, idx, ws, kStaticScratchBytes, stream, true, true);
}

int rotconv_pool_bwd_data(const rotconv_plan* plan, const void* gpool, const uint8_t* idx, const void* w, void* dx,
                          void* ws, size_t ws_bytes, void* stream) {
  if (!plan || !gpool || (!idx && !plan->avg_child) || !w || !dx) return ROTCONV_ERR_NULL;
  if (plan->pad_child && plan->pad_use[1]) {     // padded columns: zero gradient, idx 255 (matches no orientation)
    PadCtx c;
    int rc = pad_ctx(plan, ws, ws_bytes, stream, &c);
    if (rc) return rc;
    launch_repitch(gpool, c.out, c.rows_p, c.W, c.Wp, c.es, 0, c.st);
    launch_repitch(idx, c.idx, c.rows_p, c.W, c.Wp, 1, 0xff, c.st);
    if ((rc = rotconv_pool_bwd_data(c.ch, c.out, reinterpret_cast<const uint8_t*>(c.idx), w, c.in, c.cws,
                                    c.ch->ws_bytes, stream)))
      return rc;
    launch_repitch(c.in, dx, c.rows_x, c.Wp, c.W, c.es, 0, c.st);
    return finish();
  }
  if (!is_bf16(plan)) return f32_rotconv_pool_bwd_data(plan, gpool, idx, w, dx, ws, ws_bytes, stream);
  if (!ws || ws_bytes < plan->ws_bytes) return ROTCONV_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (plan->native16[1] && aligned(gpool, 4) && aligned(idx, 2) && aligned(dx, 16) && aligned(ws, 16)) {
    rotconv_plan* p = const_cast<rotconv_plan*>(plan);
    const int rc = ensure_device_tables(p);
    if (rc) return rc;
    uint16_t* wt = static_cast<uint16_t*>(ws);
    if (p->bwd_lut16[1]) {     // routed-gradient table: one contraction with the base bank
      launch_p4_pack_bwd_bf16_lut(p, h16(w), wt, st);
      float* lpart = reinterpret_cast<float*>(static_cast<char*>(ws) + align256(p4_bwd_data_bf16_lut_pack_bytes(p)));
      launch_p4_bwd_data_bf16_lut(p, h16(gpool), idx, wt, static_cast<uint16_t*>(dx), lpart, st);
      return finish();
    }
    launch_p4_pack_bwd_bf16(p, h16(w), wt, st);
    float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + align256(p4_bwd_data_bf16_pack_bytes(p)));
    launch_p4_bwd_data_bf16(p, h16(gpool), idx, wt, static_cast<uint16_t*>(dx), part, st);
    return finish();
  }
  const Stage s = carve(plan, ws, ws_bytes);
  launch_widen(h16(gpool), s.y, plan->n_yp, st);
  launch_widen(h16(w), s.w, plan->n_w, st);
  const int rc = f32_rotconv_pool_bwd_data(plan, s.y, idx, s.w, s.x, s.inner, s.inner_bytes, stream);
  if (rc) return rc;
  launch_narrow(s.x, static_cast<uint16_t*>(dx), plan->n_x, st);
  return finish();
}

int rotconv_pool_bwd_weight(const rotconv_plan* plan, const void* x, const void* gpool, const uint8_t* idx, float* dw,
                            void* ws, size_t ws_bytes, void* stream) {
  if (!plan || !x || !gpool || (!idx && !plan->avg_child) || !dw) return ROTCONV_ERR_NULL;
  if (plan->pad_child && plan->pad_use[2]) {
    PadCtx c;
    const int rc = pad_ctx(plan, ws, ws_bytes, stream, &c);
    if (rc) return rc;
    launch_repitch(x, c.in, c.rows_x, c.W, c.Wp, c.es, 0, c.st);
    launch_repitch(gpool, c.out, c.rows_p, c.W, c.Wp, c.es, 0, c.st);
    launch_repitch(idx, c.idx, c.rows_p, c.W, c.Wp, 1, 0xff, c.st);
    return rotconv_pool_bwd_weight(c.ch, c.in, c.out, reinterpret_cast<const uint8_t*>(c.idx), dw, c.cws,
                                   c.ch->ws_bytes, stream);
  }
  if (plan->direct[2] && aligned(x, is_bf16(plan) ? 2 : 4) && aligned(gpool, is_bf16(plan) ? 2 : 4) && aligned(ws, 16)) {
    if (!ws || ws_bytes < plan->ws_bytes) return ROTCONV_ERR_WORKSPACE;
    rotconv_plan* p = const_cast<rotconv_plan*>(plan);
    const int rc = ensure_device_tables(p);
    if (rc) return rc;
    launch_direct_bwd_weight(p, x, gpool, idx, static_cast<float*>(ws), dw, static_cast<hipStream_t>(stream));
    return finish();
  }
  if (!is_bf16(plan)) return f32_rotconv_pool_bwd_weight(plan, x, gpool, idx, dw, ws, ws_bytes, stream);
  if (!ws || ws_bytes < plan->ws_bytes) return ROTCONV_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (plan->native16[2] && aligned(x, 16) && aligned(gpool, 16) && aligned(idx, 8) && aligned(ws, 16)) {
    rotconv_plan* p = const_cast<rotconv_plan*>(plan);
    const int rc = ensure_device_tables(p);
    if (rc) return rc;
    launch_p4_bwd_weight_bf16(p, h16(x), h16(gpool), idx, static_cast<float*>(ws), dw, st);
    return finish();
  }
  const Stage s = carve(plan, ws, ws_bytes);
  launch_widen(h16(x), s.x, plan->n_x, st);
  launch_widen(h16(gpool), s.y, plan->n_yp, st);
  return f32_rotconv_pool_bwd_weight(plan, s.x, s.y, idx, dw, s.inner, s.inner_bytes, stream);
}

const char* rotconv_status_string(int status) {
  switch (status) {
    case ROTCONV_OK: return "ok";
    case ROTCONV_ERR_NULL: return "null pointer argument";
    case ROTCONV_ERR_SHAPE: return "invalid shape, stride, padding or pool group";
    case ROTCONV_ERR_ANGLES: return "invalid angle set for this mode";
    case ROTCONV_ERR_UNSUPPORTED: return "request not supported by this build";
    case ROTCONV_ERR_WORKSPACE: return "workspace missing or too small";
    case ROTCONV_ERR_LAUNCH: return "HIP runtime error";
    default: return "unknown status";
  }
}

double rotconv_plan_conv_equivalents(const rotconv_plan* plan, int pass) {
  if (!plan || pass < 0 || pass > 2) return 0.0;
  if (plan->pad_child && plan->pad_use[pass]) return rotconv_plan_conv_equivalents(plan->pad_child, pass);
  const int Q = plan->host.Q, B = plan->B;
  if (plan->avg_child) return (double)plan->ng * rotconv_plan_conv_equivalents(plan->avg_child, pass);
  if (plan->direct[pass]) return Q;     // one product set per first-quadrant bank, on the vector ALU
  if (plan->d.dtype == ROTCONV_BF16 && plan->native16[pass]) {
    int present = 0;      // orientations in the set: the bf16 gradient kernels multiply every quarter turn on its own
    for (int i = 0; i < Q * 4; ++i) present += plan->rot_of[i] >= 0 ? 1 : 0;
    if (pass == 0) return Q;
    if (plan->bwd_lut16[pass]) return B;       // routed gradients folded into the base taps
    if (pass == 1) return p4_bwd_data_bf16_sparse(plan) ? 0.5 * present : present;   // 2-of-4 sparse operand: half the instructions
    return present;
  }
  if (plan->fast[pass]) {
    if (pass == 0) return plan->fwd_base ? B : Q;
    return plan->bwd_lut ? B : Q;
  }
  if (plan->gs) return Q;
  return plan->d.R;
}

const char* rotconv_plan_kernel_name(const rotconv_plan* plan, int pass) {
  if (!plan || pass < 0 || pass > 4) return "none";
  if (pass >= 3)      // the unfused gradient calls, given rotconv_workspace_bytes_unfused of scratch
    return plan->gs || (plan->d.pool_op != ROTCONV_POOL_AVG && gs_wanted(plan)) ? "mfma_gemm_scatter" : "generic";
  if (plan->pad_child && plan->pad_use[pass]) return rotconv_plan_kernel_name(plan->pad_child, pass);
  if (plan->direct[pass]) return "valu_direct";
  if (pass == 0 && plan->px16) return "mfma_px_bf16";
  if (plan->d.dtype == ROTCONV_BF16 && plan->native16[pass]) return plan->bwd_lut16[pass] ? "mfma_p4_bf16_lut" : "mfma_p4_bf16";
  if (pass == 0 && plan->fast[0] && plan->fwd_base) return "mfma_p4_base";   // the pooled forward; rotconv_fwd: mfma_p4
  return plan->fast[pass] ? "mfma_p4" : plan->gs ? "mfma_gemm_scatter" : "generic";
}

}  // extern "C"
