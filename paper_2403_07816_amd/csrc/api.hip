// C ABI of the library: argument validation, workspace carving, and the order in which
// the stages of the layer are enqueued.  See include/btx_moe.h for the contract.
#include <cmath>

#include "common.h"

using namespace btx;

namespace {

struct Carver {
  char* base; size_t used;
  explicit Carver(void* p) : base(static_cast<char*>(p)), used(0) {}
  void* take(size_t bytes) {
    void* p = base ? base + used : nullptr;
    used += align_up(bytes, 256);
    return p;
  }
};

inline int esize(int dtype) { return dtype == BTX_BF16 ? 2 : 4; }
inline bool dtype_ok(int dtype) { return dtype == BTX_F32 || dtype == BTX_BF16; }

struct FwdWs { void *xs, *act, *y, *h1, *h3, *partial; size_t bytes; };
FwdWs carve_forward(void* ws, int T, int d, int f, int k, int dtype, bool save) {
  const size_t R = (size_t)T * k, es = esize(dtype);
  Carver c(ws);
  FwdWs w;
  // gathered token rows, unless the GEMMs read them through perm themselves
  w.xs = ff_gather_fused(dtype, T, d, f) ? nullptr : c.take(R * d * es);
  w.act = c.take(R * f * es);
  w.y = c.take(R * d * es);
  // h1/h3 when the caller does not keep them: only the plain path needs them at all
  const bool own_h = !save && ff_up_needs_h(dtype, d, f);
  w.h1 = own_h ? c.take(R * f * es) : nullptr;
  w.h3 = own_h ? c.take(R * f * es) : nullptr;
  const size_t split = ff_split_bytes(dtype, d, f);      // K slices of DOWN's last round
  w.partial = split ? c.take(split) : nullptr;
  w.bytes = c.used;
  return w;
}

struct BwdWs { void *xs, *dysT, *dys, *dh1, *dh3, *ga, *dxs, *scratch, *router, *partial; float* dg_part; size_t bytes; };
BwdWs carve_backward(void* ws, int T, int d, int f, int E, int k, int dtype) {
  const size_t R = (size_t)T * k, es = esize(dtype);
  Carver c(ws);
  BwdWs w;
  // the dW products take x and dY either as grouped rows or transposed and padded
  const bool tr = ff_dw_transposed(dtype, d, f);
  const size_t dw_op = tr ? (size_t)d * ff_dw_pitch((int)R, E) * es : R * d * es;
  w.xs = c.take(dw_op);
  w.dysT = tr ? c.take(dw_op) : nullptr;
  w.dys = ff_gather_fused(dtype, T, d, f) ? nullptr : c.take(R * d * es);
  w.dh1 = c.take(R * f * es);
  w.dh3 = c.take(R * f * es);
  // transposed path: dW2 reads ga as [f][padded rows]
  w.ga = c.take(tr ? (size_t)f * ff_dw_pitch((int)R, E) * es : R * f * es);
  w.dxs = c.take(R * d * es);
  w.dg_part = static_cast<float*>(c.take(R * (size_t)bwd_act_partials(dtype, d, f) * sizeof(float)));
  w.scratch = c.take(ff_scratch_bytes(dtype, (int)R, f));
  w.router = c.take(router_bwd_workspace_bytes(T, d, E));
  const size_t split = ff_split_bytes(dtype, d, f);      // K slices of BWD_DX's last round
  w.partial = split ? c.take(split) : nullptr;
  w.bytes = c.used;
  return w;
}

// Optional profiling aid: when set, every stage of the layer is bracketed by a pair of
// events recorded on the caller's stream (see btx_profile_stages in the header).
hipEvent_t* g_stage_events = nullptr;
int g_stage_event_pairs = 0;

struct StageTimer {
  int id; hipStream_t s;
  StageTimer(int id_, hipStream_t s_) : id(id_), s(s_) {
    if (g_stage_events && id < g_stage_event_pairs) (void)hipEventRecord(g_stage_events[2 * id], s);
  }
  ~StageTimer() {
    if (g_stage_events && id < g_stage_event_pairs) (void)hipEventRecord(g_stage_events[2 * id + 1], s);
  }
};
#define BTX_STAGE(id, call)            \
  do {                                 \
    StageTimer timer_(id, s);          \
    if (int rc_ = (call)) return rc_;  \
  } while (0)

// Workspace of btx_moe_route_noalloc: a fixed array in the library's device image instead of a
// buffer the caller allocates.  Every GPU holds its own copy at its own address; the array's
// name is only a host-side handle, so the address is looked up once per device (with that
// device current) and the kernels are given that pointer.
constexpr size_t kStaticRouteBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticRouteBytes];
void* g_scratch_ptr[64] = {};

int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return BTX_ERR_HIP;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BTX_ERR_HIP;
    g_scratch_ptr[dev] = p;       // threads racing here store the same value
  }
  *out = g_scratch_ptr[dev];
  return BTX_OK;
}

bool shapes_ok(int T, int d, int f, int E, int k) {
  return T >= 0 && d > 0 && f > 0 && E >= 1 && E <= kMaxExperts && k >= 1 && k <= E && d % 8 == 0 && f % 8 == 0 &&
         (int64_t)T * k < (int64_t)1 << 31 && (int64_t)T * k * (int64_t)(d > f ? d : f) < (int64_t)1 << 40;
}
// valid shapes that the kernels' 32-bit offsets or grid limits cannot take
bool shapes_supported(int dtype, int T, int d, int f, int E, int k) { return ff_rows_supported(dtype, T * k, d, f, E); }

// The kernels move rows as 16-byte pieces: every tensor of rows must start on a 16-byte boundary (NULL passes:
// optional arguments), and with d, f multiples of 8 every row then does.
template <typename... P> bool aligned16(P... p) { return (((uintptr_t)p | ...) & 15) == 0; }

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

const char* btx_status_string(int status) {
  switch (status) {
    case BTX_OK: return "ok";
    case BTX_ERR_INVALID_ARG: return "invalid argument";
    case BTX_ERR_UNSUPPORTED: return "unsupported configuration";
    case BTX_ERR_WORKSPACE: return "workspace too small";
    case BTX_ERR_HIP: return "HIP launch error";
    default: return "unknown status";
  }
}

int btx_version(void) { return 1; }

int btx_profile_stages(void** events, int n_pairs) {
  if (n_pairs < 0 || (n_pairs > 0 && !events)) return BTX_ERR_INVALID_ARG;
  g_stage_events = n_pairs ? reinterpret_cast<hipEvent_t*>(events) : nullptr;
  g_stage_event_pairs = n_pairs;
  return BTX_OK;
}

size_t btx_moe_route_workspace_bytes(int T, int d, int E, int k) {
  if (T <= 0 || d <= 0 || E < 1 || E > kMaxExperts || k < 1 || k > E) return 0;
  return route_workspace_bytes(T, d, E, k);
}

namespace {
int route_impl(const void* x, int x_dtype, const float* gain, float eps, void* xn, float* rstd,
               const float* W_router, const float* b_router, const float* U, int T, int d, int E, int k,
               int route_mode, int lb_mode, float lb_alpha, float tau, float capacity_factor,
               int32_t* topk_idx, float* gates, float* probs, int32_t* counts, int32_t* offsets, int32_t* perm,
               int32_t* inv_pos, float* gate_sum, float* prob_sum, float* lb_loss, void* workspace,
               size_t workspace_bytes, void* stream) {
  if (!dtype_ok(x_dtype) || T < 0 || d <= 0 || d % 8 != 0 || E < 1 || E > kMaxExperts || k < 1 || k > E)
    return BTX_ERR_INVALID_ARG;
  if ((int64_t)T * k >= (int64_t)1 << 31) return BTX_ERR_INVALID_ARG;
  if (route_mode < BTX_ROUTE_TOPK_RENORM || route_mode > BTX_ROUTE_GUMBEL_TOP1) return BTX_ERR_INVALID_ARG;
  if (lb_mode != BTX_LB_TOKEN_FRAC && lb_mode != BTX_LB_GATE_MEAN) return BTX_ERR_INVALID_ARG;
  if (route_mode != BTX_ROUTE_TOPK_RENORM && k != 1) return BTX_ERR_INVALID_ARG;
  const bool needs_U = route_mode == BTX_ROUTE_SAMPLE_TOP1 || route_mode == BTX_ROUTE_GUMBEL_TOP1;
  if (needs_U != (U != nullptr)) return BTX_ERR_INVALID_ARG;
  if (route_mode == BTX_ROUTE_GUMBEL_TOP1 && !(tau > 0.f)) return BTX_ERR_INVALID_ARG;
  if (!(capacity_factor >= 0.f)) return BTX_ERR_INVALID_ARG;
  if (T == 0) return BTX_OK;
  if (!x || !W_router || !topk_idx || !gates || !probs || !counts || !offsets || !perm || !inv_pos || !gate_sum ||
      !prob_sum || !lb_loss || !workspace)
    return BTX_ERR_INVALID_ARG;
  if (!aligned16(x, xn, gain, workspace)) return BTX_ERR_INVALID_ARG;
  if (workspace_bytes < route_workspace_bytes(T, d, E, k)) return BTX_ERR_WORKSPACE;
  // capacity in double, as the specification of the limit is ceil(cf * T*k / E) over the reals
  const double cap_d = capacity_factor > 0.f ? std::ceil((double)capacity_factor * T * k / E) : 0.0;
  const int cap = cap_d > (double)T * k ? T * k : (int)cap_d;
  RouteArgs a{x, x_dtype, W_router, b_router, U, T, d, E, k, route_mode, lb_mode, lb_alpha, tau, cap, topk_idx, gates, probs,
              counts, offsets, perm, inv_pos, gate_sum, prob_sum, lb_loss, workspace, gain, eps, xn, rstd};
  hipStream_t s = static_cast<hipStream_t>(stream);
  BTX_STAGE(BTX_STAGE_ROUTE, launch_route(a, s));
  return BTX_OK;
}
}  // namespace

int btx_moe_route(const void* x, int x_dtype, const float* W_router, const float* b_router, const float* U, int T, int d,
                  int E, int k, int route_mode, int lb_mode, float lb_alpha, float tau, float capacity_factor,
                  int32_t* topk_idx, float* gates, float* probs, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_pos, float* gate_sum,
                  float* prob_sum, float* lb_loss, void* workspace, size_t workspace_bytes, void* stream) {
  return route_impl(x, x_dtype, nullptr, 0.f, nullptr, nullptr, W_router, b_router, U, T, d, E, k, route_mode, lb_mode,
                    lb_alpha, tau, capacity_factor, topk_idx, gates, probs, counts, offsets, perm, inv_pos, gate_sum,
                    prob_sum, lb_loss, workspace, workspace_bytes, stream);
}

int btx_init(void) {
  void* p = nullptr;
  if (int rc = static_scratch(&p)) return rc;   // also looks up this device's copy of the fixed workspace
  return ff_prepare();
}

size_t btx_moe_route_noalloc_max_workspace_bytes(void) { return kStaticRouteBytes; }

int btx_moe_route_noalloc(const void* x, int x_dtype, const float* W_router, const float* b_router, const float* U, int T,
                          int d, int E, int k, int route_mode, int lb_mode, float lb_alpha, float tau,
                          float capacity_factor, int32_t* topk_idx, float* gates, float* probs, int32_t* counts,
                          int32_t* offsets, int32_t* perm, int32_t* inv_pos, float* gate_sum, float* prob_sum,
                          float* lb_loss, void* stream) {
  // the size check comes first: a problem that does not fit is refused whatever else is wrong with it
  if (T > 0 && d > 0 && E >= 1 && E <= kMaxExperts && k >= 1 && k <= E &&
      route_workspace_bytes(T, d, E, k) > kStaticRouteBytes)
    return BTX_ERR_WORKSPACE;
  void* ws = nullptr;
  if (T > 0) {
    if (int rc = static_scratch(&ws)) return rc;
  }
  return route_impl(x, x_dtype, nullptr, 0.f, nullptr, nullptr, W_router, b_router, U, T, d, E, k, route_mode, lb_mode,
                    lb_alpha, tau, capacity_factor, topk_idx, gates, probs, counts, offsets, perm, inv_pos, gate_sum,
                    prob_sum, lb_loss, ws, kStaticRouteBytes, stream);
}


int btx_moe_norm_route(const void* h, int x_dtype, const float* gain, float eps, void* xn, float* rstd,
                       const float* W_router, const float* b_router, const float* U, int T, int d, int E, int k,
                       int route_mode, int lb_mode, float lb_alpha, float tau, float capacity_factor,
                       int32_t* topk_idx, float* gates, float* probs, int32_t* counts, int32_t* offsets, int32_t* perm,
                       int32_t* inv_pos, float* gate_sum, float* prob_sum, float* lb_loss, void* workspace,
                       size_t workspace_bytes, void* stream) {
  if (!(eps >= 0.f)) return BTX_ERR_INVALID_ARG;
  if (T > 0 && (!gain || !xn || !rstd || xn == h)) return BTX_ERR_INVALID_ARG;
  return route_impl(h, x_dtype, gain, eps, xn, rstd, W_router, b_router, U, T, d, E, k, route_mode, lb_mode, lb_alpha,
                    tau, capacity_factor, topk_idx, gates, probs, counts, offsets, perm, inv_pos, gate_sum, prob_sum,
                    lb_loss, workspace, workspace_bytes, stream);
}

size_t btx_rmsnorm_backward_workspace_bytes(int T, int d) {
  if (T <= 0 || d <= 0) return 0;
  return rmsnorm_bwd_workspace_bytes(T, d);
}

int btx_rmsnorm_backward(const void* dXn, const void* h, const float* gain, const float* rstd, const void* dres,
                         int dtype, int T, int d, void* dH, float* dgain, void* workspace, size_t workspace_bytes,
                         void* stream) {
  if (!dtype_ok(dtype) || T < 0 || d <= 0 || d % 8 != 0 || d > 16384) return BTX_ERR_INVALID_ARG;
  if (T == 0) return BTX_OK;
  if (!dXn || !h || !gain || !rstd || !dH || !dgain || !workspace) return BTX_ERR_INVALID_ARG;
  if (!aligned16(dXn, h, gain, dres, dH, dgain, workspace)) return BTX_ERR_INVALID_ARG;
  if (workspace_bytes < rmsnorm_bwd_workspace_bytes(T, d)) return BTX_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  BTX_STAGE(BTX_STAGE_NORM_BWD, launch_rmsnorm_bwd(dXn, h, gain, rstd, dres, dtype, T, d, dH, dgain, workspace, s));
  return BTX_OK;
}

size_t btx_moe_ff_forward_workspace_bytes(int T, int d, int f, int E, int k, int dtype) {
  if (!dtype_ok(dtype) || !shapes_ok(T, d, f, E, k) || T == 0) return 0;
  return carve_forward(nullptr, T, d, f, k, dtype, /*save=*/false).bytes;   // the larger of the two cases
}

int btx_moe_ff_forward(const void* x, const void* W1, const void* W3, const void* W2, int dtype,
                       int64_t w13_expert_stride, int64_t w2_expert_stride, int T, int d, int f, int E, int k,
                       const float* gates, const int32_t* offsets, const int32_t* perm, const int32_t* inv_pos,
                       const void* residual, void* out, void* save_h1, void* save_h3, void* workspace,
                       size_t workspace_bytes, void* stream) {
  if (!dtype_ok(dtype) || !shapes_ok(T, d, f, E, k)) return BTX_ERR_INVALID_ARG;
  if (w13_expert_stride < (int64_t)d * f || w2_expert_stride < (int64_t)d * f) return BTX_ERR_INVALID_ARG;
  if ((save_h1 == nullptr) != (save_h3 == nullptr)) return BTX_ERR_INVALID_ARG;
  if (T == 0) return BTX_OK;
  if (!shapes_supported(dtype, T, d, f, E, k)) return BTX_ERR_UNSUPPORTED;
  if (!x || !W1 || !W3 || !W2 || !gates || !offsets || !perm || !inv_pos || !out || !workspace)
    return BTX_ERR_INVALID_ARG;
  if (!aligned16(x, W1, W3, W2, residual, out, save_h1, save_h3, workspace) || w13_expert_stride % 8 || w2_expert_stride % 8)
    return BTX_ERR_INVALID_ARG;
  const FwdWs w = carve_forward(workspace, T, d, f, k, dtype, save_h1 != nullptr);
  if (workspace_bytes < w.bytes) return BTX_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int R = T * k;
  const FfShapes sh{R, d, f, E, w13_expert_stride, w2_expert_stride};
  void* h1 = save_h1 ? save_h1 : w.h1;
  void* h3 = save_h3 ? save_h3 : w.h3;
  const bool fused = ff_gather_fused(dtype, T, d, f);
  if (!fused) BTX_STAGE(BTX_STAGE_GATHER_X, launch_gather_rows(x, w.xs, perm, R, k, d, dtype, s));
  const RowSource xs = fused ? RowSource{x, perm, k} : RowSource{w.xs, nullptr, 1};
  BTX_STAGE(BTX_STAGE_UP, launch_up_swiglu(dtype, xs, W1, W3, offsets, sh, h1, h3, w.act, w.partial, s));
  BTX_STAGE(BTX_STAGE_DOWN, launch_down(dtype, w.act, W2, offsets, sh, w.y, w.partial, s));
  BTX_STAGE(BTX_STAGE_COMBINE, launch_combine(w.y, gates, inv_pos, residual, out, T, k, d, dtype, s));
  return BTX_OK;
}

size_t btx_moe_ff_backward_workspace_bytes(int T, int d, int f, int E, int k, int dtype) {
  if (!dtype_ok(dtype) || !shapes_ok(T, d, f, E, k) || T == 0) return 0;
  return carve_backward(nullptr, T, d, f, E, k, dtype).bytes;
}

int btx_moe_ff_backward(const void* dY, const void* x, const float* W_router, const void* W1, const void* W3,
                        const void* W2, int dtype, int64_t w13_expert_stride, int64_t w2_expert_stride, int T, int d,
                        int f, int E, int k, int route_mode, int lb_mode, float lb_alpha, float lb_grad_scale,
                        unsigned flags, const float* noise, float tau, const int32_t* topk_idx, const float* gates,
                        const float* probs,
                        const int32_t* offsets, const int32_t* perm, const int32_t* inv_pos, const float* gate_sum,
                        const float* prob_sum, const int32_t* counts, const void* save_h1, const void* save_h3, void* dX,
                        float* dW_router, float* db_router, void* dW1, void* dW3, void* dW2, int dW_dtype,
                        void* workspace, size_t workspace_bytes, void* stream) {
  if (!dtype_ok(dtype) || !dtype_ok(dW_dtype) || !shapes_ok(T, d, f, E, k)) return BTX_ERR_INVALID_ARG;
  if (dW_dtype != dtype && dW_dtype != BTX_F32) return BTX_ERR_INVALID_ARG;
  if (w13_expert_stride < (int64_t)d * f || w2_expert_stride < (int64_t)d * f) return BTX_ERR_INVALID_ARG;
  if (route_mode < BTX_ROUTE_TOPK_RENORM || route_mode > BTX_ROUTE_GUMBEL_TOP1) return BTX_ERR_INVALID_ARG;
  if (route_mode != BTX_ROUTE_TOPK_RENORM && k != 1) return BTX_ERR_INVALID_ARG;
  if ((route_mode == BTX_ROUTE_GUMBEL_TOP1) != (noise != nullptr)) return BTX_ERR_INVALID_ARG;
  if (route_mode == BTX_ROUTE_GUMBEL_TOP1 && !(tau > 0.f)) return BTX_ERR_INVALID_ARG;
  if (lb_mode != BTX_LB_TOKEN_FRAC && lb_mode != BTX_LB_GATE_MEAN) return BTX_ERR_INVALID_ARG;
  if (flags & ~BTX_FLAG_LB_GRAD_THROUGH_U) return BTX_ERR_INVALID_ARG;
  if ((flags & BTX_FLAG_LB_GRAD_THROUGH_U) && lb_mode != BTX_LB_GATE_MEAN) return BTX_ERR_INVALID_ARG;
  const int n_dw = (dW1 != nullptr) + (dW3 != nullptr) + (dW2 != nullptr);
  if (n_dw != 0 && n_dw != 3) return BTX_ERR_INVALID_ARG;
  if (T == 0) return BTX_OK;
  if (!shapes_supported(dtype, T, d, f, E, k)) return BTX_ERR_UNSUPPORTED;
  if (!dY || !x || !W_router || !W1 || !W3 || !W2 || !topk_idx || !gates || !probs || !offsets || !perm || !inv_pos ||
      !gate_sum || !prob_sum || !counts || !save_h1 || !save_h3 || !dX || !dW_router || !workspace)
    return BTX_ERR_INVALID_ARG;
  if (!aligned16(dY, x, W1, W3, W2, save_h1, save_h3, dX, dW1, dW3, dW2, workspace) || w13_expert_stride % 8 ||
      w2_expert_stride % 8)
    return BTX_ERR_INVALID_ARG;
  const BwdWs w = carve_backward(workspace, T, d, f, E, k, dtype);
  if (workspace_bytes < w.bytes) return BTX_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int R = T * k;
  const FfShapes sh{R, d, f, E, w13_expert_stride, w2_expert_stride};
  const bool fused = ff_gather_fused(dtype, T, d, f);
  if (!fused) BTX_STAGE(BTX_STAGE_GATHER_DY, launch_gather_rows(dY, w.dys, perm, R, k, d, dtype, s));
  const RowSource dys = fused ? RowSource{dY, perm, k} : RowSource{w.dys, nullptr, 1};
  BTX_STAGE(BTX_STAGE_BWD_ACT, launch_bwd_act(dtype, dys, W2, save_h1, save_h3, gates, perm, offsets, sh, w.dh1,
                                              w.dh3, w.ga, n_dw == 3, w.dg_part, w.scratch, s));
  BTX_STAGE(BTX_STAGE_BWD_DX, launch_bwd_dx(dtype, w.dh1, w.dh3, W1, W3, offsets, sh, w.dxs, w.partial, s));
  if (n_dw == 3) {
    const bool tr = ff_dw_transposed(dtype, d, f);
    auto gather_dw_operands = [&]() -> int {
      if (!tr) return launch_gather_rows(x, w.xs, perm, R, k, d, dtype, s);
      const int pitch = ff_dw_pitch(R, E);
      if (int rc = launch_gather_rows_t(x, w.xs, perm, offsets, R, k, d, E, pitch, s)) return rc;
      return launch_gather_rows_t(dY, w.dysT, perm, offsets, R, k, d, E, pitch, s);
    };
    BTX_STAGE(BTX_STAGE_GATHER_X_BWD, gather_dw_operands());
    BTX_STAGE(BTX_STAGE_DW13, launch_bwd_dw13(dtype, dW_dtype, w.xs, w.dh1, w.dh3, offsets, sh, dW1, dW3, s));
    BTX_STAGE(BTX_STAGE_DW2, launch_bwd_dw2(dtype, dW_dtype, w.ga, tr ? w.dysT : w.dys, offsets, sh, dW2, s));
  }
  RouterBwdArgs ra{x, dtype, W_router, T, d, E, k, route_mode, lb_mode, lb_alpha, lb_grad_scale, flags, noise, tau,
                   topk_idx, gates, probs, inv_pos, gate_sum, prob_sum, counts, w.dg_part, bwd_act_partials(dtype, d, f), w.dxs, dX,
                   dW_router, db_router, w.router};
  BTX_STAGE(BTX_STAGE_ROUTER_BWD, launch_router_bwd(ra, s));
  return BTX_OK;
}

int btx_merge_average(const void* const* inputs, int N, void* out, int64_t numel, int dtype, void* stream) {
  if (!dtype_ok(dtype) || N < 1 || N > 16 || numel < 0 || !inputs) return BTX_ERR_INVALID_ARG;
  if (numel == 0) return BTX_OK;
  if (!out || ((uintptr_t)out & 15)) return BTX_ERR_INVALID_ARG;
  for (int n = 0; n < N; ++n)
    if (!inputs[n] || ((uintptr_t)inputs[n] & 15)) return BTX_ERR_INVALID_ARG;
  return launch_merge_average(inputs, N, out, numel, dtype, static_cast<hipStream_t>(stream));
}

int btx_merge_weighted(const void* const* inputs, const float* weights, int N, void* out, int64_t numel, int dtype,
                       void* stream) {
  if (!dtype_ok(dtype) || N < 1 || N > 16 || numel < 0 || !inputs || !weights) return BTX_ERR_INVALID_ARG;
  for (int n = 0; n < N; ++n)
    if (!(weights[n] == weights[n]) || weights[n] > 3.0e38f || weights[n] < -3.0e38f) return BTX_ERR_INVALID_ARG;
  if (numel == 0) return BTX_OK;
  if (!out || ((uintptr_t)out & 15)) return BTX_ERR_INVALID_ARG;
  for (int n = 0; n < N; ++n)
    if (!inputs[n] || ((uintptr_t)inputs[n] & 15)) return BTX_ERR_INVALID_ARG;
  return launch_merge_weighted(inputs, weights, N, out, numel, dtype, static_cast<hipStream_t>(stream));
}

int btx_adamw_step(float* master, float* m, float* v, const void* grad, int grad_dtype, void* lowp, int64_t numel,
                   int step, float lr, float beta1, float beta2, float eps, float weight_decay, void* stream) {
  if (!dtype_ok(grad_dtype) || numel < 0 || step < 1) return BTX_ERR_INVALID_ARG;
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f)) return BTX_ERR_INVALID_ARG;
  if (numel == 0) return BTX_OK;
  if (!master || !m || !v || !grad) return BTX_ERR_INVALID_ARG;
  if ((((uintptr_t)master | (uintptr_t)m | (uintptr_t)v | (uintptr_t)grad) & 15) || ((uintptr_t)lowp & 7))
    return BTX_ERR_INVALID_ARG;
  return launch_adamw(master, m, v, grad, grad_dtype, lowp, numel, step, lr, beta1, beta2, eps, weight_decay,
                      static_cast<hipStream_t>(stream));
}

int btx_mix_experts(const void* W1, const void* W3, const void* W2, int dtype, int N, int d, int f, int mode, int C,
                    void* oW1, void* oW3, void* oW2, void* stream) {
  if (!dtype_ok(dtype) || N < 1 || d < 1 || f < 1) return BTX_ERR_INVALID_ARG;
  if (mode != BTX_MIX_SPLIT && mode != BTX_MIX_BLEND) return BTX_ERR_INVALID_ARG;
  const int chunks = mode == BTX_MIX_SPLIT ? C : N;
  if (chunks < 1 || f % chunks != 0) return BTX_ERR_INVALID_ARG;
  if (mode == BTX_MIX_SPLIT && (int64_t)N * C > kMaxExperts) return BTX_ERR_INVALID_ARG;
  if (!W1 || !W3 || !W2 || !oW1 || !oW3 || !oW2) return BTX_ERR_INVALID_ARG;
  if (W1 == oW1 || W3 == oW3 || W2 == oW2) return BTX_ERR_INVALID_ARG;   // not an in-place operation
  return launch_mix_experts(W1, W3, W2, dtype, N, d, f, mode, C, oW1, oW3, oW2, static_cast<hipStream_t>(stream));
}

#pragma GCC visibility pop
}  // extern "C"
