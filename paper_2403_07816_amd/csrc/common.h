// Shared device/host helpers of the gfx950 MoE feed-forward library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cmath>

#include "btx_moe.h"

namespace btx {

constexpr int kWave = 64;
constexpr int kMaxExperts = 64;

typedef uint16_t bf16_t;  // raw bfloat16 bits
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// Round to nearest even; inputs are finite by contract.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// Two floats -> packed bf16 pair, round to nearest even: one v_cvt_pk_bf16_f32 on gfx950.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const bf16x2_t r = __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t);
  return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// N consecutive elements of a row (N = 8; the address is N-element aligned) as floats
template <typename T, int N> struct RowVec;
template <> struct RowVec<bf16_t, 8> {
  static __device__ __forceinline__ void ld(const bf16_t* p, float* v) {
    const u32x4 w = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[2 * i] = bf16lo(w[i]); v[2 * i + 1] = bf16hi(w[i]); }
  }
  static __device__ __forceinline__ void st(bf16_t* p, const float* v) {
    *reinterpret_cast<u32x4*>(p) =
        u32x4{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
  }
  // the same, streamed past the caches (data that is read or written exactly once)
  static __device__ __forceinline__ void ld_stream(const bf16_t* p, float* v) {
    const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[2 * i] = bf16lo(w[i]); v[2 * i + 1] = bf16hi(w[i]); }
  }
  static __device__ __forceinline__ void st_stream(bf16_t* p, const float* v) {
    __builtin_nontemporal_store(
        u32x4{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])},
        reinterpret_cast<u32x4*>(p));
  }
};
template <> struct RowVec<float, 8> {
  static __device__ __forceinline__ void ld(const float* p, float* v) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
  }
  static __device__ __forceinline__ void st(float* p, const float* v) {
    *reinterpret_cast<f32x4*>(p) = f32x4{v[0], v[1], v[2], v[3]};
    *reinterpret_cast<f32x4*>(p + 4) = f32x4{v[4], v[5], v[6], v[7]};
  }
  static __device__ __forceinline__ void ld_stream(const float* p, float* v) {
    const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p + 4));
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
  }
  static __device__ __forceinline__ void st_stream(float* p, const float* v) {
    __builtin_nontemporal_store(f32x4{v[0], v[1], v[2], v[3]}, reinterpret_cast<f32x4*>(p));
    __builtin_nontemporal_store(f32x4{v[4], v[5], v[6], v[7]}, reinterpret_cast<f32x4*>(p + 4));
  }
};

// sigmoid via the hardware exp2 and reciprocal (about 1 ulp each): far inside the fp32 bar
__device__ __forceinline__ float sigmoid_f(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }
__device__ __forceinline__ float silu_f(float z) { return z * sigmoid_f(z); }

// Wavefront reductions without LDS traffic: four DPP steps (lane xor 1, xor 2, then rotations
// by 4 and 8 inside each row of 16 lanes) leave every lane with its row's result; the four row
// results are fetched with v_readlane and combined.  All 64 lanes must be active.  A butterfly
// of ds_bpermute shuffles costs an LDS round trip per step; the router kernels spend most of
// their instructions in such reductions.
template <int CTRL> __device__ __forceinline__ int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
template <int CTRL> __device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(dpp_i32<CTRL>(__float_as_int(v)));
}
constexpr int kDppXor1 = 0xB1;    // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;    // quad_perm [2,3,0,1]
constexpr int kDppRor4 = 0x124;   // row_ror:4
constexpr int kDppRor8 = 0x128;   // row_ror:8
__device__ __forceinline__ float lane_f32(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
// sum of part[r * ld + i] over r = first, first + step, ... < n: four independent chains so that
// the loads overlap, combined in a fixed order (the result depends on first, step and n only)
__device__ __forceinline__ float strided_row_sum(const float* __restrict__ part, size_t ld, size_t i, int first, int step,
                                                 int n) {
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  int r = first;
  for (; r + 3 * step < n; r += 4 * step) {
    a0 += part[(size_t)r * ld + i];
    a1 += part[(size_t)(r + step) * ld + i];
    a2 += part[(size_t)(r + 2 * step) * ld + i];
    a3 += part[(size_t)(r + 3 * step) * ld + i];
  }
  for (; r < n; r += step) a0 += part[(size_t)r * ld + i];
  return (a0 + a1) + (a2 + a3);
}

// fp64 -> bf16 with one rounding: through fp32 first would round twice, which only matters when
// the fp32 value is an exact bf16 tie; the sign of what the first rounding dropped settles it.
__device__ __forceinline__ bf16_t f64_to_bf16(double v) {
  const float q = (float)v;
  uint32_t u = __float_as_uint(q);
  if ((u & 0xffffu) == 0x8000u) {
    const double r = v - (double)q;
    if (r != 0.0) {
      const bool up = (r > 0.0) == (q > 0.f);
      return (bf16_t)((u >> 16) + (up ? 1u : 0u));
    }
  }
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<kDppXor1>(v);
  v += dpp_f32<kDppXor2>(v);
  v += dpp_f32<kDppRor4>(v);
  v += dpp_f32<kDppRor8>(v);
  return (lane_f32(v, 0) + lane_f32(v, 16)) + (lane_f32(v, 32) + lane_f32(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f32<kDppXor1>(v));
  v = fmaxf(v, dpp_f32<kDppXor2>(v));
  v = fmaxf(v, dpp_f32<kDppRor4>(v));
  v = fmaxf(v, dpp_f32<kDppRor8>(v));
  return fmaxf(fmaxf(lane_f32(v, 0), lane_f32(v, 16)), fmaxf(lane_f32(v, 32), lane_f32(v, 48)));
}

// Inclusive prefix sum over the 64 lanes of a wavefront (all lanes active): four DPP shifts inside
// each row of 16 lanes, then the row totals (lanes 15, 31, 47) are added to the rows behind them.
constexpr int kDppShr1 = 0x111, kDppShr2 = 0x112, kDppShr4 = 0x114, kDppShr8 = 0x118;   // row_shr:n, zeros shifted in
__device__ __forceinline__ int wave_incl_scan_i32(int v, int lane) {
  v += dpp_i32<kDppShr1>(v);
  v += dpp_i32<kDppShr2>(v);
  v += dpp_i32<kDppShr4>(v);
  v += dpp_i32<kDppShr8>(v);
  const int t0 = __builtin_amdgcn_readlane(v, 15), t1 = __builtin_amdgcn_readlane(v, 31),
            t2 = __builtin_amdgcn_readlane(v, 47);
  const int row = lane >> 4;
  return v + (row == 0 ? 0 : row == 1 ? t0 : row == 2 ? t0 + t1 : t0 + t1 + t2);
}

// Which expert owns grouped row-tile `tile` when every expert's rows are cut
// into tiles of BM rows, experts laid one after another.  Returns false past
// the last tile.  offsets has E+1 entries.
__device__ __forceinline__ bool find_row_tile(const int32_t* __restrict__ offsets, int E, int BM, int tile,
                                               int& expert, int& row0, int& row_end) {
  int t = tile;
  for (int e = 0; e < E; ++e) {
    const int b = offsets[e], n = offsets[e + 1] - b;
    const int nt = (n + BM - 1) / BM;
    if (t < nt) {
      expert = e;
      row0 = b + t * BM;
      row_end = b + n;
      return true;
    }
    t -= nt;
  }
  return false;
}

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

#define BTX_LAUNCH_CHECK()                                   \
  do {                                                       \
    if (hipGetLastError() != hipSuccess) return BTX_ERR_HIP; \
  } while (0)

// ---- internal launchers (one translation unit each) ------------------------
struct RouteArgs {
  const void* x; int x_dtype; const float* W_router; const float* b_router; const float* U;
  int T, d, E, k, route_mode, lb_mode; float lb_alpha, tau; int cap;   // cap: rows an expert keeps (0 = all)
  int32_t* topk_idx; float* gates; float* probs; int32_t* counts; int32_t* offsets; int32_t* perm;
  int32_t* inv_pos; float* gate_sum; float* prob_sum; float* lb_loss;
  void* workspace;
  // optional RMS normalisation of the rows in front of the router (gain NULL: none): x is then
  // the raw row, xn [T,d] (x's dtype) receives gain * x * rstd and rstd [T] the row factors
  const float* gain; float eps; void* xn; float* rstd;
};
size_t route_workspace_bytes(int T, int d, int E, int k);
// backward of the normalisation: dH = d(xn)/d(h)^T dXn (+ dres), dgain[c] = sum_t dXn[t,c] h[t,c] rstd[t]
size_t rmsnorm_bwd_workspace_bytes(int T, int d);
int launch_rmsnorm_bwd(const void* dXn, const void* h, const float* gain, const float* rstd, const void* dres,
                       int dtype, int T, int d, void* dH, float* dgain, void* workspace, hipStream_t s);
int launch_route(const RouteArgs& a, hipStream_t s);
// WrT[e][c] = Wr[c][e]: the router kernels read W_router expert-major
int launch_transpose_wr(const float* Wr, int d, int E, float* WrT, hipStream_t s);

// rows: dst[r] = src[perm[r] / k]  (k = 1 with perm = NULL copies nothing; perm required)
int launch_gather_rows(const void* src, void* dst, const int32_t* perm, int R, int k, int d, int dtype, hipStream_t s);
// bf16 only: dst[c][P_e + i] = src[perm[o_e + i] / k][c], every expert's rows padded with zeros to a
// multiple of 64 (P_e = padded rows of the experts before e); dst is [d][pitch]
int launch_gather_rows_t(const void* src, void* dst, const int32_t* perm, const int32_t* offsets, int R, int k, int d,
                         int E, int pitch, hipStream_t s);
// out[t] = sum_j gates[t,j] * y[inv_pos[t,j]]   (gates NULL => unit weights; inv_pos < 0: dropped pair, skipped)
// residual (may be NULL): [T,d] added to the sum in fp32 before the one rounding
int launch_combine(const void* y, const float* gates, const int32_t* inv_pos, const void* residual, void* out, int T,
                   int k, int d, int dtype, hipStream_t s);

// Expert GEMM stages.  `offsets` = E+1 grouped-row offsets on the device.
struct FfShapes { int R, d, f, E; int64_t s13, s2; };
// Grouped rows of a [.., d] operand: row r is row perm[r] / k of `base`, or simply row r of
// `base` when perm is NULL (rows already gathered).  ff_gather_fused() says whether the
// stages of a problem read token rows through perm themselves.
struct RowSource { const void* base; const int32_t* perm; int k; };
bool ff_gather_fused(int dtype, int T, int d, int f);
// a = silu(xs W1) * (xs W3); h1/h3 stored when non-null.  They may be null only when
// ff_up_needs_h() is false: the plain path computes act from the stored h1/h3.
bool ff_up_needs_h(int dtype, int d, int f);
int launch_up_swiglu(int dtype, const RowSource& xs, const void* W1, const void* W3, const int32_t* offsets,
                     const FfShapes& sh, void* h1, void* h3, void* act, void* partial, hipStream_t s);
// partial (here, in launch_down and in launch_bwd_dx): ff_split_bytes() of scratch (the bf16 MFMA path cuts the
// tiles of a partly filled last round along K and adds the slices in a second kernel); may be NULL when
// ff_split_bytes() is 0.  Products that follow each other on a stream may share it.
size_t ff_split_bytes(int dtype, int d, int f);
// y = act W2
int launch_down(int dtype, const void* act, const void* W2, const int32_t* offsets, const FfShapes& sh, void* y,
                void* partial, hipStream_t s);
// D = dys W2^T; dg_part[r,p] partial sums of D*a; da = g*D; dh1 = da*h3*silu'(h1); dh3 = da*silu(h1); ga = g*a.
// dh1, dh3: [R,f].  When ff_dw_transposed() holds, `ga` receives g*a transposed and padded
// ([f][ff_dw_pitch()]), or nothing at all when want_dw is false; otherwise ga is [R,f].
// bwd_act_partials: partial sums per grouped row that launch_bwd_act writes for these shapes (one per 256-column
// tile on the bf16 MFMA path, a single sum otherwise)
int bwd_act_partials(int dtype, int d, int f);
int launch_bwd_act(int dtype, const RowSource& dys, const void* W2, const void* h1, const void* h3, const float* gates,
                   const int32_t* perm, const int32_t* offsets, const FfShapes& sh, void* dh1, void* dh3, void* ga,
                   bool want_dw, float* dg_part, void* scratch, hipStream_t s);
// dxs = dh1 W1^T + dh3 W3^T
int launch_bwd_dx(int dtype, const void* dh1, const void* dh3, const void* W1, const void* W3, const int32_t* offsets,
                  const FfShapes& sh, void* dxs, void* partial, hipStream_t s);
// dW1 = xs^T dh1, dW3 = xs^T dh3, dW2 = ga^T dys, per expert over its rows.  When
// ff_dw_transposed() holds, xs, dys and ga are passed in the transposed, padded form with
// pitch ff_dw_pitch() (xs and dys as launch_gather_rows_t writes them, ga as launch_bwd_act
// does); otherwise as grouped rows.
bool ff_dw_transposed(int dtype, int d, int f);
int ff_dw_pitch(int R, int E);
int launch_bwd_dw13(int dtype, int dW_dtype, const void* xs, const void* dh1, const void* dh3, const int32_t* offsets,
                    const FfShapes& sh, void* dW1, void* dW3, hipStream_t s);
int launch_bwd_dw2(int dtype, int dW_dtype, const void* ga, const void* dys, const int32_t* offsets, const FfShapes& sh,
                   void* dW2, hipStream_t s);
size_t ff_scratch_bytes(int dtype, int R, int f);
// one-time set-up of the expert GEMM kernels on the current device (everything that may not run inside a stream capture)
int ff_prepare();
// false when R routed rows are more than the kernels of this dtype and shape can address
bool ff_rows_supported(int dtype, int R, int d, int f, int E);

struct RouterBwdArgs {
  const void* x; int dtype; const float* W_router; int T, d, E, k, route_mode, lb_mode; float lb_alpha, lb_grad_scale;
  unsigned flags; const float* noise; float tau; const int32_t* topk_idx; const float* gates; const float* probs; const int32_t* inv_pos;
  const float* gate_sum; const float* prob_sum; const int32_t* counts; const float* dg_part; int n_part;
  const void* dxs; void* dX; float* dW_router; float* db_router; void* workspace;
};
size_t router_bwd_workspace_bytes(int T, int d, int E);
int launch_router_bwd(const RouterBwdArgs& a, hipStream_t s);

int launch_mix_experts(const void* W1, const void* W3, const void* W2, int dtype, int N, int d, int f, int mode, int C,
                       void* oW1, void* oW3, void* oW2, hipStream_t s);
int launch_adamw(float* P, float* M, float* V, const void* G, int grad_dtype, void* lowp, int64_t n, int step, float lr,
                 float beta1, float beta2, float eps, float wd, hipStream_t s);
int launch_merge_average(const void* const* inputs, int N, void* out, int64_t numel, int dtype, hipStream_t s);
int launch_merge_weighted(const void* const* inputs, const float* weights, int N, void* out, int64_t numel, int dtype,
                          hipStream_t s);

}  // namespace btx
