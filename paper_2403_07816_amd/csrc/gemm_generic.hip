// Plain LDS-tiled FMA grouped GEMM (no matrix cores) and the elementwise kernels that go
// with it.  This is the fp32 parity path of the expert FFNs (SwiGLU feed-forward of the
// seed model, Sec. 4.1, inside the layer equation of Sec. 3.2) and of their backward.
// It accepts any element type for storage and always computes in fp32; it is not the
// fast path (the bf16 MFMA kernels are).
#include <algorithm>
#include "common.h"
#include "gemm_generic.h"

namespace btx {
namespace {

constexpr int BT = 64;  // output tile edge
constexpr int BK = 16;

enum { GROUP_M = 0, GROUP_K = 1 };

struct GArgs {
  const void* A; const void* B; void* C;
  int64_t sam, sak, sbk, sbn, ldc;
  int M, N, K;
  const int32_t* offsets; int E;
  int64_t strideB_e, strideC_e;
  int group_mode, accumulate;
};

template <typename TA, typename TB, typename TC>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GArgs g) {
  __shared__ float As[BK][BT + 4];
  __shared__ float Bs[BK][BT + 4];
  const TA* A = static_cast<const TA*>(g.A);
  const TB* B = static_cast<const TB*>(g.B);
  TC* C = static_cast<TC*>(g.C);
  int m0, m_end, k0, k_end;
  if (g.group_mode == GROUP_M) {
    int e;
    if (!find_row_tile(g.offsets, g.E, BT, blockIdx.y, e, m0, m_end)) return;
    B += e * g.strideB_e;
    k0 = 0;
    k_end = g.K;
  } else {
    const int e = blockIdx.z;
    m0 = blockIdx.y * BT;
    m_end = g.M;
    k0 = g.offsets[e];
    k_end = g.offsets[e + 1];
    C += e * g.strideC_e;
  }
  const int n0 = blockIdx.x * BT;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int kk = k0; kk < k_end; kk += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = threadIdx.x + i * 256;  // 0..1023
      {
        const int k = idx % BK, m = idx / BK;
        const int gm = m0 + m, gk = kk + k;
        As[k][m] = (gm < m_end && gk < k_end) ? Elem<TA>::ld(A + gm * g.sam + gk * g.sak) : 0.f;
      }
      {
        const int n = idx % BT, k = idx / BT;
        const int gn = n0 + n, gk = kk + k;
        Bs[k][n] = (gn < g.N && gk < k_end) ? Elem<TB>::ld(B + gk * g.sbk + gn * g.sbn) : 0.f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= m_end) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= g.N) continue;
      TC* p = C + gm * g.ldc + gn;
      float v = acc[i][j];
      if (g.accumulate) v += Elem<TC>::ld(p);
      Elem<TC>::st(p, v);
    }
  }
}

template <typename TA, typename TB, typename TC>
int run(const GArgs& g, int R, hipStream_t s) {
  dim3 grid;
  if (g.group_mode == GROUP_M) grid = dim3(ceil_div(g.N, BT), ceil_div(R, BT) + g.E, 1);
  else grid = dim3(ceil_div(g.N, BT), ceil_div(g.M, BT), g.E);
  gemm_generic_kernel<TA, TB, TC><<<grid, 256, 0, s>>>(g);
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

template <typename ET>
__global__ __launch_bounds__(256) void swiglu_kernel(const ET* __restrict__ h1, const ET* __restrict__ h3,
                                                     ET* __restrict__ act, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    Elem<ET>::st(act + i, silu_f(Elem<ET>::ld(h1 + i)) * Elem<ET>::ld(h3 + i));
}

// One wavefront per grouped row.
template <typename ET>
__global__ __launch_bounds__(256) void bwd_act_kernel(const float* __restrict__ D, const ET* __restrict__ h1,
                                                      const ET* __restrict__ h3, const float* __restrict__ gates,
                                                      const int32_t* __restrict__ perm, int R, int f,
                                                      ET* __restrict__ dh1, ET* __restrict__ dh3, ET* __restrict__ ga,
                                                      float* __restrict__ dg_part) {
  const int lane = threadIdx.x & (kWave - 1);
  const int r = blockIdx.x * 4 + threadIdx.x / kWave;
  if (r >= R) return;
  const float g = gates[perm[r]];
  float dot = 0.f;
  for (int c = lane; c < f; c += kWave) {
    const size_t i = (size_t)r * f + c;
    const float z = Elem<ET>::ld(h1 + i), v3 = Elem<ET>::ld(h3 + i), dd = D[i];
    const float sg = sigmoid_f(z), sl = z * sg;
    const float a = sl * v3;
    dot = fmaf(dd, a, dot);
    const float da = g * dd;
    Elem<ET>::st(dh1 + i, da * v3 * (sg * (1.f + z * (1.f - sg))));
    Elem<ET>::st(dh3 + i, da * sl);
    Elem<ET>::st(ga + i, g * a);
  }
  dot = wave_sum(dot);
  if (lane == 0) dg_part[r] = dot;
}

template <typename ET>
struct Generic {
  static int up(const void* xs, const void* W1, const void* W3, const int32_t* off, const FfShapes& sh, void* h1,
                void* h3, void* act, hipStream_t s) {
    GArgs g{};
    g.A = xs; g.sam = sh.d; g.sak = 1; g.sbk = sh.f; g.sbn = 1; g.ldc = sh.f; g.N = sh.f; g.K = sh.d;
    g.offsets = off; g.E = sh.E; g.strideB_e = sh.s13; g.group_mode = GROUP_M;
    g.B = W1; g.C = h1;
    if (int rc = run<ET, ET, ET>(g, sh.R, s)) return rc;
    g.B = W3; g.C = h3;
    if (int rc = run<ET, ET, ET>(g, sh.R, s)) return rc;
    const size_t n = (size_t)sh.R * sh.f;
    swiglu_kernel<ET><<<(unsigned)std::min<size_t>((n + 255) / 256, 65535), 256, 0, s>>>(
        static_cast<const ET*>(h1), static_cast<const ET*>(h3), static_cast<ET*>(act), n);
    BTX_LAUNCH_CHECK();
    return BTX_OK;
  }
  static int down(const void* act, const void* W2, const int32_t* off, const FfShapes& sh, void* y, hipStream_t s) {
    GArgs g{};
    g.A = act; g.sam = sh.f; g.sak = 1; g.B = W2; g.sbk = sh.d; g.sbn = 1; g.C = y; g.ldc = sh.d; g.N = sh.d;
    g.K = sh.f; g.offsets = off; g.E = sh.E; g.strideB_e = sh.s2; g.group_mode = GROUP_M;
    return run<ET, ET, ET>(g, sh.R, s);
  }
  static int bwd_act(const void* dys, const void* W2, const void* h1, const void* h3, const float* gates,
                     const int32_t* perm, const int32_t* off, const FfShapes& sh, void* dh1, void* dh3, void* ga,
                     float* dg_part, void* scratch, hipStream_t s) {
    GArgs g{};  // D[r,c] = sum_m dys[r,m] W2[c,m]
    g.A = dys; g.sam = sh.d; g.sak = 1; g.B = W2; g.sbk = 1; g.sbn = sh.d; g.C = scratch; g.ldc = sh.f; g.N = sh.f;
    g.K = sh.d; g.offsets = off; g.E = sh.E; g.strideB_e = sh.s2; g.group_mode = GROUP_M;
    if (int rc = run<ET, ET, float>(g, sh.R, s)) return rc;
    bwd_act_kernel<ET><<<ceil_div(sh.R, 4), 256, 0, s>>>(
        static_cast<const float*>(scratch), static_cast<const ET*>(h1), static_cast<const ET*>(h3), gates, perm, sh.R,
        sh.f, static_cast<ET*>(dh1), static_cast<ET*>(dh3), static_cast<ET*>(ga), dg_part);
    BTX_LAUNCH_CHECK();
    return BTX_OK;
  }
  static int bwd_dx(const void* dh1, const void* dh3, const void* W1, const void* W3, const int32_t* off,
                    const FfShapes& sh, void* dxs, hipStream_t s) {
    GArgs g{};  // dxs[r,m] = sum_c dh1[r,c] W1[m,c] + dh3[r,c] W3[m,c]
    g.A = dh1; g.sam = sh.f; g.sak = 1; g.B = W1; g.sbk = 1; g.sbn = sh.f; g.C = dxs; g.ldc = sh.d; g.N = sh.d;
    g.K = sh.f; g.offsets = off; g.E = sh.E; g.strideB_e = sh.s13; g.group_mode = GROUP_M;
    if (int rc = run<ET, ET, ET>(g, sh.R, s)) return rc;
    // second product accumulated in fp32 on top of the stored first one would round
    // twice for bf16 storage; the fp32 path has no such rounding and this path is the
    // fp32 one.  (The bf16 MFMA kernel keeps one accumulator for both products.)
    g.A = dh3; g.B = W3; g.accumulate = 1;
    return run<ET, ET, ET>(g, sh.R, s);
  }
  template <typename WT>
  static int bwd_dw13(const void* xs, const void* dh1, const void* dh3, const int32_t* off, const FfShapes& sh,
                      void* dW1, void* dW3, hipStream_t s) {
    GArgs g{};  // dW1[m,c] = sum_r xs[r,m] dh1[r,c]
    g.A = xs; g.sam = 1; g.sak = sh.d; g.B = dh1; g.sbk = sh.f; g.sbn = 1; g.C = dW1; g.ldc = sh.f; g.M = sh.d;
    g.N = sh.f; g.offsets = off; g.E = sh.E; g.strideC_e = sh.s13; g.group_mode = GROUP_K;
    if (int rc = run<ET, ET, WT>(g, sh.R, s)) return rc;
    g.B = dh3; g.C = dW3;
    return run<ET, ET, WT>(g, sh.R, s);
  }
  template <typename WT>
  static int bwd_dw2(const void* ga, const void* dys, const int32_t* off, const FfShapes& sh, void* dW2,
                     hipStream_t s) {
    GArgs g{};  // dW2[c,m] = sum_r ga[r,c] dys[r,m]
    g.A = ga; g.sam = 1; g.sak = sh.f; g.B = dys; g.sbk = sh.d; g.sbn = 1; g.C = dW2; g.ldc = sh.d; g.M = sh.f;
    g.N = sh.d; g.offsets = off; g.E = sh.E; g.strideC_e = sh.s2; g.group_mode = GROUP_K;
    return run<ET, ET, WT>(g, sh.R, s);
  }
};

}  // namespace

bool generic_rows_ok(int R, int E) { return ceil_div(R, BT) + E <= 65535; }

int generic_up_swiglu(int dtype, const void* xs, const void* W1, const void* W3, const int32_t* off, const FfShapes& sh,
                      void* h1, void* h3, void* act, hipStream_t s) {
  return dtype == BTX_BF16 ? Generic<bf16_t>::up(xs, W1, W3, off, sh, h1, h3, act, s)
                           : Generic<float>::up(xs, W1, W3, off, sh, h1, h3, act, s);
}
int generic_down(int dtype, const void* act, const void* W2, const int32_t* off, const FfShapes& sh, void* y,
                 hipStream_t s) {
  return dtype == BTX_BF16 ? Generic<bf16_t>::down(act, W2, off, sh, y, s) : Generic<float>::down(act, W2, off, sh, y, s);
}
int generic_bwd_act(int dtype, const void* dys, const void* W2, const void* h1, const void* h3, const float* gates,
                    const int32_t* perm, const int32_t* off, const FfShapes& sh, void* dh1, void* dh3, void* ga,
                    float* dg_part, void* scratch, hipStream_t s) {
  return dtype == BTX_BF16
             ? Generic<bf16_t>::bwd_act(dys, W2, h1, h3, gates, perm, off, sh, dh1, dh3, ga, dg_part, scratch, s)
             : Generic<float>::bwd_act(dys, W2, h1, h3, gates, perm, off, sh, dh1, dh3, ga, dg_part, scratch, s);
}
int generic_bwd_dx(int dtype, const void* dh1, const void* dh3, const void* W1, const void* W3, const int32_t* off,
                   const FfShapes& sh, void* dxs, hipStream_t s) {
  return dtype == BTX_BF16 ? Generic<bf16_t>::bwd_dx(dh1, dh3, W1, W3, off, sh, dxs, s)
                           : Generic<float>::bwd_dx(dh1, dh3, W1, W3, off, sh, dxs, s);
}
int generic_bwd_dw13(int dtype, int dW_dtype, const void* xs, const void* dh1, const void* dh3, const int32_t* off,
                     const FfShapes& sh, void* dW1, void* dW3, hipStream_t s) {
  if (dtype == BTX_BF16) {
    return dW_dtype == BTX_BF16 ? Generic<bf16_t>::bwd_dw13<bf16_t>(xs, dh1, dh3, off, sh, dW1, dW3, s)
                                : Generic<bf16_t>::bwd_dw13<float>(xs, dh1, dh3, off, sh, dW1, dW3, s);
  }
  return Generic<float>::bwd_dw13<float>(xs, dh1, dh3, off, sh, dW1, dW3, s);
}
int generic_bwd_dw2(int dtype, int dW_dtype, const void* ga, const void* dys, const int32_t* off, const FfShapes& sh,
                    void* dW2, hipStream_t s) {
  if (dtype == BTX_BF16) {
    return dW_dtype == BTX_BF16 ? Generic<bf16_t>::bwd_dw2<bf16_t>(ga, dys, off, sh, dW2, s)
                                : Generic<bf16_t>::bwd_dw2<float>(ga, dys, off, sh, dW2, s);
  }
  return Generic<float>::bwd_dw2<float>(ga, dys, off, sh, dW2, s);
}

}  // namespace btx
