// Backward of the RMS normalisation that sits in front of the feed-forward sublayer in the seed
// model's blocks (Sec. 4.1; the forward is folded into the router's read of the rows).
// With xn = gain * h * rstd, rstd = 1/sqrt(mean(h^2) + eps):
//   dH[t]    = rstd[t] * gain * dXn[t] - h[t] * rstd[t]^3 * (sum_c gain_c dXn[t,c] h[t,c]) / d   (+ dres[t])
//   dgain[c] = sum_t dXn[t,c] * h[t,c] * rstd[t]
// HBM-bound: dXn and h are streamed (the second pass over a row hits the cache), dH is written
// once.  A workgroup owns kNormTok consecutive tokens and all d columns, 4 tokens in flight; the
// row sums are reduced through LDS in a fixed order, the column sums leave as one partial row
// per workgroup and a second kernel adds those in a fixed order: no atomics.
#include "common.h"

namespace btx {
namespace {

constexpr int kNormTok = 16;     // tokens per workgroup
constexpr int kNormThreads = 256;

// MAXC: 8-column chunks a thread owns (d <= MAXC * 2048); its column sums stay in registers
template <typename XT, int MAXC>
// dH may be the same buffer as dXn or dres (every thread writes only the chunks it has read, and a
// row is written after its row sum is complete): those three carry no __restrict__.
__global__ __launch_bounds__(kNormThreads) void rmsnorm_bwd_kernel(const XT* dXn, const XT* __restrict__ h,
                                                                   const float* __restrict__ gain,
                                                                   const float* __restrict__ rstd, const XT* dres, int T,
                                                                   int d, XT* dH, float* __restrict__ part) {
  __shared__ float s_part[kNormThreads / kWave][4];
  __shared__ float s_coef[4];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int t0 = blockIdx.x * kNormTok;
  float gacc[MAXC][8] = {};
  for (int tq = 0; tq < kNormTok && t0 + tq < T; tq += 4) {
    // ---- pass 1: S[q] = sum_c gain_c dXn[t,c] h[t,c]
    float sq[4] = {};
#pragma unroll
    for (int m = 0; m < MAXC; ++m) {
      const int c0 = (m * kNormThreads + threadIdx.x) * 8;
      if (c0 < d) {
        float gv[8];
        RowVec<float, 8>::ld(gain + c0, gv);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const size_t row = (size_t)min(t0 + tq + q, T - 1) * d + c0;   // clamped rows are computed and dropped
          float a[8], b[8];
          RowVec<XT, 8>::ld(dXn + row, a);
          RowVec<XT, 8>::ld(h + row, b);
#pragma unroll
          for (int i = 0; i < 8; ++i) sq[q] = fmaf(gv[i] * a[i], b[i], sq[q]);
        }
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float s = wave_sum(sq[q]);
      if (lane == 0) s_part[wave][q] = s;
    }
    __syncthreads();
    if (threadIdx.x < 4) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < kNormThreads / kWave; ++w) s += s_part[w][threadIdx.x];
      const float r = rstd[min(t0 + tq + (int)threadIdx.x, T - 1)];
      s_coef[threadIdx.x] = r * r * r * s / (float)d;
    }
    __syncthreads();
    // ---- pass 2: dH and the column sums
#pragma unroll
    for (int m = 0; m < MAXC; ++m) {
      const int c0 = (m * kNormThreads + threadIdx.x) * 8;
      if (c0 < d) {
        float gv[8];
        RowVec<float, 8>::ld(gain + c0, gv);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int t = t0 + tq + q;
          if (t < T) {
            const size_t row = (size_t)t * d + c0;
            const float r = rstd[t], coef = s_coef[q];
            float a[8], b[8], o[8];
            RowVec<XT, 8>::ld(dXn + row, a);
            RowVec<XT, 8>::ld(h + row, b);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              o[i] = r * gv[i] * a[i] - b[i] * coef;
              gacc[m][i] = fmaf(a[i] * b[i], r, gacc[m][i]);
            }
            if (dres) {
              float e[8];
              RowVec<XT, 8>::ld(dres + row, e);
#pragma unroll
              for (int i = 0; i < 8; ++i) o[i] += e[i];
            }
            RowVec<XT, 8>::st(dH + row, o);
          }
        }
      }
    }
    __syncthreads();   // s_part / s_coef are reused by the next four tokens
  }
#pragma unroll
  for (int m = 0; m < MAXC; ++m) {
    const int c0 = (m * kNormThreads + threadIdx.x) * 8;
    if (c0 < d) RowVec<float, 8>::st(part + (size_t)blockIdx.x * d + c0, gacc[m]);
  }
}

// 64 columns per block; 16 thread groups each add every 16th partial row, then the 16 sums are
// added in group order
constexpr int kRedGroups = 16;
__global__ __launch_bounds__(64 * kRedGroups) void rmsnorm_dgain_reduce_kernel(const float* __restrict__ part, int nblk,
                                                                                int d, float* __restrict__ dgain) {
  __shared__ float s_sum[kRedGroups][64];
  const int o = threadIdx.x % 64, grp = threadIdx.x / 64;
  const int c = blockIdx.x * 64 + o;
  s_sum[grp][o] = c < d ? strided_row_sum(part, d, c, grp, kRedGroups, nblk) : 0.f;
  __syncthreads();
  if (grp == 0 && c < d) {
    float a = 0.f;
#pragma unroll
    for (int g = 0; g < kRedGroups; ++g) a += s_sum[g][o];
    dgain[c] = a;
  }
}

template <typename XT>
int launch_typed(const void* dXn, const void* h, const float* gain, const float* rstd, const void* dres, int T, int d,
                 void* dH, float* part, hipStream_t s) {
  const int nblk = ceil_div(T, kNormTok);
#define BTX_NORM_LAUNCH(MAXC)                                                                                      \
  rmsnorm_bwd_kernel<XT, MAXC><<<nblk, kNormThreads, 0, s>>>(static_cast<const XT*>(dXn), static_cast<const XT*>(h), \
                                                             gain, rstd, static_cast<const XT*>(dres), T, d,         \
                                                             static_cast<XT*>(dH), part)
  if (d <= 2048) BTX_NORM_LAUNCH(1);
  else if (d <= 4096) BTX_NORM_LAUNCH(2);
  else if (d <= 8192) BTX_NORM_LAUNCH(4);
  else if (d <= 16384) BTX_NORM_LAUNCH(8);
  else return BTX_ERR_UNSUPPORTED;
#undef BTX_NORM_LAUNCH
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

}  // namespace

size_t rmsnorm_bwd_workspace_bytes(int T, int d) {
  return align_up((size_t)ceil_div(T, kNormTok) * d * sizeof(float), 256);
}

int launch_rmsnorm_bwd(const void* dXn, const void* h, const float* gain, const float* rstd, const void* dres,
                       int dtype, int T, int d, void* dH, float* dgain, void* workspace, hipStream_t s) {
  float* part = static_cast<float*>(workspace);
  const int rc = dtype == BTX_BF16 ? launch_typed<bf16_t>(dXn, h, gain, rstd, dres, T, d, dH, part, s)
                                   : launch_typed<float>(dXn, h, gain, rstd, dres, T, d, dH, part, s);
  if (rc) return rc;
  rmsnorm_dgain_reduce_kernel<<<ceil_div(d, 64), 64 * kRedGroups, 0, s>>>(part, ceil_div(T, kNormTok), d, dgain);
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

}  // namespace btx
