// Elementwise mean of N tensors: the merge of the branched models' non-feed-forward
// parameters (Sec. 3.2).  HBM-bound streaming kernel: 16-byte loads from each input,
// sum in input order (fp32 for bf16 storage, fp64 for fp32 storage), one division, one
// rounding.
#include <algorithm>
#include "common.h"

namespace btx {
namespace {

constexpr int kMaxInputs = 16;
struct Ptrs { const void* p[kMaxInputs]; };

// Quotient sum/n rounded once to bf16.  q = fl32(sum/n) alone would round twice; the
// sign of the exact remainder sum - q*n (one fma) says on which side of q the true
// quotient lies, which settles the only case where the second rounding can go wrong:
// q exactly half-way between two bf16 values.
__device__ __forceinline__ bf16_t mean_to_bf16(float sum, float n) {
  const float q = sum / n;
  uint32_t u = __float_as_uint(q);
  if ((u & 0xffffu) == 0x8000u) {
    const float r = fmaf(-q, n, sum);
    if (r != 0.f) {
      const bool up = (r > 0.f) == (q > 0.f);  // true quotient has larger magnitude than q
      return (bf16_t)((u >> 16) + (up ? 1u : 0u));
    }
  }
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// NT > 0: the number of inputs is a compile-time constant, so that a thread's loads (UNROLL chunks
// of 16 bytes from each input) are all in flight before the first one is used; NT = 0 takes any N.
constexpr int kMergeUnroll = 2;
template <int NT>
__global__ __launch_bounds__(256) void merge_bf16_kernel(Ptrs in, int N_rt, bf16_t* __restrict__ out, int64_t numel) {
  constexpr int UNROLL = kMergeUnroll;
  const int N = NT > 0 ? NT : N_rt;
  const int64_t nchunk = numel / 8;
  const float fn = (float)N;
  auto finish = [&](const float* acc, int64_t c) {
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      o[i] = (uint32_t)mean_to_bf16(acc[2 * i], fn) | ((uint32_t)mean_to_bf16(acc[2 * i + 1], fn) << 16);
    __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(out) + c);   // streamed once: keep it out of the caches
  };
  auto ld = [&](int n, int64_t c) {
    return __builtin_nontemporal_load(static_cast<const u32x4*>(in.p[n]) + c);
  };
  // The tensor is cut into UNROLL equal runs of `run` chunks; a thread takes the chunk at its own position
  // in every run, so the chip streams UNROLL * (N + 1) separate regions at a time.  One thread per position
  // and no loop over the grid: a grid-stride loop over 8192 workgroups was a third slower.
  const int64_t run = (nchunk + UNROLL - 1) / UNROLL;
  const int64_t c0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (c0 < run) {
    if (NT > 0 && c0 + (UNROLL - 1) * run < nchunk) {
      u32x4 w[UNROLL][NT > 0 ? NT : 1];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
#pragma unroll
        for (int n = 0; n < NT; ++n) w[u][n] = ld(n, c0 + u * run);
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        float acc[8] = {};
#pragma unroll
        for (int n = 0; n < NT; ++n)       // input order, as the definition sums
#pragma unroll
          for (int i = 0; i < 4; ++i) { acc[2 * i] += bf16lo(w[u][n][i]); acc[2 * i + 1] += bf16hi(w[u][n][i]); }
        finish(acc, c0 + u * run);
      }
    } else {
      for (int u = 0; u < UNROLL; ++u) {
        const int64_t c = c0 + u * run;
        if (c >= nchunk) break;
        float acc[8] = {};
        for (int n = 0; n < N; ++n) {
          const u32x4 w = ld(n, c);
#pragma unroll
          for (int i = 0; i < 4; ++i) { acc[2 * i] += bf16lo(w[i]); acc[2 * i + 1] += bf16hi(w[i]); }
        }
        finish(acc, c);
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < (int)(numel - nchunk * 8)) {  // ragged tail
    const int64_t i = nchunk * 8 + threadIdx.x;
    float a = 0.f;
    for (int n = 0; n < N; ++n) a += bf16_to_f32(static_cast<const bf16_t*>(in.p[n])[i]);
    out[i] = mean_to_bf16(a, fn);
  }
}

// fp32 storage: the sum and the division run in fp64 (free on an HBM-bound kernel), so the
// result is the correctly rounded mean and the mean of N equal values is that value.
__global__ __launch_bounds__(256) void merge_f32_kernel(Ptrs in, int N, float* __restrict__ out, int64_t numel) {
  const int64_t nchunk = numel / 4;
  const double fn = (double)N;
  for (int64_t c = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; c < nchunk; c += (int64_t)gridDim.x * blockDim.x) {
    double acc[4] = {};
    for (int n = 0; n < N; ++n) {
      const f32x4 v = static_cast<const f32x4*>(in.p[n])[c];
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] += (double)v[i];
    }
    f32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (float)(acc[i] / fn);
    reinterpret_cast<f32x4*>(out)[c] = o;
  }
  if (blockIdx.x == 0 && threadIdx.x < (int)(numel - nchunk * 4)) {
    const int64_t i = nchunk * 4 + threadIdx.x;
    double a = 0.0;
    for (int n = 0; n < N; ++n) a += (double)static_cast<const float*>(in.p[n])[i];
    out[i] = (float)(a / fn);
  }
}

// Weighted merge: sum_n w_n * in_n, accumulated in fp64 in input order (every product of a
// float weight and a bf16 / fp32 value is exact in fp64, so the sum is the same fp64 number a
// host computes in that order) and rounded once to the storage type.
struct Weights { float w[kMaxInputs]; };

__global__ __launch_bounds__(256) void merge_weighted_bf16_kernel(Ptrs in, Weights wt, int N, bf16_t* __restrict__ out,
                                                                   int64_t numel) {
  const int64_t nchunk = numel / 8;
  for (int64_t c = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; c < nchunk; c += (int64_t)gridDim.x * blockDim.x) {
    double acc[8] = {};
    for (int n = 0; n < N; ++n) {
      const u32x4 w = static_cast<const u32x4*>(in.p[n])[c];
      const double wn = (double)wt.w[n];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] += wn * (double)bf16lo(w[i]);
        acc[2 * i + 1] += wn * (double)bf16hi(w[i]);
      }
    }
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (uint32_t)f64_to_bf16(acc[2 * i]) | ((uint32_t)f64_to_bf16(acc[2 * i + 1]) << 16);
    reinterpret_cast<u32x4*>(out)[c] = o;
  }
  if (blockIdx.x == 0 && threadIdx.x < (int)(numel - nchunk * 8)) {  // ragged tail
    const int64_t i = nchunk * 8 + threadIdx.x;
    double a = 0.0;
    for (int n = 0; n < N; ++n) a += (double)wt.w[n] * (double)bf16_to_f32(static_cast<const bf16_t*>(in.p[n])[i]);
    out[i] = f64_to_bf16(a);
  }
}

__global__ __launch_bounds__(256) void merge_weighted_f32_kernel(Ptrs in, Weights wt, int N, float* __restrict__ out,
                                                                  int64_t numel) {
  const int64_t nchunk = numel / 4;
  for (int64_t c = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; c < nchunk; c += (int64_t)gridDim.x * blockDim.x) {
    double acc[4] = {};
    for (int n = 0; n < N; ++n) {
      const f32x4 v = static_cast<const f32x4*>(in.p[n])[c];
      const double wn = (double)wt.w[n];
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] += wn * (double)v[i];
    }
    f32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (float)acc[i];
    reinterpret_cast<f32x4*>(out)[c] = o;
  }
  if (blockIdx.x == 0 && threadIdx.x < (int)(numel - nchunk * 4)) {
    const int64_t i = nchunk * 4 + threadIdx.x;
    double a = 0.0;
    for (int n = 0; n < N; ++n) a += (double)wt.w[n] * (double)static_cast<const float*>(in.p[n])[i];
    out[i] = (float)a;
  }
}

}  // namespace

int launch_merge_weighted(const void* const* inputs, const float* weights, int N, void* out, int64_t numel, int dtype,
                          hipStream_t s) {
  Ptrs p{};
  Weights w{};
  for (int n = 0; n < N; ++n) { p.p[n] = inputs[n]; w.w[n] = weights[n]; }
  const int per = dtype == BTX_BF16 ? 8 : 4;
  const int64_t chunks = numel / per;
  // one chunk per thread wherever the grid allows it (a loop over fewer workgroups streams slower)
  const int grid = (int)std::min<int64_t>(std::max<int64_t>((chunks + 255) / 256, 1), 0x7fffffff);
  if (dtype == BTX_BF16) merge_weighted_bf16_kernel<<<grid, 256, 0, s>>>(p, w, N, static_cast<bf16_t*>(out), numel);
  else merge_weighted_f32_kernel<<<grid, 256, 0, s>>>(p, w, N, static_cast<float*>(out), numel);
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

int launch_merge_average(const void* const* inputs, int N, void* out, int64_t numel, int dtype, hipStream_t s) {
  Ptrs p{};
  for (int n = 0; n < N; ++n) p.p[n] = inputs[n];
  const int per = dtype == BTX_BF16 ? 8 : 4;
  const int64_t chunks = numel / per;
  const int64_t bf16_run = (numel / 8 + kMergeUnroll - 1) / kMergeUnroll;   // chunks per run, one thread each
  const int64_t bf16_blocks = std::max<int64_t>((bf16_run + 255) / 256, 1);
  if (dtype == BTX_BF16 && bf16_blocks > 0x7fffffff) return BTX_ERR_UNSUPPORTED;
  const int grid = dtype == BTX_BF16 ? (int)bf16_blocks
                                     : (int)std::min<int64_t>(std::max<int64_t>((chunks + 255) / 256, 1), 0x7fffffff);
  if (dtype == BTX_BF16) {
    bf16_t* o = static_cast<bf16_t*>(out);
    switch (N) {
      case 2: merge_bf16_kernel<2><<<grid, 256, 0, s>>>(p, N, o, numel); break;
      case 3: merge_bf16_kernel<3><<<grid, 256, 0, s>>>(p, N, o, numel); break;
      case 4: merge_bf16_kernel<4><<<grid, 256, 0, s>>>(p, N, o, numel); break;
      case 5: merge_bf16_kernel<5><<<grid, 256, 0, s>>>(p, N, o, numel); break;
      case 6: merge_bf16_kernel<6><<<grid, 256, 0, s>>>(p, N, o, numel); break;
      case 8: merge_bf16_kernel<8><<<grid, 256, 0, s>>>(p, N, o, numel); break;
      default: merge_bf16_kernel<0><<<grid, 256, 0, s>>>(p, N, o, numel); break;
    }
  } else {
    merge_f32_kernel<<<grid, 256, 0, s>>>(p, N, static_cast<float*>(out), numel);
  }
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

}  // namespace btx
