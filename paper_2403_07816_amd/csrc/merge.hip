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

__global__ __launch_bounds__(256) void merge_bf16_kernel(Ptrs in, int N, bf16_t* __restrict__ out, int64_t numel) {
  const int64_t nchunk = numel / 8;
  const float fn = (float)N;
  for (int64_t c = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; c < nchunk; c += (int64_t)gridDim.x * blockDim.x) {
    float acc[8] = {};
    for (int n = 0; n < N; ++n) {
      const u32x4 w = static_cast<const u32x4*>(in.p[n])[c];
#pragma unroll
      for (int i = 0; i < 4; ++i) { acc[2 * i] += bf16lo(w[i]); acc[2 * i + 1] += bf16hi(w[i]); }
    }
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      o[i] = (uint32_t)mean_to_bf16(acc[2 * i], fn) | ((uint32_t)mean_to_bf16(acc[2 * i + 1], fn) << 16);
    reinterpret_cast<u32x4*>(out)[c] = o;
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
  const int grid = (int)std::min<int64_t>(std::max<int64_t>((chunks + 255) / 256, 1), 256 * 32);
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
  const int grid = (int)std::min<int64_t>(std::max<int64_t>((chunks + 255) / 256, 1), 256 * 32);
  if (dtype == BTX_BF16) merge_bf16_kernel<<<grid, 256, 0, s>>>(p, N, static_cast<bf16_t*>(out), numel);
  else merge_f32_kernel<<<grid, 256, 0, s>>>(p, N, static_cast<float*>(out), numel);
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

}  // namespace btx
