// Measurement aid: what the matrix cores sustain on this chip when nothing else runs.
// Every lane keeps 8 + 8 operand fragments of caller-supplied bf16 data in registers and
// issues v_mfma_f32_16x16x32_bf16 (the instruction of the expert GEMMs) over all 64 (A,B) pairs,
// so consecutive instructions see different operands, as in a GEMM, but there is no LDS or
// memory traffic.  The chip lowers
// its clock under this load (the nominal 2.5 PFLOP/s assumes 2.4 GHz); the rate measured here,
// on the same kind of data as the layer's, is the ceiling the expert GEMMs can be held against.
#include "common.h"

namespace btx {
namespace {

constexpr int kProbeThreads = 512;   // 8 wavefronts per CU, 2 per SIMD, like the GEMM kernels
constexpr int kFrags = 8;
constexpr int kRounds = 2;           // passes over the 64 pairs per iteration

__global__ __launch_bounds__(kProbeThreads) void mfma_rate_kernel(const u32x4* __restrict__ data, size_t n_chunks,
                                                                   float* __restrict__ out, int iters) {
  const size_t t = (size_t)blockIdx.x * kProbeThreads + threadIdx.x;
  bf16x8 a[kFrags], b[kFrags];
#pragma unroll
  for (int i = 0; i < kFrags; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, data[(t * 2 * kFrags + i) % n_chunks]);
    b[i] = __builtin_bit_cast(bf16x8, data[(t * 2 * kFrags + kFrags + i) % n_chunks]);
  }
  f32x4 acc[32];
#pragma unroll
  for (int i = 0; i < 32; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[i][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < kRounds; ++r)
#pragma unroll
      for (int i = 0; i < kFrags; ++i)
#pragma unroll
        for (int j = 0; j < kFrags; ++j)
          acc[(i * kFrags + j) % 32] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[(i * kFrags + j) % 32], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) s += acc[i][v];
  out[t] = s;   // keeps the loop alive
}

}  // namespace
}  // namespace btx

extern "C" {
#pragma GCC visibility push(default)

size_t btx_probe_mfma_out_bytes(int n_blocks) {
  return n_blocks > 0 ? (size_t)n_blocks * btx::kProbeThreads * sizeof(float) : 0;
}

int btx_probe_mfma(const void* data, size_t data_bytes, float* out, int n_blocks, int iters, double* flops,
                   void* stream) {
  if (!data || !out || data_bytes < 16 || ((uintptr_t)data & 15) || n_blocks < 1 || n_blocks > 65536 || iters < 1)
    return BTX_ERR_INVALID_ARG;
  btx::mfma_rate_kernel<<<n_blocks, btx::kProbeThreads, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const btx::u32x4*>(data), data_bytes / 16, out, iters);
  if (hipGetLastError() != hipSuccess) return BTX_ERR_HIP;
  if (flops)
    *flops = 2.0 * 16 * 16 * 32 * btx::kRounds * btx::kFrags * btx::kFrags * (double)iters * n_blocks *
             (btx::kProbeThreads / btx::kWave);
  return BTX_OK;
}

#pragma GCC visibility pop
}
