// Row movement around the expert GEMMs (both HBM-bound streaming kernels):
//   gather_rows  dst[r] = src[perm[r] / k]: token rows copied into expert-grouped order
//                (forward: x -> xs; backward: dY -> dys).
//   gather_rows_t  the same rows, transposed and padded for the weight-gradient products,
//                whose contraction runs over grouped rows: dst[c][P_e + i] = src[perm[o_e + i] / k][c]
//                for row i of expert e, with P_e = sum over e' < e of n_e' rounded up to 64 and
//                zeros from P_e + n_e to P_(e+1).  64 rows x 128 columns are turned around in LDS.
//   combine      out[t] = (residual[t] +) sum_j gates[t,j] * y[inv_pos[t,j]]: the gate-weighted sum of the
//                layer equation (Sec. 3.2), one wavefront per token row, slots summed in
//                ascending j in fp32, one rounding.  No atomics: every output row has
//                exactly one writer.
// Rows are moved as 16-byte chunks, consecutive lanes on consecutive chunks.
#include <type_traits>

#include "common.h"

// rows that a kernel reads or writes exactly once are streamed past the caches (with 8 slots per token combine
// gained 7 % from it; nothing lost elsewhere)
#define BTX_LD(p) __builtin_nontemporal_load(p)
#define BTX_ST(p, v) __builtin_nontemporal_store(v, p)

namespace btx {
namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void gather_rows_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                               const int32_t* __restrict__ perm, int R, int k,
                                                               int chunks_per_row) {
  const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
  const int r = blockIdx.x * (kThreads / kWave) + wave;
  if (r >= R) return;
  const int t = perm[r] / k;
  const u32x4* s = src + (size_t)t * chunks_per_row;
  u32x4* o = dst + (size_t)r * chunks_per_row;
  for (int c = lane; c < chunks_per_row; c += kWave) o[c] = s[c];
}

constexpr int kTRows = 64, kTCols = 128;
__global__ __launch_bounds__(kThreads) void gather_rows_t_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst,
                                                                 const int32_t* __restrict__ perm,
                                                                 const int32_t* __restrict__ offsets, int E, int k,
                                                                 int d, int pitch) {
  __shared__ uint32_t tile[kTRows][kTCols / 2 + 1];     // +1 dword: the column reads below hit distinct banks
  const int pb = blockIdx.x * kTRows;                   // first padded row of this block
  int e = 0, P = 0, base = 0, n = 0;
  for (; e < E; ++e) {
    base = offsets[e];
    n = offsets[e + 1] - base;
    const int np = (n + kTRows - 1) & ~(kTRows - 1);
    if (pb < P + np) break;
    P += np;
  }
  if (e == E) return;
  const int i0 = pb - P, c0 = blockIdx.y * kTCols;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int row = threadIdx.x / 16 + 16 * it, chunk = threadIdx.x % 16;
    u32x4 v{0u, 0u, 0u, 0u};
    if (i0 + row < n && c0 + 8 * chunk < d)
      v = *reinterpret_cast<const u32x4*>(src + (size_t)(perm[base + i0 + row] / k) * d + c0 + 8 * chunk);
#pragma unroll
    for (int x = 0; x < 4; ++x) tile[row][4 * chunk + x] = v[x];
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int col = threadIdx.x / 8 + 32 * it, tc = threadIdx.x % 8;
    uint32_t h[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const uint32_t w = tile[8 * tc + x][col >> 1];
      h[x] = (col & 1) ? (w >> 16) : (w & 0xffffu);
    }
    if (c0 + col < d)
      BTX_ST(reinterpret_cast<u32x4*>(dst + (size_t)(c0 + col) * pitch + pb + 8 * tc),
             (u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)}));
  }
}

template <typename ET> struct Chunk;  // 16 bytes of elements <-> floats
template <> struct Chunk<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const u32x4& w, float* v) {
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[2 * i] = bf16lo(w[i]); v[2 * i + 1] = bf16hi(w[i]); }
  }
  static __device__ __forceinline__ u32x4 pack(const float* v) {
    u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
    return w;
  }
};
template <> struct Chunk<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const u32x4& w, float* v) {
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(w[i]);
  }
  static __device__ __forceinline__ u32x4 pack(const float* v) {
    u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = __float_as_uint(v[i]);
    return w;
  }
};

// KMAX: slots whose grouped rows and gates a wavefront keeps in registers; the rows of those slots are
// requested together for every 16-byte column chunk (k > KMAX: the remaining slots are looked up as they come).
template <typename ET, int KMAX>
__global__ __launch_bounds__(kThreads) void combine_kernel(const u32x4* __restrict__ y, const float* __restrict__ gates,
                                                           const int32_t* __restrict__ inv_pos,
                                                           const u32x4* __restrict__ residual, u32x4* __restrict__ out,
                                                           int T, int k, int chunks_per_row) {
  constexpr int N = Chunk<ET>::N;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
  const int t = blockIdx.x * (kThreads / kWave) + wave;
  if (t >= T) return;
  int row[KMAX];
  float gate[KMAX];
#pragma unroll
  for (int j = 0; j < KMAX; ++j) {
    row[j] = j < k ? inv_pos[(size_t)t * k + j] : -1;             // -1: no such slot, or the pair was dropped
    gate[j] = (j < k && gates) ? gates[(size_t)t * k + j] : 1.f;
  }
  for (int c = lane; c < chunks_per_row; c += kWave) {
    float acc[N];
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.f;
    u32x4 w[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) w[j] = BTX_LD(y + (size_t)max(row[j], 0) * chunks_per_row + c);   // all slots in flight
    if (residual) Chunk<ET>::unpack(residual[(size_t)t * chunks_per_row + c], acc);   // block input, added in fp32
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {          // ascending slot order, as the definition sums
      float v[N];
      Chunk<ET>::unpack(w[j], v);
      if (row[j] >= 0) {
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = fmaf(gate[j], v[i], acc[i]);
      }
    }
    for (int j = KMAX; j < k; ++j) {
      const int r = inv_pos[(size_t)t * k + j];
      if (r < 0) continue;                  // pair dropped at its expert's capacity
      const float g = gates ? gates[(size_t)t * k + j] : 1.f;
      float v[N];
      Chunk<ET>::unpack(y[(size_t)r * chunks_per_row + c], v);
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] = fmaf(g, v[i], acc[i]);
    }
    BTX_ST(out + (size_t)t * chunks_per_row + c, Chunk<ET>::pack(acc));
  }
}

}  // namespace

int launch_gather_rows(const void* src, void* dst, const int32_t* perm, int R, int k, int d, int dtype, hipStream_t s) {
  const int esz = dtype == BTX_BF16 ? 2 : 4;
  const int chunks = d * esz / 16;
  gather_rows_kernel<<<ceil_div(R, kThreads / kWave), kThreads, 0, s>>>(
      static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), perm, R, k, chunks);
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

int launch_gather_rows_t(const void* src, void* dst, const int32_t* perm, const int32_t* offsets, int R, int k, int d,
                         int E, int pitch, hipStream_t s) {
  if (pitch % 8 != 0 || pitch < (int)align_up((size_t)R, kTRows) + kTRows * E) return BTX_ERR_INVALID_ARG;
  const dim3 grid(ceil_div(R, kTRows) + E, ceil_div(d, kTCols));
  gather_rows_t_kernel<<<grid, kThreads, 0, s>>>(static_cast<const bf16_t*>(src), static_cast<bf16_t*>(dst), perm,
                                                 offsets, E, k, d, pitch);
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

int launch_combine(const void* y, const float* gates, const int32_t* inv_pos, const void* residual, void* out, int T,
                   int k, int d, int dtype, hipStream_t s) {
  const int esz = dtype == BTX_BF16 ? 2 : 4;
  const int chunks = d * esz / 16;
  dim3 grid(ceil_div(T, kThreads / kWave));
  auto run = [&](auto tag, auto kmax) {
    using ET = decltype(tag);
    combine_kernel<ET, decltype(kmax)::value><<<grid, kThreads, 0, s>>>(
        static_cast<const u32x4*>(y), gates, inv_pos, static_cast<const u32x4*>(residual), static_cast<u32x4*>(out), T, k,
        chunks);
  };
  auto by_k = [&](auto tag) {
    if (k <= 1) run(tag, std::integral_constant<int, 1>{});
    else if (k <= 2) run(tag, std::integral_constant<int, 2>{});
    else run(tag, std::integral_constant<int, 4>{});   // eight slots in flight were no faster than four
  };
  if (dtype == BTX_BF16) by_k(bf16_t{});
  else by_k(float{});
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

}  // namespace btx
