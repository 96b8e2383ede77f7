// Router: logits, softmax, expert selection, gates, load-balancing statistics and
// the stable grouping of (token, slot) pairs by expert (Sec. 3.2 router and Top-k;
// Sec. 3.3 load balancing, Switch and sample-top-1 routing).
//
// Four launches, no atomics, no host round trip:
//   (optional) the RMS normalisation in front of the sublayer (the seed model's blocks
//   normalise before their feed-forward, Sec. 4.1) is folded into route_tokens: the raw rows
//   are read once more for their mean square (fp64), the normalised, rounded rows are written
//   out for the expert GEMMs and are what the logits are computed from.
//   0. transpose_wr   W_router [d,E] -> [E,d] in the workspace: a lane then reads its 8 columns of
//                     an expert as 32 contiguous bytes and a wavefront's load covers 2 KB in one
//                     piece, where the [d,E] form costs one cache line per lane and load.
//   1. route_tokens   one wavefront handles kTokPerWave tokens at a time: fp32 dot
//                     products of the token row with W_router (lanes split the row,
//                     butterfly reduction; with more than 8 experts fp32 matrix instructions
//                     on 16 tokens x 16 experts instead), then softmax / selection / gates
//                     with one lane per expert.  Each workgroup owns kTokPerBlock consecutive
//                     tokens and writes its per-expert counts and gate/prob sums.
//   2. route_scan     one workgroup per expert: exclusive scan of its block counts (fixed
//                     order) and its finished statistics.
//   3. route_scatter  every wavefront rebuilds the expert offsets from the counts (one lane per
//                     expert); one wavefront per block re-reads its indices and writes perm and
//                     inv_pos; ranks inside a block come from wavefront ballots, so the
//                     order inside every expert group is the (token, slot) order.  The first
//                     wavefront also writes offsets and lb_loss.
#include <type_traits>

#include "common.h"

namespace btx {
namespace {

constexpr int kTokPerWave = 4;
constexpr int kWavesPerBlock = 4;
constexpr int kTokPerBlock = kTokPerWave * kWavesPerBlock;  // 16 consecutive tokens per workgroup
constexpr int kScanThreads = 1024;
// blocks of kTokPerBlock tokens per workgroup when the logits run on the matrix cores: they share each
// load of W_router (1: 130 us, 2: 112 us, 4: 204 us for 16384 tokens x 32 experts; with 4 the launch has
// one wavefront per SIMD left)
constexpr int kMatrixGroups = 2;

// normalised value, rounded once to the row's storage type; `back` is that value again as float
template <typename XT> struct NormRound;
template <> struct NormRound<bf16_t> {
  static __device__ __forceinline__ bf16_t rnd(double v, float& back) {
    const bf16_t h = f64_to_bf16(v);
    back = bf16_to_f32(h);
    return h;
  }
  static __device__ __forceinline__ void st8(bf16_t* p, const bf16_t* h) {
    *reinterpret_cast<u32x4*>(p) = u32x4{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16),
                                         (uint32_t)h[4] | ((uint32_t)h[5] << 16), (uint32_t)h[6] | ((uint32_t)h[7] << 16)};
  }
};
template <> struct NormRound<float> {
  static __device__ __forceinline__ float rnd(double v, float& back) { return back = (float)v; }
  static __device__ __forceinline__ void st8(float* p, const float* h) {
    *reinterpret_cast<f32x4*>(p) = f32x4{h[0], h[1], h[2], h[3]};
    *reinterpret_cast<f32x4*>(p + 4) = f32x4{h[4], h[5], h[6], h[7]};
  }
};
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);   // every lane ends with the same bits
  return v;
}

struct Best { float v; int i; };
// larger value wins; equal values: lower index wins
__device__ __forceinline__ Best best_of(Best a, Best b) {
  return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;
}
template <int CTRL> __device__ __forceinline__ Best dpp_best(Best x) {
  return best_of(x, Best{dpp_f32<CTRL>(x.v), dpp_i32<CTRL>(x.i)});
}
__device__ __forceinline__ Best lane_best(Best x, int lane) {
  return Best{lane_f32(x.v, lane), __builtin_amdgcn_readlane(x.i, lane)};
}
// (value, index) arg-max over the wavefront; the same DPP scheme as wave_sum
__device__ __forceinline__ Best wave_best(Best x) {
  x = dpp_best<kDppXor1>(x);
  x = dpp_best<kDppXor2>(x);
  x = dpp_best<kDppRor4>(x);
  x = dpp_best<kDppRor8>(x);
  return best_of(best_of(lane_best(x, 0), lane_best(x, 16)), best_of(lane_best(x, 32), lane_best(x, 48)));
}
__device__ __forceinline__ float wave_incl_scan(float v, int lane) {
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const float u = __shfl_up(v, o, kWave);
    if (lane >= o) v += u;
  }
  return v;
}

// 8 consecutive elements of a row as they are loaded (the conversion to float waits until they are used,
// so that loads issued ahead stay in flight)
template <typename XT> struct Raw8;
template <> struct Raw8<bf16_t> {
  u32x4 r;
  __device__ __forceinline__ void load(const bf16_t* p) { r = *reinterpret_cast<const u32x4*>(p); }
  __device__ __forceinline__ float get(int i) const { return (i & 1) ? bf16hi(r[i >> 1]) : bf16lo(r[i >> 1]); }
};
template <> struct Raw8<float> {
  f32x4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = *reinterpret_cast<const f32x4*>(p);
    b = *reinterpret_cast<const f32x4*>(p + 4);
  }
  __device__ __forceinline__ float get(int i) const { return i < 4 ? a[i] : b[i - 4]; }
};

// EC experts are accumulated per pass over the row; kTokPerWave tokens share each
// load of the (transposed) W_router.
template <typename XT, int EC, bool NORM, int MG = 1, int NS = 1>
__global__ __launch_bounds__(kWavesPerBlock* kWave) void route_tokens_kernel(
    const XT* __restrict__ x, const float* __restrict__ WrT, const float* __restrict__ br,
    const float* __restrict__ U, int T, int d, int E, int k, int mode, float inv_tau, int32_t* __restrict__ topk_idx,
    float* __restrict__ gates, float* __restrict__ probs, int32_t* __restrict__ blk_counts,
    float* __restrict__ blk_gsum, float* __restrict__ blk_psum, const float* __restrict__ gain, float eps,
    XT* __restrict__ xn, float* __restrict__ rstd_out) {
  constexpr bool MATRIX = EC == 0;                      // logits on the matrix cores (many experts)
  static_assert(!(MATRIX && NORM), "the matrix-core logits take the rows as they are");
  // the matrix variant covers G blocks of kTokPerBlock tokens per workgroup (they share every load of
  // W_router); the statistics stay per block of kTokPerBlock tokens either way
  constexpr int G = MATRIX ? MG : 1;
  __shared__ float s_logit[kWavesPerBlock][kTokPerWave][kMaxExperts];
  __shared__ float s_stat[kWavesPerBlock][3][kMaxExperts];
  extern __shared__ float s_part[];                     // MATRIX: [wavefront][G * kTokPerBlock tokens][16 NS experts]
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int n_blk = (T + kTokPerBlock - 1) / kTokPerBlock;
  const int pitch = 16 * NS;                            // MATRIX: NS = ceil(E / 16) sets of 16 experts
  int t0 = blockIdx.x * G * kTokPerBlock + wave * kTokPerWave;

  // ---- row factors of the normalisation -------------------------------------
  // fp64 throughout: the rounded rows then agree with a host fp64 evaluation except where the
  // exact value lies within 1e-16 (relative) of a rounding tie, and so do the routing decisions.
  double rs[kTokPerWave];
  if (NORM) {
    double ss[kTokPerWave] = {};
    for (int c0 = lane * 8; c0 < d; c0 += kWave * 8) {
#pragma unroll
      for (int q = 0; q < kTokPerWave; ++q) {
        float v[8];
        RowVec<XT, 8>::ld(x + (size_t)min(t0 + q, T - 1) * d + c0, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) ss[q] += (double)v[i] * (double)v[i];
      }
    }
#pragma unroll
    for (int q = 0; q < kTokPerWave; ++q) {
      rs[q] = 1.0 / sqrt(wave_sum_f64(ss[q]) / (double)d + (double)eps);
      if (lane == 0 && t0 + q < T) rstd_out[t0 + q] = (float)rs[q];
    }
  }

  // ---- logits -------------------------------------------------------------
  if constexpr (MATRIX) {
    // fp32 16x16x4 matrix products: the workgroup's 16 tokens are the rows, 16 experts at a time the
    // columns; wavefront w takes the 32-column pieces w, w + 4, ... of the rows and the four partial
    // sums are added in that order below.  A lane supplies A[token = lane % 16][k] and
    // B[k][expert = lane % 16] for the 8 columns k = 32 piece + 8 (lane / 16) + i, one product per i,
    // and receives the sums of expert lane % 16 for the tokens 4 (lane / 16) + v.
    const int row = lane & 15, kc = lane >> 4;
    const XT* xrow[G];
    const float* wrow[NS];
    f32x4 acc[G][NS];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      xrow[g] = x + (size_t)min((blockIdx.x * G + g) * kTokPerBlock + row, T - 1) * d;   // clamped rows are dropped later
#pragma unroll
      for (int u = 0; u < NS; ++u) acc[g][u] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // the lanes of the experts past E read expert E - 1; their sums are never looked at
#pragma unroll
    for (int u = 0; u < NS; ++u) wrow[u] = WrT + (size_t)min(u * 16 + row, E - 1) * d;
    // Trip `it` of this wavefront covers columns 32 (wave + 4 it) ... + 31.  The loads of kAhead trips are
    // in flight ahead of the products, and nothing in the loop is conditional (the matrix instructions
    // take all 64 lanes, and a branch would make the compiler wait for every load): a trip past the
    // last one repeats the last one's loads, and a lane whose 8 columns lie past the row's end reads the
    // row's first 8; both supply zeros for the tokens.
    constexpr int kAhead = 3;
    struct Piece { Raw8<XT> xr[G]; Raw8<float> wr[NS]; };
    Piece buf[kAhead];
    const int n_it = max(0, (d - wave * 32 + kWavesPerBlock * 32 - 1) / (kWavesPerBlock * 32));
    auto col0 = [&](int it, bool& live) {
      const int c = (wave + kWavesPerBlock * min(it, max(n_it - 1, 0))) * 32 + kc * 8;
      live = it < n_it && c < d;
      return c < d ? c : 0;
    };
    auto fetch = [&](Piece& pc, int it) {
      bool live;
      const int c0 = col0(it, live);
#pragma unroll
      for (int g = 0; g < G; ++g) pc.xr[g].load(xrow[g] + c0);
#pragma unroll
      for (int u = 0; u < NS; ++u) pc.wr[u].load(wrow[u] + c0);
    };
    auto multiply = [&](const Piece& pc, int it) {
      bool live;
      col0(it, live);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float xa[G];
#pragma unroll
        for (int g = 0; g < G; ++g) xa[g] = live ? pc.xr[g].get(i) : 0.f;
#pragma unroll
        for (int u = 0; u < NS; ++u) {
          const float wb = pc.wr[u].get(i);
#pragma unroll
          for (int g = 0; g < G; ++g) acc[g][u] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[g], wb, acc[g][u], 0, 0, 0);
        }
      }
    };
#pragma unroll
    for (int j = 0; j < kAhead - 1; ++j) fetch(buf[j], j);
    for (int it0 = 0; it0 < n_it; it0 += kAhead) {
#pragma unroll
      for (int j = 0; j < kAhead; ++j) {
        fetch(buf[(j + kAhead - 1) % kAhead], it0 + j + kAhead - 1);
        __builtin_amdgcn_sched_barrier(0);              // keeps the compiler from sinking the loads to their uses
        multiply(buf[j], it0 + j);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int u = 0; u < NS; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          s_part[((wave * G + g) * kTokPerBlock + 4 * kc + v) * pitch + u * 16 + row] = acc[g][u][v];
  }
  constexpr int ECN = MATRIX ? 1 : EC;                  // (the loop below is not instantiated for MATRIX)
  if constexpr (!MATRIX) for (int e0 = 0; e0 < E; e0 += ECN) {
    float acc[kTokPerWave][ECN];
#pragma unroll
    for (int q = 0; q < kTokPerWave; ++q)
#pragma unroll
      for (int j = 0; j < ECN; ++j) acc[q][j] = 0.f;
    for (int c0 = lane * 8; c0 < d; c0 += kWave * 8) {
      float xv[kTokPerWave][8];
#pragma unroll
      for (int q = 0; q < kTokPerWave; ++q) {
        const int t = min(t0 + q, T - 1);  // clamped rows are computed and then dropped
        RowVec<XT, 8>::ld(x + (size_t)t * d + c0, xv[q]);
      }
      if (NORM) {
        float gv[8];
        RowVec<float, 8>::ld(gain + c0, gv);
#pragma unroll
        for (int q = 0; q < kTokPerWave; ++q) {
          XT h[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) h[i] = NormRound<XT>::rnd((double)xv[q][i] * rs[q] * (double)gv[i], xv[q][i]);
          if (e0 == 0 && t0 + q < T) NormRound<XT>::st8(xn + (size_t)(t0 + q) * d + c0, h);
        }
      }
#pragma unroll
      for (int j = 0; j < ECN; ++j) {
        float w[8] = {};
        if (e0 + j < E) RowVec<float, 8>::ld(WrT + (size_t)(e0 + j) * d + c0, w);
#pragma unroll
        for (int q = 0; q < kTokPerWave; ++q)
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[q][j] = fmaf(xv[q][i], w[i], acc[q][j]);
      }
    }
#pragma unroll
    for (int q = 0; q < kTokPerWave; ++q)
#pragma unroll
      for (int j = 0; j < ECN; ++j) {
        const float s = wave_sum(acc[q][j]);
        if (lane == 0 && e0 + j < E) s_logit[wave][q][e0 + j] = s;
      }
  }
  const bool live = lane < E;
  for (int g = 0; g < G; ++g, t0 += kTokPerBlock) {
    const int blk = blockIdx.x * G + g;                   // block of kTokPerBlock tokens
    if (blk >= n_blk) break;                              // uniform across the workgroup
    __syncthreads();                                      // logits (or partial sums) written; s_stat free again
    if (MATRIX && live) {                                 // the wavefronts' partial sums, in wavefront order
#pragma unroll
      for (int q = 0; q < kTokPerWave; ++q) {
        const int tok = g * kTokPerBlock + wave * kTokPerWave + q;
        float sum = s_part[tok * pitch + lane];
#pragma unroll
        for (int w = 1; w < kWavesPerBlock; ++w) sum += s_part[(w * G * kTokPerBlock + tok) * pitch + lane];
        s_logit[wave][q][lane] = sum;                     // read back by this lane only
      }
    }

    // ---- per token: softmax, selection, gates; lane e owns expert e ----------
    int cnt = 0;
    float gsum = 0.f, psum = 0.f;
    for (int q = 0; q < kTokPerWave; ++q) {
      const int t = t0 + q;
      if (t >= T) break;  // uniform across the wave
      const float s = live ? s_logit[wave][q][lane] + (br ? br[lane] : 0.f) : -INFINITY;
      const float smax = wave_max(s);
      const float z = live ? __expf(s - smax) : 0.f;
      const float zsum = wave_sum(z);
      const float p = z / zsum;
      if (live) probs[(size_t)t * E + lane] = p;
      psum += p;
      if (mode == BTX_ROUTE_TOPK_RENORM) {
        float cand = s;
        int my_slot = -1;
        for (int j = 0; j < k; ++j) {
          const Best b = wave_best(Best{cand, lane});
          if (lane == b.i) { my_slot = j; cand = -INFINITY; }
        }
        const float zsel = wave_sum(my_slot >= 0 ? z : 0.f);
        if (my_slot >= 0) {
          const float g = z / zsel;
          topk_idx[(size_t)t * k + my_slot] = lane;
          gates[(size_t)t * k + my_slot] = g;
          gsum += g;
          cnt += 1;
        }
      } else {
        int chosen;
        float g = p;
        if (mode == BTX_ROUTE_SWITCH_TOP1) {
          chosen = wave_best(Best{s, lane}).i;
        } else if (mode == BTX_ROUTE_GUMBEL_TOP1) {
          // soft sample softmax((logits + noise) / tau); its largest entry is 1 / sum of the
          // others' ratios to it, and that entry alone is kept
          const float noisy = live ? s + U[(size_t)t * E + lane] : -INFINITY;
          const Best b = wave_best(Best{noisy, lane});
          chosen = b.i;
          g = 1.f / wave_sum(live ? __expf((noisy - b.v) * inv_tau) : 0.f);
        } else {
          const float c = wave_incl_scan(p, lane);
          const unsigned long long m = __ballot(live && c > U[t]);
          chosen = m ? (__ffsll((long long)m) - 1) : (E - 1);
        }
        if (lane == chosen) {
          topk_idx[t] = lane;
          gates[t] = g;
          gsum += g;
          cnt += 1;
        }
      }
    }
    s_stat[wave][0][lane] = __int_as_float(cnt);
    s_stat[wave][1][lane] = gsum;
    s_stat[wave][2][lane] = psum;
    __syncthreads();
    if (threadIdx.x < E) {
      const int e = threadIdx.x;
      int c = 0;
      float gs = 0.f, p = 0.f;
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) {
        c += __float_as_int(s_stat[w][0][e]);
        gs += s_stat[w][1][e];
        p += s_stat[w][2][e];
      }
      blk_counts[(size_t)blk * E + e] = c;
      blk_gsum[(size_t)blk * E + e] = gs;
      blk_psum[(size_t)blk * E + e] = p;
    }
  }
}

// Exclusive scan of v over the workgroup (kScanThreads threads); returns the
// exclusive prefix and writes the total to `total`.
__device__ __forceinline__ int block_excl_scan(int v, int& total, int* s_wave) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  int incl = v;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int u = __shfl_up(incl, o, kWave);
    if (lane >= o) incl += u;
  }
  if (lane == kWave - 1) s_wave[wave] = incl;
  __syncthreads();
  int base = 0, tot = 0;
  for (int w = 0; w < kScanThreads / kWave; ++w) {
    const int c = s_wave[w];
    if (w < wave) base += c;
    tot += c;
  }
  __syncthreads();
  total = tot;
  return base + incl - v;
}

// one workgroup per expert
__global__ __launch_bounds__(kScanThreads) void route_scan_kernel(
    int nblk, int E, const int32_t* __restrict__ blk_counts, const float* __restrict__ blk_gsum,
    const float* __restrict__ blk_psum, int32_t* __restrict__ blk_base, int32_t* __restrict__ counts,
    float* __restrict__ gate_sum, float* __restrict__ prob_sum) {
  __shared__ int s_wave[kScanThreads / kWave];
  __shared__ float s_red[2][kScanThreads / kWave];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int e = blockIdx.x;
  int running = 0;
  float g = 0.f, p = 0.f;
  for (int b0 = 0; b0 < nblk; b0 += kScanThreads) {
    const int b = b0 + threadIdx.x;
    const int v = b < nblk ? blk_counts[(size_t)b * E + e] : 0;
    int total;
    const int ex = block_excl_scan(v, total, s_wave);
    if (b < nblk) {
      blk_base[(size_t)b * E + e] = running + ex;
      g += blk_gsum[(size_t)b * E + e];
      p += blk_psum[(size_t)b * E + e];
    }
    running += total;
  }
  // fixed-order reduction of the per-thread partial sums
  g = wave_sum(g);
  p = wave_sum(p);
  if (lane == 0) { s_red[0][wave] = g; s_red[1][wave] = p; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float gs = 0.f, ps = 0.f;
    for (int w = 0; w < kScanThreads / kWave; ++w) { gs += s_red[0][w]; ps += s_red[1][w]; }
    counts[e] = running;
    gate_sum[e] = gs;
    prob_sum[e] = ps;
  }
}

// grid: one wavefront per token block, plus workgroups that only clear perm's tail
__global__ __launch_bounds__(kWavesPerBlock* kWave) void route_scatter_kernel(
    int nblk, int T, int E, int k, int cap, int lb_mode, float lb_alpha, const int32_t* __restrict__ topk_idx,
    const int32_t* __restrict__ blk_base, const int32_t* __restrict__ counts, const float* __restrict__ gate_sum,
    const float* __restrict__ prob_sum, int32_t* __restrict__ offsets, float* __restrict__ lb_loss,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv_pos) {
  const int lane = threadIdx.x & (kWave - 1);
  // lane e: expert e's first grouped row.  capacity: an expert keeps its first `cap` pairs; the
  // statistics see the routing
  const int cnt = lane < E ? counts[lane] : 0;
  const int kept = cap > 0 ? min(cnt, cap) : cnt;
  int incl = kept;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int u = __shfl_up(incl, o, kWave);
    if (lane >= o) incl += u;
  }
  const int group0 = incl - kept;
  const int kept_total = __shfl(incl, kWave - 1, kWave);
  if (blockIdx.x == 0 && threadIdx.x < kWave) {
    if (lane < E) offsets[lane] = group0;
    if (lane == 0) offsets[E] = kept_total;
    float term = 0.f;
    if (lane < E) {
      const float u = lb_mode == BTX_LB_TOKEN_FRAC ? (float)cnt / ((float)T * (float)k) : gate_sum[lane] / (float)T;
      term = u * (prob_sum[lane] / (float)T);
    }
    float loss = 0.f;
    for (int e = 0; e < E; ++e) loss += __shfl(term, e, kWave);   // expert order
    if (lane == 0) *lb_loss = lb_alpha * (float)E * loss;
  }
  // grouped rows past the kept ones do not exist; whoever indexes through perm there
  // (kernels that run over all T*k rows) must still find a valid pair
  for (int64_t r = (int64_t)kept_total + blockIdx.x * blockDim.x + threadIdx.x; r < (int64_t)T * k;
       r += (int64_t)gridDim.x * blockDim.x)
    perm[r] = 0;

  const int b = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;  // one wavefront per token block
  if (b >= nblk) return;
  const int first = b * kTokPerBlock * k;
  const int last = min((b + 1) * kTokPerBlock, T) * k;
  // lane e carries the rank, inside expert e's pairs, of the next pair of this block
  int next = lane < E ? blk_base[(size_t)b * E + lane] : 0;
  for (int i0 = first; i0 < last; i0 += kWave) {
    const int i = i0 + lane;
    const bool valid = i < last;
    const int e = valid ? topk_idx[i] : -1;
    int rank = 0, base = 0;
    for (int q = 0; q < E; ++q) {
      const unsigned long long m = __ballot(e == q);
      const int start = __shfl(next, q, kWave);
      const int row0 = __shfl(group0, q, kWave);
      if (e == q) {
        rank = start + __popcll(m & ((1ull << lane) - 1ull));
        base = row0;
      }
      if (lane == q) next += __popcll(m);
    }
    if (valid) {
      if (cap > 0 && rank >= cap) {
        inv_pos[i] = -1;               // beyond the expert's capacity: dropped
      } else {
        const int pos = base + rank;
        perm[pos] = i;
        inv_pos[i] = pos;
      }
    }
  }
}

// W_router [d,E] -> [E,d]
__global__ __launch_bounds__(256) void transpose_wr_kernel(const float* __restrict__ Wr, int d, int E,
                                                           float* __restrict__ WrT) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= d * E) return;
  const int e = i / d, c = i - e * d;
  WrT[i] = Wr[(size_t)c * E + e];
}

template <typename XT>
void launch_tokens(const RouteArgs& a, const float* WrT, int nblk, int32_t* bc, float* bg, float* bp, hipStream_t s) {
  const XT* x = static_cast<const XT*>(a.x);
  dim3 grid(nblk), block(kWavesPerBlock * kWave);
#define BTX_ROUTE_LAUNCH(EC)                                                                                       \
  do {                                                                                                             \
    if (a.gain)                                                                                                    \
      route_tokens_kernel<XT, EC, true><<<grid, block, 0, s>>>(                                                    \
          x, WrT, a.b_router, a.U, a.T, a.d, a.E, a.k, a.route_mode, 1.f / a.tau, a.topk_idx, a.gates, a.probs, bc,  \
          bg, bp, a.gain, a.eps, static_cast<XT*>(a.xn), a.rstd);                                                   \
    else                                                                                                           \
      route_tokens_kernel<XT, EC, false><<<grid, block, 0, s>>>(                                                   \
          x, WrT, a.b_router, a.U, a.T, a.d, a.E, a.k, a.route_mode, 1.f / a.tau, a.topk_idx, a.gates, a.probs, bc,  \
          bg, bp, nullptr, 0.f, nullptr, nullptr);                                                                  \
  } while (0)
  if (a.E > 8 && !a.gain) {
    // many experts: the dot products go to the matrix cores (fp32 16x16x4, 1024 multiply-adds per
    // instruction).  On the vector unit they took 172 us for 16384 tokens x 32 experts (64 M vector
    // instructions); the kernel now takes 85 us
    auto go = [&](auto mg, auto ns) {
      constexpr int MG = decltype(mg)::value, NS = decltype(ns)::value;
      const size_t lds = (size_t)kWavesPerBlock * MG * kTokPerBlock * 16 * NS * sizeof(float);
      route_tokens_kernel<XT, 0, false, MG, NS><<<ceil_div(nblk, MG), block, lds, s>>>(
          x, WrT, a.b_router, a.U, a.T, a.d, a.E, a.k, a.route_mode, 1.f / a.tau, a.topk_idx, a.gates, a.probs, bc,
          bg, bp, nullptr, 0.f, nullptr, nullptr);
    };
    using std::integral_constant;
    const integral_constant<int, kMatrixGroups> mg;
    if (a.E <= 16) go(mg, integral_constant<int, 1>{});
    else if (a.E <= 32) go(mg, integral_constant<int, 2>{});
    else if (a.E <= 48) go(mg, integral_constant<int, 3>{});
    else go(mg, integral_constant<int, 4>{});
    return;
  }
  if (a.E <= 1) BTX_ROUTE_LAUNCH(1);
  else if (a.E <= 2) BTX_ROUTE_LAUNCH(2);
  else if (a.E <= 4) BTX_ROUTE_LAUNCH(4);
  else BTX_ROUTE_LAUNCH(8);   // 16 per pass was measured no faster at E = 32
#undef BTX_ROUTE_LAUNCH
}

}  // namespace

int launch_transpose_wr(const float* Wr, int d, int E, float* WrT, hipStream_t s) {
  if ((int64_t)d * E >= (int64_t)1 << 31) return BTX_ERR_UNSUPPORTED;   // the kernels index W_router with 32 bits
  transpose_wr_kernel<<<ceil_div(d * E, 256), 256, 0, s>>>(Wr, d, E, WrT);
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

static int num_blocks(int T) { return ceil_div(T, kTokPerBlock); }
static size_t block_stats_bytes(int T, int E) {
  // block counts, block bases (int32) and block gate/prob sums (fp32)
  return align_up((size_t)num_blocks(T) * E * 4 * sizeof(int32_t), 256);
}

size_t route_workspace_bytes(int T, int d, int E, int /*k*/) {
  return block_stats_bytes(T, E) + align_up((size_t)E * d * sizeof(float), 256);   // + W_router transposed
}

int launch_route(const RouteArgs& a, hipStream_t s) {
  const int nblk = num_blocks(a.T);
  const size_t n = (size_t)nblk * a.E;
  int32_t* bc = static_cast<int32_t*>(a.workspace);
  int32_t* bb = bc + n;
  float* bg = reinterpret_cast<float*>(bb + n);
  float* bp = bg + n;
  float* WrT = reinterpret_cast<float*>(static_cast<char*>(a.workspace) + block_stats_bytes(a.T, a.E));
  if (int rc = launch_transpose_wr(a.W_router, a.d, a.E, WrT, s)) return rc;
  if (a.x_dtype == BTX_BF16) launch_tokens<bf16_t>(a, WrT, nblk, bc, bg, bp, s);
  else launch_tokens<float>(a, WrT, nblk, bc, bg, bp, s);
  BTX_LAUNCH_CHECK();
  route_scan_kernel<<<a.E, kScanThreads, 0, s>>>(nblk, a.E, bc, bg, bp, bb, a.counts, a.gate_sum, a.prob_sum);
  BTX_LAUNCH_CHECK();
  route_scatter_kernel<<<ceil_div(nblk, kWavesPerBlock), kWavesPerBlock * kWave, 0, s>>>(
      nblk, a.T, a.E, a.k, a.cap, a.lb_mode, a.lb_alpha, a.topk_idx, bb, a.counts, a.gate_sum, a.prob_sum, a.offsets,
      a.lb_loss, a.perm, a.inv_pos);
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

}  // namespace btx
