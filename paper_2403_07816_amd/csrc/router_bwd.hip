// Backward of the router and the last step of dX (chain rule on the routing function of
// Sec. 3.2 / 3.3 with the expert selection held fixed, plus the gradient of the
// load-balancing loss of Sec. 3.3).  All reductions run in a fixed order; no atomics.
//
//   router_ds       one wavefront per token, lane e = expert e: dg (summed partials of
//                   <dY, expert output>), gate Jacobian, load-balancing term -> ds[T,E]
//   dwr_partial     dW_router = x^T ds as per-token-chunk partial sums
//   dwr_reduce      fixed-order sum of the partials (and of db_router)
//   dx_finish       dX[t] = sum_j dxs[inv_pos[t,j]] + ds[t] W_router^T, W_router slice kept in registers
// The rows these kernels stream (x, dxs, dX) are touched once per kernel and go past the caches.
// dwr_partial and dx_finish work expert-major (partials [chunk][E][d], W_router as [E,d]): a
// lane's 8 columns of one expert are then 32 contiguous bytes instead of 8 pieces E floats apart.
#include "common.h"

namespace btx {
namespace {

constexpr int kColsPerThread = 8;

__global__ __launch_bounds__(256) void router_ds_kernel(
    int T, int E, int k, int mode, int lb_mode, float lb_alpha, float lam, unsigned flags,
    const float* __restrict__ noise, float inv_tau,
    const int32_t* __restrict__ topk_idx, const float* __restrict__ gates, const float* __restrict__ probs,
    const int32_t* __restrict__ inv_pos, const float* __restrict__ gate_sum, const float* __restrict__ prob_sum,
    const int32_t* __restrict__ counts, const float* __restrict__ dg_part, int n_part, float* __restrict__ ds) {
  const int lane = threadIdx.x & (kWave - 1);
  const int t = blockIdx.x * 4 + threadIdx.x / kWave;
  if (t >= T) return;
  const bool live = lane < E;
  const float lbc = lb_alpha * (float)E / (float)T;
  const float pbar = live ? prob_sum[lane] / (float)T : 0.f;
  // lane j < k: slot j of this token
  int my_e = -1;
  float g = 0.f, dg = 0.f;
  if (lane < k) {
    my_e = topk_idx[(size_t)t * k + lane];
    g = gates[(size_t)t * k + lane];
    const int r = inv_pos[(size_t)t * k + lane];
    if (r >= 0) {                            // a dropped pair produced no output: dg = 0
      const float* part = dg_part + (size_t)r * n_part;
      for (int p = 0; p < n_part; ++p) dg += part[p];
    }
  }
  if (flags & BTX_FLAG_LB_GRAD_THROUGH_U) {
    const float pb = __shfl(pbar, my_e < 0 ? 0 : my_e, kWave);
    if (lane < k) dg += lam * lbc * pb;
  }
  const float p = live ? probs[(size_t)t * E + lane] : 0.f;
  float dsv = 0.f;
  if (mode == BTX_ROUTE_TOPK_RENORM) {
    const float inner = wave_sum(g * dg);  // lanes >= k contribute 0
    const float mine = g * (dg - inner);
    for (int j = 0; j < k; ++j) {
      const int e = __shfl(my_e, j, kWave);
      const float v = __shfl(mine, j, kWave);
      if (lane == e) dsv = v;
    }
  } else if (mode == BTX_ROUTE_GUMBEL_TOP1) {
    // gate = y_e, y = softmax((logits + noise) / tau), rebuilt from log p (= logits up to a
    // constant per token): d gate / d logit_j = y_e (delta_ej - y_j) / tau
    const int e = __shfl(my_e, 0, kWave);
    const float dg0 = __shfl(dg, 0, kWave);
    const float v = live ? (__logf(p) + noise[(size_t)t * E + lane]) * inv_tau : -INFINITY;
    const float vmax = wave_max(v);
    const float z = live ? __expf(v - vmax) : 0.f;
    const float y = z / wave_sum(z);
    const float ye = __shfl(y, e, kWave);
    dsv = dg0 * ye * ((lane == e ? 1.f : 0.f) - y) * inv_tau;
  } else {
    const int e = __shfl(my_e, 0, kWave);
    const float dg0 = __shfl(dg, 0, kWave);
    const float pe = __shfl(p, e, kWave);
    dsv = dg0 * pe * ((lane == e ? 1.f : 0.f) - p);
  }
  if (lam != 0.f) {
    const float u = !live ? 0.f
                    : lb_mode == BTX_LB_TOKEN_FRAC ? (float)counts[lane] / ((float)T * (float)k)
                                                   : gate_sum[lane] / (float)T;
    const float up = wave_sum(u * p);
    dsv += lam * lbc * p * (u - up);
  }
  if (live) ds[(size_t)t * E + lane] = dsv;
}

// grid: (token chunks of CHUNK, column blocks of 256*8, expert passes of KEC).  The partial sums
// are stored expert-major ([chunk][E][d]): a thread's 8 columns of an expert are 32 contiguous bytes.
template <typename XT, int KEC, int CHUNK>
__global__ __launch_bounds__(256) void dwr_partial_kernel(const XT* __restrict__ x, const float* __restrict__ ds, int T,
                                                          int d, int E, float* __restrict__ part,
                                                          float* __restrict__ db_part) {
  __shared__ float s_ds[CHUNK][KEC];
  const int t0 = blockIdx.x * CHUNK, e0 = blockIdx.z * KEC;
  const int nt = min(CHUNK, T - t0);
  for (int i = threadIdx.x; i < CHUNK * KEC; i += 256) {
    const int q = i / KEC, j = i % KEC;
    s_ds[q][j] = (q < nt && e0 + j < E) ? ds[(size_t)(t0 + q) * E + e0 + j] : 0.f;
  }
  __syncthreads();
  const int c0 = (blockIdx.y * 256 + threadIdx.x) * kColsPerThread;
  if (c0 < d) {
    float acc[KEC][kColsPerThread] = {};
    // 4 token rows in flight; rows past the chunk's end are read from a clamped address and
    // meet the zeros of s_ds
    for (int q = 0; q < nt; q += 4) {
      float xv[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) RowVec<XT, 8>::ld_stream(x + (size_t)min(t0 + q + u, T - 1) * d + c0, xv[u]);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < KEC; ++j) {
          const float w = s_ds[q + u][j];
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[j][i] = fmaf(xv[u][i], w, acc[j][i]);
        }
    }
#pragma unroll
    for (int j = 0; j < KEC; ++j)
      if (e0 + j < E) RowVec<float, 8>::st(part + ((size_t)blockIdx.x * E + e0 + j) * d + c0, acc[j]);
  }
  if (blockIdx.y == 0 && threadIdx.x < KEC && e0 + threadIdx.x < E) {
    float a = 0.f;
    for (int q = 0; q < nt; ++q) a += s_ds[q][threadIdx.x];
    db_part[(size_t)blockIdx.x * E + e0 + threadIdx.x] = a;
  }
}

// 64 sums per block, taken in the partials' expert-major order (coalesced reads) and written to
// dW_router's [d,E] place; 16 thread groups each add every 16th partial, then the 16 sums are
// added in group order (a fixed order, like everything else here).
constexpr int kRedGroups = 16;
__global__ __launch_bounds__(64 * kRedGroups) void dwr_reduce_kernel(const float* __restrict__ part,
                                                                      const float* __restrict__ db_part, int nchunk,
                                                                      int d, int E, float* __restrict__ dWr,
                                                                      float* __restrict__ db) {
  __shared__ float s_sum[kRedGroups][64];
  const int o = threadIdx.x % 64, grp = threadIdx.x / 64;
  const int dE = d * E;
  const int i = blockIdx.x * 64 + o;
  s_sum[grp][o] = i < dE ? strided_row_sum(part, dE, i, grp, kRedGroups, nchunk) : 0.f;
  __syncthreads();
  if (grp == 0 && i < dE) {
    float a = 0.f;
#pragma unroll
    for (int g = 0; g < kRedGroups; ++g) a += s_sum[g][o];
    const int e = i / d, c = i - e * d;
    dWr[(size_t)c * E + e] = a;
  }
  if (db && blockIdx.x == 0 && threadIdx.x < E) {
    float b = 0.f;
    for (int c = 0; c < nchunk; ++c) b += db_part[(size_t)c * E + threadIdx.x];
    db[threadIdx.x] = b;
  }
}

// dX[t] = sum_j dxs[inv_pos[t,j]] + ds[t] W_router^T.  A wavefront owns 512 columns (8 per lane)
// for TOK tokens, 4 of them in flight at a time; its slice of W_router (read from the [E,d]
// copy) stays in registers when E <= EC, so the kernel streams dxs and dX and little else.
// With more experts the slice is reloaded in pieces of EC per 4 tokens (cache hits): 4 columns
// per lane with the whole slice resident was measured slower (8-byte row loads).
template <typename XT, int EC, int TOK>
__global__ __launch_bounds__(256) void dx_finish_kernel(const XT* __restrict__ dxs, const int32_t* __restrict__ inv_pos,
                                                        const float* __restrict__ ds, const float* __restrict__ WrT,
                                                        int T, int d, int E, int k, XT* __restrict__ dX) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int c0 = ((blockIdx.y * 4 + wave) * kWave + lane) * 8;
  const int t0 = blockIdx.x * TOK;
  if (c0 >= d) return;                      // no cross-lane traffic below
  const int n_ch = (E + EC - 1) / EC;
  float wr[EC][8];
  auto load_wr = [&](int e0) {
#pragma unroll
    for (int j = 0; j < EC; ++j) {
      if (e0 + j < E) {
        RowVec<float, 8>::ld(WrT + (size_t)(e0 + j) * d + c0, wr[j]);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) wr[j][i] = 0.f;
      }
    }
  };
  if (n_ch == 1) load_wr(0);
  for (int tq = 0; tq < TOK; tq += 4) {
    float acc[4][8] = {};
    // slot by slot, the four tokens' rows in flight together; a dropped pair (or a token past
    // the end) reads row 0 and adds zero
#pragma unroll 2
    for (int j = 0; j < k; ++j) {
      float v[4][8];
      bool have[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int t = t0 + tq + q;
        const int r = t < T ? inv_pos[(size_t)t * k + j] : -1;
        have[q] = r >= 0;
        RowVec<XT, 8>::ld_stream(dxs + (size_t)max(r, 0) * d + c0, v[q]);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[q][i] += have[q] ? v[q][i] : 0.f;
    }
    for (int ch = 0; ch < n_ch; ++ch) {
      if (n_ch > 1) load_wr(ch * EC);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int t = t0 + tq + q;
        if (t >= T) break;
#pragma unroll
        for (int j = 0; j < EC; ++j) {
          const int e = ch * EC + j;
          const float w = e < E ? ds[(size_t)t * E + e] : 0.f;
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[q][i] = fmaf(w, wr[j][i], acc[q][i]);
        }
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (t0 + tq + q < T) RowVec<XT, 8>::st_stream(dX + (size_t)(t0 + tq + q) * d + c0, acc[q]);
  }
}

// The same for 9 to 32 experts, where the slice of W_router no longer fits the registers and reloading it
// per 4 tokens (from the caches) cost 110 of the kernel's 337 us at 32 experts: the 8 wavefronts of a
// workgroup share one slice of kDxCols columns, staged once in LDS ([expert][half][lane] 16-byte
// pieces, so that consecutive lanes read consecutive pieces), and split the workgroup's tokens, 4 in
// flight per wavefront.
constexpr int kDxCols = kWave * 8;                      // columns of a workgroup: 8 per lane
constexpr int kDxWaves = 8;
constexpr int kDxLdsMaxE = 32;                          // 32 experts x 512 columns x 4 bytes = 64 KB
template <typename XT>
__global__ __launch_bounds__(kDxWaves* kWave) void dx_finish_lds_kernel(const XT* __restrict__ dxs,
                                                                        const int32_t* __restrict__ inv_pos,
                                                                        const float* __restrict__ ds,
                                                                        const float* __restrict__ WrT, int T, int d, int E,
                                                                        int k, int tok_per_block, XT* __restrict__ dX) {
  extern __shared__ f32x4 s_wr[];                       // [E][2][kWave]
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int cb = blockIdx.y * kDxCols, c0 = cb + lane * 8;
  for (int i = threadIdx.x; i < E * (kDxCols / 4); i += kDxWaves * kWave) {
    const int e = i / (kDxCols / 4), c4 = i % (kDxCols / 4);      // 16-byte piece c4 of expert e's slice
    f32x4 w{0.f, 0.f, 0.f, 0.f};
    if (cb + 4 * c4 < d) w = *reinterpret_cast<const f32x4*>(WrT + (size_t)e * d + cb + 4 * c4);
    s_wr[(e * 2 + (c4 & 1)) * kWave + (c4 >> 1)] = w;
  }
  __syncthreads();
  if (c0 >= d) return;                      // no barrier and no cross-lane traffic below
  const int t_end = min(T, (int)(blockIdx.x + 1) * tok_per_block);
  for (int t0 = blockIdx.x * tok_per_block + wave * 4; t0 < t_end; t0 += kDxWaves * 4) {
    float acc[4][8] = {};
    // slot by slot, the four tokens' rows in flight together; a dropped pair (or a token past
    // the end) reads row 0 and adds zero
#pragma unroll 2
    for (int j = 0; j < k; ++j) {
      float v[4][8];
      bool have[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int t = t0 + q;
        const int r = t < t_end ? inv_pos[(size_t)t * k + j] : -1;
        have[q] = r >= 0;
        RowVec<XT, 8>::ld_stream(dxs + (size_t)max(r, 0) * d + c0, v[q]);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[q][i] += have[q] ? v[q][i] : 0.f;
    }
    for (int e = 0; e < E; ++e) {
      const f32x4 wa = s_wr[(e * 2) * kWave + lane], wb = s_wr[(e * 2 + 1) * kWave + lane];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float w = ds[(size_t)min(t0 + q, T - 1) * E + e];   // uniform across the wavefront
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[q][i] = fmaf(w, wa[i], acc[q][i]);
          acc[q][4 + i] = fmaf(w, wb[i], acc[q][4 + i]);
        }
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (t0 + q < t_end) RowVec<XT, 8>::st_stream(dX + (size_t)(t0 + q) * d + c0, acc[q]);
  }
}

}  // namespace

// token chunk of the dW_router partial sums: longer chunks for many experts keep the partials
// (chunks * d * E floats) small next to x
static int tok_chunk(int E) { return E <= 8 ? 64 : 128; }
static int n_chunks(int T, int E) { return ceil_div(T, tok_chunk(E)); }

size_t router_bwd_workspace_bytes(int T, int d, int E) {
  const size_t ds = align_up((size_t)T * E * sizeof(float), 256);
  const size_t part = align_up((size_t)n_chunks(T, E) * d * E * sizeof(float), 256);
  const size_t dbp = align_up((size_t)n_chunks(T, E) * E * sizeof(float), 256);
  const size_t wrt = align_up((size_t)E * d * sizeof(float), 256);
  return ds + part + dbp + wrt;
}

int launch_router_bwd(const RouterBwdArgs& a, hipStream_t s) {
  const int nch = n_chunks(a.T, a.E);
  char* w = static_cast<char*>(a.workspace);
  float* ds = reinterpret_cast<float*>(w);
  w += align_up((size_t)a.T * a.E * sizeof(float), 256);
  float* part = reinterpret_cast<float*>(w);
  w += align_up((size_t)nch * a.d * a.E * sizeof(float), 256);
  float* dbp = reinterpret_cast<float*>(w);
  w += align_up((size_t)nch * a.E * sizeof(float), 256);
  float* WrT = reinterpret_cast<float*>(w);

  if (int rc = launch_transpose_wr(a.W_router, a.d, a.E, WrT, s)) return rc;
  router_ds_kernel<<<ceil_div(a.T, 4), 256, 0, s>>>(a.T, a.E, a.k, a.route_mode, a.lb_mode, a.lb_alpha, a.lb_grad_scale,
                                                   a.flags, a.noise, a.noise ? 1.f / a.tau : 1.f, a.topk_idx, a.gates,
                                                   a.probs, a.inv_pos, a.gate_sum,
                                                   a.prob_sum, a.counts, a.dg_part, a.n_part, ds);
  BTX_LAUNCH_CHECK();
  auto typed = [&](auto tag) {
    using XT = decltype(tag);
    const XT* x = static_cast<const XT*>(a.x);
    const int col_blocks = ceil_div(a.d, 256 * kColsPerThread);
    if (a.E <= 8)
      dwr_partial_kernel<XT, 8, 64><<<dim3(nch, col_blocks, 1), 256, 0, s>>>(x, ds, a.T, a.d, a.E, part, dbp);
    else
      dwr_partial_kernel<XT, 16, 128><<<dim3(nch, col_blocks, ceil_div(a.E, 16)), 256, 0, s>>>(x, ds, a.T, a.d, a.E,
                                                                                             part, dbp);
  };
  if (a.dtype == BTX_BF16) typed(bf16_t{});
  else typed(float{});
  BTX_LAUNCH_CHECK();
  dwr_reduce_kernel<<<ceil_div(a.d * a.E, 64), 64 * kRedGroups, 0, s>>>(part, dbp, nch, a.d, a.E, a.dW_router,
                                                                       a.db_router);
  BTX_LAUNCH_CHECK();
  auto dx_launch = [&](auto tag) {
    using XT = decltype(tag);
    const XT* dxs = static_cast<const XT*>(a.dxs);
    XT* dX = static_cast<XT*>(a.dX);
#define BTX_DX_LAUNCH(EC, TOK)                                                                                       \
  dx_finish_kernel<XT, EC, TOK><<<dim3(ceil_div(a.T, TOK), ceil_div(a.d, 4 * kWave * 8)), 256, 0, s>>>(dxs, a.inv_pos, \
                                                                                                      ds, WrT, a.T, a.d, \
                                                                                                      a.E, a.k, dX)
    if (a.E <= 4) BTX_DX_LAUNCH(4, 16);
    else if (a.E <= 8) BTX_DX_LAUNCH(8, 16);
    else if (a.E <= kDxLdsMaxE) {
      const int tok = 128;                              // tokens per workgroup: the slice is staged once for them
      dx_finish_lds_kernel<XT><<<dim3(ceil_div(a.T, tok), ceil_div(a.d, kDxCols)), kDxWaves * kWave,
                                 (size_t)a.E * kDxCols * sizeof(float), s>>>(dxs, a.inv_pos, ds, WrT, a.T, a.d, a.E, a.k,
                                                                              tok, dX);
    } else BTX_DX_LAUNCH(16, 32);
#undef BTX_DX_LAUNCH
  };
  if (a.dtype == BTX_BF16) dx_launch(bf16_t{});
  else dx_launch(float{});
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

}  // namespace btx
