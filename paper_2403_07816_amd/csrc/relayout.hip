// MiX construction utilities (Sec. 3.3 "Splitting Experts" and "Blending Experts"): one-off
// re-indexing of stacked expert weights, a plain HBM-bound copy (every byte read once and
// written once).  Both cut each FF along d_ff into chunks of fc hidden units:
//   split  (C chunks):  expert i*C+c  = chunk c of FF i                      (N*C experts of width f/C)
//   blend  (N chunks):  expert n      = chunk n of FF 0, of FF 1, ... in turn (N experts of width f)
// W1 / W3 [.,d,f] are cut by columns, W2 [.,f,d] by rows.  The copy is organised as row
// segments (fc elements of a W1/W3 row, or a whole W2 row), one wavefront per segment.
#include "common.h"

namespace btx {
namespace {

struct MixArgs {
  int mode, N, C, d, fc;        // C = chunks per source FF (split: C, blend: N)
  int cpo;                      // chunks per output expert (split: 1, blend: N)
  int n_out;                    // output experts
};

// VT: copy unit (16 bytes when the segments allow it, else one element)
template <typename VT, bool BY_ROWS>
__global__ __launch_bounds__(256) void mix_copy_kernel(const VT* __restrict__ src, VT* __restrict__ dst, MixArgs a,
                                                       int seg_units, int chunk_rows, int64_t n_seg) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t s = (int64_t)blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
  if (s >= n_seg) return;
  // segment -> (output expert o, chunk slot q of that expert, row r inside the chunk's row range)
  const int r = (int)(s % chunk_rows);
  const int q = (int)((s / chunk_rows) % a.cpo);
  const int o = (int)(s / ((int64_t)chunk_rows * a.cpo));
  const int se = a.mode == BTX_MIX_SPLIT ? o / a.C : q;     // source FF
  const int sc = a.mode == BTX_MIX_SPLIT ? o % a.C : o;     // chunk of that FF
  int64_t so, dof;                                          // offsets in copy units
  if (BY_ROWS) {   // W2: chunk = fc consecutive rows of d elements; a segment is one row
    so = ((int64_t)se * a.C * a.fc + (int64_t)sc * a.fc + r) * seg_units;
    dof = ((int64_t)o * a.cpo * a.fc + (int64_t)q * a.fc + r) * seg_units;
  } else {         // W1 / W3: chunk = fc consecutive columns; a segment is that part of row r
    so = (((int64_t)se * a.d + r) * a.C + sc) * seg_units;
    dof = (((int64_t)o * a.d + r) * a.cpo + q) * seg_units;
  }
  for (int c = lane; c < seg_units; c += kWave) dst[dof + c] = src[so + c];
}

template <typename VT>
int launch_one(const void* src, void* dst, const MixArgs& a, bool by_rows, int seg_units, hipStream_t s) {
  const int chunk_rows = by_rows ? a.fc : a.d;
  const int64_t n_seg = (int64_t)a.n_out * a.cpo * chunk_rows;
  if (n_seg == 0) return BTX_OK;
  const int64_t blocks = (n_seg + 3) / 4;
  if (blocks > 0x7fffffff) return BTX_ERR_INVALID_ARG;
  if (by_rows)
    mix_copy_kernel<VT, true><<<(unsigned)blocks, 256, 0, s>>>(static_cast<const VT*>(src), static_cast<VT*>(dst), a,
                                                               seg_units, chunk_rows, n_seg);
  else
    mix_copy_kernel<VT, false><<<(unsigned)blocks, 256, 0, s>>>(static_cast<const VT*>(src), static_cast<VT*>(dst), a,
                                                                seg_units, chunk_rows, n_seg);
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

}  // namespace

int launch_mix_experts(const void* W1, const void* W3, const void* W2, int dtype, int N, int d, int f, int mode, int C,
                       void* oW1, void* oW3, void* oW2, hipStream_t s) {
  const int es = dtype == BTX_BF16 ? 2 : 4;
  MixArgs a;
  a.mode = mode; a.N = N; a.d = d;
  a.C = mode == BTX_MIX_SPLIT ? C : N;
  a.fc = f / a.C;
  a.cpo = mode == BTX_MIX_SPLIT ? 1 : N;
  a.n_out = mode == BTX_MIX_SPLIT ? N * C : N;
  auto one = [&](const void* src, void* dst, bool by_rows) -> int {
    const int seg_elems = by_rows ? d : a.fc;
    const bool vec = (seg_elems * es) % 16 == 0 && !(((uintptr_t)src | (uintptr_t)dst) & 15);
    if (vec) return launch_one<u32x4>(src, dst, a, by_rows, seg_elems * es / 16, s);
    if (es == 2) return launch_one<uint16_t>(src, dst, a, by_rows, seg_elems, s);
    return launch_one<uint32_t>(src, dst, a, by_rows, seg_elems, s);
  };
  if (int rc = one(W1, oW1, false)) return rc;
  if (int rc = one(W3, oW3, false)) return rc;
  return one(W2, oW2, true);
}

}  // namespace btx
