// bf16 MFMA grouped GEMMs of the expert FFNs (the SwiGLU feed-forward FF_i of the layer
// equation in Sec. 3.2, forward and backward), written for gfx950.
//
// One kernel template covers the six products of the layer:
//   UP      h1 = xs W1_e, h3 = xs W3_e, act = silu(h1)*h3          (two B panels share one A tile)
//   DOWN    y = act W2_e
//   BWD_ACT D = dys W2_e^T with the SwiGLU backward fused into the epilogue
//   BWD_DX  dxs = dh1 W1_e^T + dh3 W3_e^T                           (two K passes, one accumulator)
//   DW13    dW1_e = xs_e^T dh1_e, dW3_e = xs_e^T dh3_e              (K = the expert's ragged row count)
//   DW2     dW2_e = ga_e^T dys_e
//
// Structure of a workgroup (WM x WN wavefronts, BM x BN x BK tile):
//   * global -> LDS copies are direct (global_load_lds, 16 bytes per lane, no VGPR staging),
//     three stages of the A tile and two of the B tile; the two wavefronts of a SIMD alternate
//     between a memory phase and a compute phase (see the main loop);
//   * an operand whose K index is contiguous in memory is stored [row][BK] with a 16-byte
//     chunk XOR swizzle and read with ds_read_b128; an operand whose K index is strided
//     (the weights in UP and DOWN, dh1/dh3 in DW13) is stored as it lies in memory, [BK][cols],
//     and read with the transposing ds_read_b64_tr_b16; x, dY and ga reach the dW products
//     transposed and zero-padded per expert (x and dY from a gather kernel, ga written that way
//     by BWD_ACT's epilogue).  The swizzles are applied by choosing which
//     global chunk each lane fetches, since a direct copy fixes the LDS position per lane;
//   * v_mfma_f32_16x16x32_bf16 (on this chip it sustains a seventh more than the 32x32x16 form
//     under the same power limit) with the roles of the operands swapped (the N-side fragment
//     is passed first), so that each lane ends up with 4 consecutive output columns of one row
//     and stores 8 bytes at a time;
//   * grouped rows: tiles are enumerated per expert on the device (no host sync); a tile past
//     the last one exits.  Rows beyond a group's end are loaded from a clamped address and
//     never stored.  A last k tile that is half empty (K = 32 mod 64) has its copies re-pointed
//     at valid data and the A fragments of its empty half zeroed in registers;
//   * UP, DOWN and BWD_DX: the tiles of a partly filled last round of workgroups are cut along K into
//     up to 8 slices whose fp32 accumulators a second small kernel adds in ascending order and stores
//     (UP: with the SwiGLU applied to the sums), so that the round fills the chip (Gemm::split_plan).
#include "gemm_mfma.h"
#include "gemm_generic.h"
#include <type_traits>

namespace btx {
namespace {

// supertile: row tiles x column tiles that run concurrently chip-wide, and the XCDs along its
// rows (8 / kXcdM along its columns)
constexpr int kSupM = 16, kSupN = 16, kXcdM = 4;
constexpr int kSplitMaxSlices = 8;
constexpr int kSplitMaxCus = 256;   // compute units the K-cut of a last round is laid out for (see Gemm::split_plan)
static_assert(kSupM % kXcdM == 0 && 8 % kXcdM == 0 && kSupN % (8 / kXcdM) == 0 && (kSupM * kSupN) % 8 == 0, "supertile");

enum Mode { UP = 0, DOWN = 1, BWD_ACT = 2, BWD_DX = 3, DW13 = 4, DW2 = 5 };

struct MArgs {
  const bf16_t* A0; const bf16_t* A1;   // A1: second K pass (BWD_DX)
  const bf16_t* B0; const bf16_t* B1;   // B1: second panel (UP, DW13) or second K pass (BWD_DX)
  void* C0; void* C1; void* C2;         // UP: h1,h3,act; BWD_ACT: dh1,dh3 (ga goes to T2); DW13: dW1,dW3; else C0
  const bf16_t* H1; const bf16_t* H3;   // BWD_ACT inputs
  bf16_t* T2; int ldt;                  // BWD_ACT: ga transposed [N][ldt], experts' rows padded to 64 (NULL: not wanted)
  const float* gates; const int32_t* perm; float* dg_part; int n_part;
  const int32_t* a_perm; int a_k;       // UP / BWD_ACT: A row r is row a_perm[r] / a_k of A0 (NULL: row r)
  const int32_t* offsets; int E;
  int M, N, K;                          // grouped-M: M unused; grouped-K: K unused
  int lda, ldb, ldc;                    // leading dimensions in elements
  int64_t strideB_e, strideC_e;         // per-expert strides in elements
  int R;                                // total grouped rows
  int tiles_n, tiles_m;                 // tile grid (tiles_m is the worst case for grouped-M)
  int c_is_f32;
  int blocks_per_e;                     // grouped-K: block ids per expert (a multiple of 8)
  int total_ids;                        // tile ids of the launch (a few name no tile: padding of the id space)
  // UP / DOWN / BWD_DX: the tiles of the last, partly filled round are cut along K (see Gemm::split_plan)
  f32x4* partial; int cus;              // fp32 accumulators of the slices (NULL: never cut); compute units
};

__device__ __forceinline__ void wait_vmcnt(int n) {
  // gfx9 encoding: vmcnt = bits [3:0] and [15:14]; expcnt [6:4] and lgkmcnt [11:8] left at max
  switch (n) {
    case 0: __builtin_amdgcn_s_waitcnt(0x0F70); break;
    case 4: __builtin_amdgcn_s_waitcnt(0x0F74); break;
    case 6: __builtin_amdgcn_s_waitcnt(0x0F76); break;
    case 8: __builtin_amdgcn_s_waitcnt(0x0F78); break;
    case 12: __builtin_amdgcn_s_waitcnt(0x0F7C); break;
    case 16: __builtin_amdgcn_s_waitcnt(0x4F70); break;
    case 24: __builtin_amdgcn_s_waitcnt(0x4F78); break;
    default: __builtin_amdgcn_s_waitcnt(0x0F70); break;
  }
}

// Direct global -> LDS copy of 16 bytes per lane: lane l's data lands at lds_base + 16*l.
// Written as inline assembly so that the compiler does not serialise later LDS reads of
// *other* stages behind it (it cannot tell the stages apart and would wait for vmcnt(0));
// completion is awaited explicitly with wait_vmcnt() before the barrier that publishes a tile.
// `base` and `lds_base` are wave-uniform by construction; readfirstlane states that to the
// compiler where its divergence analysis cannot see it.
__device__ __forceinline__ void copy16_to_lds(const void* base, uint32_t byte_off, uint32_t lds_base) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  // readfirstlane returns int: go through uint32_t so that the halves are not sign-extended
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)p);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(p >> 32));
  const uint64_t sp = (uint64_t)lo | ((uint64_t)hi << 32);
  const uint32_t sl = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base);
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(sl), "v"(byte_off), "s"(sp)
               : "memory");
}

// Epilogue staging band: 32 rows of ROWB bytes in LDS, 16-byte chunks XOR-swizzled by row so
// that both the piece writes (PIECE bytes per lane, 32 rows at one column) and the
// row-contiguous 16-byte reads are free of bank conflicts.
template <int ROWB, int PIECE>
__device__ __forceinline__ uint32_t stage_off(int r, int chunk) {
  constexpr int CPR = ROWB / 16, RP = ROWB >= 256 ? 1 : 256 / ROWB, STEP = PIECE / 8;
  return (uint32_t)(r * ROWB + ((chunk ^ (((r / RP) * STEP) & (CPR - 1))) << 4));
}

// The 8-byte pieces that the lanes of a fragment write into (and read from) a staged band would
// meet two-way in the banks: rows r and r+1 (128-byte rows) or r and r+2 (64-byte rows) of a band
// put the same chunk in the same banks.  Those rows keep the two halves of every 16-byte chunk
// swapped, so that 16 lanes cover all 32 banks; whoever moves whole chunks swaps them back.
// BWD_ACT does without: its epilogue is bound by its vector arithmetic (about 3000 instructions
// per wavefront), the swaps would add 256 selects to it and its LDS conflicts cost no time.
template <int ROWB, int ES>
__device__ __forceinline__ uint32_t half_flip(int r) {
  return ES == 2 ? (uint32_t)(((r >> (ROWB >= 128 ? 0 : 1)) & 1) << 3) : 0u;
}
__device__ __forceinline__ u32x4 swap_halves(u32x4 v, bool yes) {
  return yes ? u32x4{v[2], v[3], v[0], v[1]} : v;
}

// Epilogue stores.  STREAM: marked non-temporal, so that the written tile does not push the operand panels
// that the other compute units are streaming out of the XCD's L2.  Measured per product: BWD_ACT (three
// tensors out per tile, the lowest L2 hit rate of the six) -5 %, DOWN -0.3 % (-3.7 % with 32 narrow experts);
// BWD_DX +0.6 % / -2 %, UP and DW13 +1 %: those keep plain stores.
template <bool STREAM, typename V> __device__ __forceinline__ void store_out(V* p, V v) {
  if constexpr (STREAM) __builtin_nontemporal_store(v, p);
  else *p = v;
}

template <int BM, int BN, int BK, int WM, int WN, int NSA, int NSB, int MODE, bool TAIL = false>
struct Gemm {
  // K index contiguous in memory?  A always is.  In the dW products K is the grouped-row index:
  // x (dW1/dW3) and ga, dY (dW2) arrive transposed, [columns][padded rows], every expert's rows
  // starting at a multiple of 64 and zero-filled up to the next one; dh1/dh3 stay row-major.
  static constexpr bool A_KC = true;
  static constexpr bool B_KC = (MODE != UP && MODE != DOWN && MODE != DW13);
  static constexpr bool DUAL = (MODE == UP || MODE == DW13);
  static constexpr bool GROUP_K = (MODE == DW13 || MODE == DW2);
  static constexpr bool STREAM_OUT = (MODE == BWD_ACT || MODE == DOWN);
  static constexpr int NW = WM * WN, NT = NW * kWave;
  static constexpr int TM = BM / WM / 16;                      // 16-row fragments per wavefront
  static constexpr int TN = BN / WN / 16;
  static constexpr int TNH = DUAL ? TN / 2 : TN;
  static constexpr int BNH = DUAL ? BN / 2 : BN;               // output columns per B panel
  static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  // LDS: NSA = 3 stages of the A tile, then NSB = 2 stages of the B tile (the ping-pong schedule)
  static constexpr int B_BASE = NSA * A_BYTES;
  static constexpr int LDS_BYTES = NSA * A_BYTES + NSB * B_BYTES;
  static_assert(NSA == 3 && NSB == 2 && WM * WN == 8 && BK == 64, "the schedule is written for 8 wavefronts, 2 k steps");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
  static constexpr int A_LOADS = A_BYTES / 1024 / NW, B_LOADS = B_BYTES / 1024 / NW;  // per wavefront per tile
  static constexpr int KSTEPS = BK / 32;                       // k steps (one MFMA deep) per tile
  static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tile must split into 1 KB wave copies");
  static_assert(TM >= 2 && TM % 2 == 0 && TN >= 1 && (!DUAL || TN % 2 == 0), "bad wave tiling");

  // ---- LDS addressing ----------------------------------------------------
  // K-contiguous tile: [rows][BK], 16-byte chunks XOR-swizzled by row
  static __device__ __forceinline__ int kc_swz(int row) { return (row >> 1) & 7; }
  // strided-K tile: [BK][COLS], 16-byte chunk index XORed with tr_swz(k): bits 2-3 keep the four
  // k rows of one transposing read apart, bit 1 the two 16-lane groups that share a pass
  static __device__ __forceinline__ int tr_swz(int k) { return ((k & 3) << 2) | (((k >> 3) & 1) << 1); }

  // byte offset inside a wave's copy `seg` (1 KB each) -> global element offset, for both layouts
  template <bool KC, int ROWS_OR_COLS>
  static __device__ __forceinline__ void copy_coords(int seg, int lane, int& major, int& minor_elem) {
    const int o = seg * 1024 + lane * 16;
    if (KC) {
      const int row = o / (BK * 2);
      const int phys = (o % (BK * 2)) / 16;
      major = row;                              // row of the tile (M or N index)
      minor_elem = (phys ^ kc_swz(row)) * 8;    // k offset inside the tile
    } else {
      constexpr int PITCH = ROWS_OR_COLS * 2;
      const int k = o / PITCH;
      const int phys = (o % PITCH) / 16;
      major = k;                                // k row of the tile
      minor_elem = (phys ^ tr_swz(k)) * 8;      // column offset inside the tile
    }
  }

  // fragment of 16 rows x 32 k: lane l holds row l % 16, k = 32 ks + 8 (l / 16) .. + 7
  static __device__ __forceinline__ bf16x8 read_kc(const char* tile, int row, int ks, int lane) {
    const int r = row + (lane & 15);
    const int chunk = 4 * ks + (lane >> 4);
    return *reinterpret_cast<const bf16x8*>(tile + r * (BK * 2) + ((chunk ^ kc_swz(r)) << 4));
  }
  template <int COLS>
  static __device__ __forceinline__ bf16x8 read_tr(const char* tile, int col, int ks, int lane) {
    // a transposing read hands lane 4a+b of a 16-lane group element b of what lanes a, a+4, a+8,
    // a+12 fetched (4 consecutive columns each): lane r fetches k row r/4 at columns 4 (r%4) ..
    const int g = lane >> 4, r = lane & 15;
    const int k = 32 * ks + 8 * g + (r >> 2);
    const int c = col + 4 * (r & 3);
    const int off = k * (COLS * 2) + ((((c >> 3) ^ tr_swz(k)) << 4) | ((c & 7) << 1));
    typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(tile + off));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(tile + off + 4 * COLS * 2));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  }

  // ---- which tile ------------------------------------------------------
  // Workgroups are dealt round-robin to the 8 XCDs (block id mod 8) and start in id order.
  // SM x SN consecutive ids form one supertile of the tile grid, so that the tiles running at
  // any moment share few operand panels chip-wide (little HBM / infinity-cache traffic, short
  // miss latency); inside it XCD x owns a (SM/XM) x (SN/XN) sub-block, so that the panels its
  // CUs stream meet in that XCD's L2.  Only whole supertiles are laid out like this.  The
  // tiles right of and below the last whole supertile form one list (right strip row by row,
  // then the bottom strip column by column) that is cut into 8 equal runs, one per XCD: a
  // ragged edge must not leave some XCDs with fewer tiles than others.  The number of row
  // tiles of the row-grouped products depends on the routing and is counted here.
  struct Tile { int e, row0, row_end, k_begin, k_end, kp_begin, tile_n, exp_row0; };
  // Row-grouped products: the experts' row ranges are looked at by the whole wavefront at once, lane x
  // taking expert x (at most 64): one load and two prefix sums instead of loops of dependent scalar
  // loads over the experts, which with 32 experts took longer than a tenth of a short tile's main loop.
  // (The products grouped along K know their expert from the block id and keep the one short loop.)
  struct Experts {
    int o0, o1, nt, pad, nt_incl, pad_incl, n_rt;
    __device__ __forceinline__ Experts(const MArgs& g, int lane) : o0(0), o1(0), nt(0), pad(0), nt_incl(0), pad_incl(0) {
      n_rt = g.tiles_m;
      if (!GROUP_K) {
        const int xe = min(lane, g.E - 1);
        o0 = g.offsets[xe];
        o1 = g.offsets[xe + 1];
        const int x_n = lane < g.E ? o1 - o0 : 0;
        nt = (x_n + BM - 1) / BM;
        pad = (x_n + 63) & ~63;
        nt_incl = wave_incl_scan_i32(nt, lane);                              // row tiles up to and including expert x
        if (MODE == BWD_ACT) pad_incl = wave_incl_scan_i32(pad, lane);       // padded rows likewise
        n_rt = __builtin_amdgcn_readlane(nt_incl, kWave - 1);
      }
    }
  };
  // tile id -> tile; false: the id names no tile (all 64 lanes must be active)
  static __device__ __forceinline__ bool locate(const MArgs& g, const Experts& x, int id, Tile& t) {
    constexpr int SM = kSupM, SN = kSupN, XM = kXcdM, XN = 8 / XM;
    const int n_rt = x.n_rt;
    const int fr = n_rt / SM, fc = g.tiles_n / SN;     // whole supertile rows / columns
    const int blocks_full = fr * fc * SM * SN;
    int e = 0;
    if (GROUP_K) {
      e = id / g.blocks_per_e;
      id -= e * g.blocks_per_e;
    }
    int tile_m, tile_n;
    if (id < blocks_full) {
      const int sup = id / (SM * SN), r = id % (SM * SN);
      const int xcd = r % 8, slot = r / 8, sub_m = SM / XM, sub_n = SN / XN;
      tile_m = (sup / fc) * SM + (xcd % XM) * sub_m + slot % sub_m;
      tile_n = (sup % fc) * SN + (xcd / XM) * sub_n + slot / sub_m;
    } else {
      const int idl = id - blocks_full;
      const int w = g.tiles_n - fc * SN, h = n_rt - fr * SM;   // strip width / height
      const int n_right = fr * SM * w, n_left = n_right + h * g.tiles_n;
      const int run = (n_left + 7) / 8;
      const int l = (idl % 8) * run + idl / 8;
      if (idl / 8 >= run || l >= n_left) return false;
      if (l < n_right) {
        tile_m = l / w;
        tile_n = fc * SN + l % w;
      } else {
        tile_m = fr * SM + (l - n_right) % h;
        tile_n = (l - n_right) / h;
      }
    }
    t.kp_begin = 0;                                     // first padded row of expert e (transposed operand)
    t.exp_row0 = 0;
    if (GROUP_K) {
      t.row0 = tile_m * BM;
      t.row_end = g.M;
      t.k_begin = g.offsets[e];
      t.k_end = g.offsets[e + 1];
      for (int q = 0; q < e; ++q) t.kp_begin += (g.offsets[q + 1] - g.offsets[q] + 63) & ~63;
    } else {
      // the expert whose row tiles include tile_m: the first lane whose running total exceeds it
      const unsigned long long owners = __ballot(x.nt_incl > tile_m);
      if (owners == 0) return false;                    // past the last row tile of this routing
      e = __ffsll((long long)owners) - 1;
      const int tt = tile_m - (__builtin_amdgcn_readlane(x.nt_incl, e) - __builtin_amdgcn_readlane(x.nt, e));
      t.exp_row0 = __builtin_amdgcn_readlane(x.o0, e);
      t.row0 = t.exp_row0 + tt * BM;
      t.row_end = __builtin_amdgcn_readlane(x.o1, e);
      t.k_begin = 0;
      t.k_end = g.K;
    }
    if (MODE == BWD_ACT)                                // where expert e starts in the transposed, padded output
      t.kp_begin = __builtin_amdgcn_readlane(x.pad_incl, e) - __builtin_amdgcn_readlane(x.pad, e);
    t.e = e;
    t.tile_n = tile_n;
    return true;
  }

  // DOWN and BWD_DX have few, long tiles (16 column tiles): their last round is often a small fraction of
  // the chip (8.25 rounds for the benchmark's top-2 layer, 4.1 for top-1, 2.25 for one sequence), and a
  // tile cannot be cut smaller; UP has 44.3, 22.2 and 11.4 rounds there.  So the tiles of that round are cut
  // along K instead: slice s of a
  // left-over tile runs k tiles [s nk/S, (s+1) nk/S) in a workgroup of its own and leaves its fp32
  // accumulators in `partial`; a second, small kernel adds the S slices of a tile in slice order and stores
  // the result.  No atomics, and the order of every sum is fixed by the shapes and the number of compute
  // units alone.  ids >= total_ids are the workgroups of the slices 1 .. S-1.
  static constexpr bool SPLIT = (MODE == DOWN || MODE == BWD_DX || MODE == UP);
  static constexpr int kMaxSlices = kSplitMaxSlices, kMinSliceTiles = 16, kIdHoles = 8;   // the id space has up to 8 ids past the last tile
  struct SplitPlan { int id_full, n_left, n_slices; };
  static __device__ __forceinline__ SplitPlan split_plan(const MArgs& g, int n_rt) {
    SplitPlan p{0, 0, 1};
    if (!SPLIT || !g.partial) return p;
    const int n_real = n_rt * g.tiles_n;
    p.id_full = n_real / g.cus * g.cus;                 // ids below this fill whole rounds
    const int left = n_real - p.id_full;
    if (left == 0) return p;
    p.n_left = left + kIdHoles;                         // ids id_full .. id_full + n_left - 1 may name a tile
    // as many slices as fill the chip, at most eight, none shorter than kMinSliceTiles k tiles (a slice pays a
    // tile's fixed costs once more, and its accumulators travel through memory)
    const int nk_all = (g.K + BK - 1) / BK * (MODE == BWD_DX ? 2 : 1);
    p.n_slices = max(1, min(min(kMaxSlices, g.cus / left), nk_all / kMinSliceTiles));
    return p;
  }
  // fp32 accumulators of (left-over tile j, slice s), as the wavefronts hold them: [wave][fragment][lane] x 4
  static __device__ __forceinline__ f32x4* partial_slot(const MArgs& g, const SplitPlan& p, int j, int slice) {
    return g.partial + (size_t)(j * p.n_slices + slice) * (NW * TM * TN * kWave);
  }

  // Second kernel of a K-cut product: TM workgroups per left-over tile (one per fragment row of the
  // wavefronts: a single workgroup per tile left most of the chip idle and took 53 us for 72 MB) add the
  // slices' accumulators in slice order and store the tile (same ownership of the elements as in run():
  // fragment (i, j) of a wavefront, lane l = row l % 16, four columns from 4 (l / 16)).
  static __device__ void finish(const MArgs& g) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int wm = wave / WN, wn = wave % WN;
    const Experts experts(g, lane);
    const SplitPlan plan = split_plan(g, experts.n_rt);
    const int j = blockIdx.x / TM, i = blockIdx.x % TM;
    if (plan.n_slices <= 1 || j >= plan.n_left) return;
    Tile tile;
    if (!locate(g, experts, plan.id_full + j, tile)) return;
    const int col0 = tile.tile_n * BNH;
    auto slices_sum = [&](int jj) {
      const size_t at = (size_t)wave * (TM * TN * kWave) + (i * TN + jj) * kWave + lane;
      f32x4 sum = __builtin_nontemporal_load(partial_slot(g, plan, j, 0) + at);
      for (int sl = 1; sl < plan.n_slices; ++sl) {
        const f32x4 v = __builtin_nontemporal_load(partial_slot(g, plan, j, sl) + at);
#pragma unroll
        for (int x = 0; x < 4; ++x) sum[x] += v[x];
      }
      return sum;
    };
    auto put = [&](void* C, size_t idx, const f32x4& v) {
      *reinterpret_cast<u32x2*>(static_cast<bf16_t*>(C) + idx) = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
    };
    const int m = tile.row0 + wm * (TM * 16) + i * 16 + (lane & 15);
#pragma unroll
    for (int jj = 0; jj < TNH; ++jj) {
      const int n = col0 + wn * (TNH * 16) + jj * 16 + 4 * (lane >> 4);
      const bool inside = m < tile.row_end && n < g.N;
      const size_t idx = (size_t)m * g.ldc + n;
      if constexpr (MODE == UP) {                        // fragment jj holds x W1, fragment jj + TNH x W3 of the same outputs
        const f32x4 h1 = slices_sum(jj), h3 = slices_sum(jj + TNH);
        f32x4 a;
#pragma unroll
        for (int x = 0; x < 4; ++x) a[x] = silu_f(h1[x]) * h3[x];
        if (inside) {
          if (g.C0) { put(g.C0, idx, h1); put(g.C1, idx, h3); }
          put(g.C2, idx, a);
        }
      } else {
        const f32x4 sum = slices_sum(jj);
        if (inside) put(g.C0, idx, sum);
      }
    }
  }

  static __device__ void run(const MArgs& g, char* smem) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int wm = wave / WN, wn = wave % WN;

    const Experts experts(g, lane);
    const SplitPlan plan = split_plan(g, experts.n_rt);
    int id = blockIdx.x, slice = 0;
    if (SPLIT && id >= g.total_ids) {                    // a workgroup for slice 1.. of a left-over tile
      if (plan.n_slices <= 1) return;
      const int w = id - g.total_ids;
      slice = 1 + w / plan.n_left;
      if (slice >= plan.n_slices) return;
      id = plan.id_full + w % plan.n_left;
    }
    const bool sliced = SPLIT && plan.n_slices > 1 && id >= plan.id_full;
    Tile tile;
    if (!locate(g, experts, id, tile)) return;
    const int e = tile.e, row0 = tile.row0, row_end = tile.row_end, k_begin = tile.k_begin, k_end = tile.k_end;
    const int kp_begin = tile.kp_begin, tile_n = tile.tile_n;
    const int col0 = tile_n * BNH;

    const bf16_t* Bp0 = g.B0;
    const bf16_t* Bp1 = g.B1;
    if (!GROUP_K) { Bp0 += e * g.strideB_e; if (Bp1) Bp1 += e * g.strideB_e; }

    // ---- per-lane byte offsets of the direct copies, relative to a per-tile uniform base --
    // KC operand:      base = P + row0*ld + k0,  offset = (clamp(row) - row0)*ld + k_in_tile
    // strided operand: base = P + k0*ld,         offset = k_in_tile*ld + clamp(col)
    uint32_t a_off[A_LOADS], b_off[B_LOADS];
    int b_k[B_LOADS], b_c[B_LOADS];                               // strided layout: k row / column
    bool b_second[B_LOADS];
    bool a_hi[A_LOADS], b_hi[B_LOADS];                            // KC layouts: chunk lies in the upper 32 k of the tile
#pragma unroll
    for (int q = 0; q < A_LOADS; ++q) {
      int major, minor;
      copy_coords<A_KC, BM>(wave * A_LOADS + q, lane, major, minor);
      const int gr = min(row0 + major, row_end - 1);
      // gathered rows: the offset is taken from the first row of A0 (it fits 32 bits, checked on the host)
      a_off[q] = g.a_perm ? (uint32_t)(g.a_perm[gr] / g.a_k) * (uint32_t)(g.lda * 2) + (uint32_t)(minor * 2)
                          : (uint32_t)((gr - row0) * g.lda + minor) * 2u;
      a_hi[q] = minor >= 32;
    }
#pragma unroll
    for (int q = 0; q < B_LOADS; ++q) {
      int major, minor;
      // DUAL: the B tile is two panels [BK][BNH] back to back, so one wave copy (1 KB) never
      // straddles W1 and W3 and its base pointer stays uniform
      constexpr int SEGS_PER_PANEL = B_BYTES / 1024 / (DUAL ? 2 : 1);
      const int seg = wave * B_LOADS + q;
      copy_coords<B_KC, BNH>(seg % SEGS_PER_PANEL, lane, major, minor);
      if (B_KC) {
        // tile rows are output columns (DUAL: BNH of the first panel, then BNH of the second)
        b_off[q] = (uint32_t)((min(col0 + major, g.N - 1) - col0) * g.ldb + minor) * 2u;
        b_k[q] = b_c[q] = 0;
        b_second[q] = DUAL && seg >= SEGS_PER_PANEL;
        b_hi[q] = minor >= 32;
      } else {
        b_hi[q] = false;
        b_k[q] = major;
        b_c[q] = min(col0 + minor, g.N - 8);
        b_off[q] = (uint32_t)(major * g.ldb + b_c[q]) * 2u;
        b_second[q] = DUAL && seg >= SEGS_PER_PANEL;     // uniform across the wavefront
      }
    }

    const int k_len = k_end - k_begin;
    const int nk1 = (k_len + BK - 1) / BK;
    const int nk_all = MODE == BWD_DX ? 2 * nk1 : nk1;
    // a slice runs k tiles kb .. kb + nk - 1 of the tile's nk_all; below, kt counts from the slice's first one
    const int kb = sliced ? slice * nk_all / plan.n_slices : 0;
    const int nk = sliced ? (slice + 1) * nk_all / plan.n_slices - kb : nk_all;
    // K is a multiple of 32 (of 64 in the dW products, whose rows are padded): when it is not
    // a multiple of 64 the last k tile of a pass is half empty.  Its copies are re-pointed at
    // the valid half (any finite data will do) and the A fragments of its second half are
    // zeroed in registers, so those k steps add nothing.
    // TAIL is a template parameter: the common shapes pay nothing for it.
    static_assert(!(TAIL && GROUP_K), "the dW products have no K tail");
    // in the slice's own count of k tiles: where the second K pass begins, and the two possible tail tiles
    const int pass2_at = nk1 - kb, tail1_at = nk1 - 1 - kb, tail2_at = nk_all - 1 - kb;
    const int k_first1 = k_begin + kb * BK, k_first2 = k_begin - pass2_at * BK;
    const int kp_first = kp_begin + kb * BK;
    auto is_tail = [&](int kt) { return TAIL && (kt == tail1_at || kt == tail2_at); };
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;   // LDS byte address of the dynamic segment

    // Copies of the A / B part of tile kt into LDS stage kt % NSA / kt % NSB.
    auto tile_k0 = [&](int kt, bool kc, bool& pass2) {
      pass2 = MODE == BWD_DX && kt >= pass2_at;
      return (GROUP_K && kc ? kp_first : (pass2 ? k_first2 : k_first1)) + kt * BK;
    };
    auto issueA = [&](int kt) {
      bool pass2;
      const int k0 = tile_k0(kt, A_KC, pass2);
      const uint32_t stage = smem_base + (kt % NSA) * A_BYTES;
      const bf16_t* Ab = pass2 ? g.A1 : g.A0;
      Ab += (g.a_perm ? (size_t)0 : (size_t)row0 * g.lda) + k0;
#pragma unroll
      for (int q = 0; q < A_LOADS; ++q) {
        uint32_t off = a_off[q];
        if (a_hi[q] && is_tail(kt)) off -= 64u;
        copy16_to_lds(Ab, off, stage + (wave * A_LOADS + q) * 1024);
      }
    };
    auto issueB = [&](int kt) {
      bool pass2;
      const int k0 = tile_k0(kt, B_KC, pass2);
      const uint32_t stage = smem_base + B_BASE + (kt % NSB) * B_BYTES;
      const bf16_t* B0b = Bp0 + (B_KC ? (size_t)col0 * g.ldb + k0 : (size_t)k0 * g.ldb);
      const bf16_t* B1b = Bp1 ? Bp1 + (B_KC ? (size_t)col0 * g.ldb + k0 : (size_t)k0 * g.ldb) : nullptr;
#pragma unroll
      for (int q = 0; q < B_LOADS; ++q) {
        uint32_t off = b_off[q];
        // grouped-K, strided operand: a k row past the expert's last grouped row is re-pointed at that last
        // row.  It meets the zero fill of the transposed operand, so it must hold finite numbers: the
        // expert's own rows were written by BWD_ACT in this call, whereas the rows behind them belong to
        // the next expert or, past the last kept row when a capacity limit dropped pairs, to nobody
        // (workspace bytes nothing has written, possibly NaN patterns).
        if (GROUP_K && !B_KC) off = (uint32_t)((min(k0 + b_k[q], k_end - 1) - k0) * g.ldb + b_c[q]) * 2u;
        if (is_tail(kt)) {
          if (B_KC) { if (b_hi[q]) off -= 64u; }
          else off = (uint32_t)(min(b_k[q], 31) * g.ldb + b_c[q]) * 2u;
        }
        const bool second = MODE == BWD_DX ? pass2 : (DUAL && b_second[q]);
        copy16_to_lds(second ? B1b : B0b, off, stage + (wave * B_LOADS + q) * 1024);
      }
    };

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

    auto load_frags = [&](int kt, int ks, bf16x8 (&af)[TM], bf16x8 (&bfr)[TN]) {
      const char* At = smem + (kt % NSA) * A_BYTES;
      const char* Bt = smem + B_BASE + (kt % NSB) * B_BYTES;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int r = wm * (TM * 16) + i * 16;
        af[i] = read_kc(At, r, ks, lane);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int c = wn * (TNH * 16) + (j % TNH) * 16;
        bfr[j] = B_KC ? read_kc(Bt, (j / TNH) * BNH + c, ks, lane)
                      : read_tr<BNH>(Bt + (j / TNH) * (BK * BNH * 2), c, ks, lane);
      }
    };
    auto mfma_step = [&](bf16x8 (&af)[TM], bf16x8 (&bfr)[TN]) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    };
    // grouped-K: the k rows past an expert's last one meet the zero fill of the transposed operand

    {
      // Ping-pong schedule.  The two wavefronts that share a SIMD (w and w+4) alternate
      // between a memory phase (LDS fragment reads of half a tile + a quarter of the copies
      // of a later tile) and a compute phase (an uninterrupted run of 32 MFMAs), half a period
      // apart and kept in step by a barrier at every phase boundary.  The matrix pipe always
      // has one wavefront feeding it and is never held up behind a wavefront that is stuck
      // issuing copies or waiting for LDS.  Time is counted in phases; tile kt occupies phases
      // 4kt .. 4kt+3 for group 0 and one phase later for group 1:
      //   phase 4kt   : G0 reads half 0 of tile kt, issues its B copies of tile kt+1   | G1 computes
      //   phase 4kt+1 : G0 computes | G1 reads half 0 of tile kt, issues its B copies of tile kt+1
      //   phase 4kt+2 : G0 reads half 1, issues its A copies of tile kt+2             | G1 computes
      //   phase 4kt+3 : G0 computes | G1 reads half 1, issues its A copies of tile kt+2
      // so the address unit sees the same 16 copies in every phase.  B has two LDS stages (its
      // copies have at least 2.5 phases to land), A has three (at least 4 phases).  Every
      // wavefront waits for its copies of tile kt+1 right before the barrier that ends phase
      // 4kt+3; its 4 youngest copies (A of tile kt+2) may stay in flight.
      constexpr int HS = KSTEPS / 2;                 // k steps per half tile
      const int grp = wave / (NW / 2);               // group 1 lags group 0 by one phase
      bf16x8 fa[HS][TM], fb[HS][TN];
      if (nk > 0) {
        issueA(0);
        issueB(0);
        if (nk > 1) issueA(1);
        if (nk > 1) wait_vmcnt(A_LOADS); else wait_vmcnt(0);
        __builtin_amdgcn_s_barrier();                // tile 0 published
      }
      if (grp == 1 && nk > 0) __builtin_amdgcn_s_barrier();   // idle during group 0's first memory phase
      // one k tile per trip: unrolled by two (the compiler's choice for some instantiations) the loop ran 2 to
      // 4 % slower
#pragma unroll 1
      for (int kt = 0; kt < nk; ++kt) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          // ---- memory phase
#pragma unroll
          for (int x = 0; x < HS; ++x) load_frags(kt, h * HS + x, fa[x], fb[x]);
          if (h == 0 && kt + 1 < nk) issueB(kt + 1);
          if (h == 1 && kt + 2 < nk) issueA(kt + 2);
          __builtin_amdgcn_s_waitcnt(0xC07F);        // lgkmcnt(0): fragments are in registers
          if (h == 1 && is_tail(kt)) {               // the half of the last k tile that lies past K
#pragma unroll
            for (int x = 0; x < HS; ++x)
#pragma unroll
              for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int v = 0; v < 8; ++v) fa[x][i][v] = (__bf16)0.0f;
          }
          if (h == 1 && grp == 1) { if (kt + 2 < nk) wait_vmcnt(A_LOADS); else wait_vmcnt(0); }
          __builtin_amdgcn_sched_barrier(0);
          __builtin_amdgcn_s_barrier();
          __builtin_amdgcn_sched_barrier(0);
          // ---- compute phase
#pragma unroll
          for (int x = 0; x < HS; ++x) mfma_step(fa[x], fb[x]);
          if (h == 1 && grp == 0) { if (kt + 2 < nk) wait_vmcnt(A_LOADS); else wait_vmcnt(0); }
          __builtin_amdgcn_sched_barrier(0);
          if (!(grp == 1 && h == 1 && kt + 1 == nk)) __builtin_amdgcn_s_barrier();
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }

    if (SPLIT && sliced) {                               // a slice leaves its accumulators for split_finish
      f32x4* slot = partial_slot(g, plan, id - plan.id_full, slice) + (size_t)wave * (TM * TN * kWave);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) __builtin_nontemporal_store(acc[i][j], slot + (i * TN + j) * kWave + lane);
      return;
    }

    // ---- epilogue ----------------------------------------------------------
    // acc[i][j][v]: row m = row0 + wm*TM*16 + i*16 + lane%16,
    //               col n = col0 + wn*TNH*16 + (j%TNH)*16 + 4*(lane/16) + v
    // In that layout one store instruction would touch 16 rows with 8 to 16 bytes each.  Instead
    // every wavefront turns its results around in a private piece of LDS, one band of 32 rows
    // (two fragment rows) at a time: the lanes write their 4-column pieces, read the band back
    // as 16-byte chunks that follow each other along a row, and store whole row segments (64 to
    // 256 contiguous bytes per row).  BWD_ACT fetches the saved h1/h3 band the same way round.
    // The operand stages are dead by now: in the ping-pong schedule the barrier that ends group
    // 0's last compute phase comes after group 1's last fragment read and after every copy has
    // landed.
    const int lane_m = lane & 15, lane_c = lane >> 4;
    const int wcol0 = col0 + wn * (TNH * 16);         // first output column of this wavefront (per panel)
    constexpr int NB = TM / 2;                         // 32-row bands per wavefront
    // byte offset, inside a band, of this lane's 4-column piece of fragment (i2, j); ES = element size
    auto piece = [&](auto rowb_tag, auto es_tag, int i2, int j) {
      constexpr int ROWB = decltype(rowb_tag)::value, ES = decltype(es_tag)::value;
      const int byte = (j * 16 + 4 * lane_c) * ES;
      const uint32_t flip = MODE == BWD_ACT ? 0u : half_flip<ROWB, ES>(i2 * 16 + lane_m);
      return stage_off<ROWB, 4 * ES>(i2 * 16 + lane_m, byte >> 4) + ((byte & 15) ^ flip);
    };
    float dg_acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) dg_acc[i] = 0.f;

    if constexpr (MODE == BWD_ACT) {
      constexpr int ROWB = TNH * 32;                  // bytes per band row
      constexpr int CPR = ROWB / 16, RPI = 64 / CPR, NI = 32 / RPI;
      static_assert(5 * 32 * ROWB * NW <= LDS_BYTES, "epilogue bands must fit the operand stages");
      char* bufA = smem + wave * (5 * 32 * ROWB);
      char* bufB = bufA + 32 * ROWB;
      char* bufC = bufB + 32 * ROWB;
      char* bufT = bufC + 32 * ROWB;                  // two bands of g * act, transposed: [column][64 rows]
      const int cr = lane / CPR, cc = lane % CPR;     // row (per pass) and chunk of the row-contiguous view
      const int cn = wcol0 + cc * 8;
      u32x4 p1[NI], p3[NI];
      float gate_next[2];
      // band ib of h1/h3 in the row-contiguous view (clamped, always valid addresses)
      auto fetch = [&](int ib) {
        const int mb = row0 + wm * (TM * 16) + ib * 32;
#pragma unroll
        for (int t = 0; t < NI; ++t) {
          const size_t idx = (size_t)min(mb + t * RPI + cr, row_end - 1) * g.ldc + min(cn, g.N - 8);
          // read once by this tile and by nobody else: streamed past the L2 (another 2 % of the kernel)
          p1[t] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(g.H1 + idx));
          p3[t] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(g.H3 + idx));
        }
#pragma unroll
        for (int i2 = 0; i2 < 2; ++i2) gate_next[i2] = g.gates[g.perm[min(mb + i2 * 16 + lane_m, row_end - 1)]];
      };
      fetch(0);
#pragma unroll
      for (int ib = 0; ib < NB; ++ib) {
        const int mb = row0 + wm * (TM * 16) + ib * 32;
#pragma unroll
        for (int t = 0; t < NI; ++t) {
          const uint32_t o = stage_off<ROWB, 8>(t * RPI + cr, cc);
          *reinterpret_cast<u32x4*>(bufA + o) = p1[t];
          *reinterpret_cast<u32x4*>(bufB + o) = p3[t];
        }
        const float gate2[2] = {gate_next[0], gate_next[1]};
        if (ib + 1 < NB) fetch(ib + 1);               // in flight during the arithmetic below
#pragma unroll
        for (int i2 = 0; i2 < 2; ++i2) {
          const int i = 2 * ib + i2;
          const bool m_ok = mb + i2 * 16 + lane_m < row_end;
          const float gate = m_ok ? gate2[i2] : 0.f;    // rows past the group's end come out as zeros
#pragma unroll
          for (int j = 0; j < TNH; ++j) {
            const uint32_t o = piece(std::integral_constant<int, ROWB>{}, std::integral_constant<int, 2>{}, i2, j);
            const u32x2 a1 = *reinterpret_cast<const u32x2*>(bufA + o);
            const u32x2 a3 = *reinterpret_cast<const u32x2*>(bufB + o);
            const float z[4] = {bf16lo(a1[0]), bf16hi(a1[0]), bf16lo(a1[1]), bf16hi(a1[1])};
            const float v3[4] = {bf16lo(a3[0]), bf16hi(a3[0]), bf16lo(a3[1]), bf16hi(a3[1])};
            float o1[4], o3[4], oa[4], dot = 0.f;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
              const float dd = acc[i][j][x];
              const float sg = sigmoid_f(z[x]), sl = z[x] * sg;
              const float a = sl * v3[x];
              dot = fmaf(dd, a, dot);
              const float da = gate * dd;
              o1[x] = da * v3[x] * fmaf(sl, 1.f - sg, sg);     // silu'(z) = sg + silu(z) (1 - sg)
              o3[x] = da * sl;
              oa[x] = gate * a;
            }
            if (m_ok && wcol0 + j * 16 + 4 * lane_c < g.N) dg_acc[i] += dot;
            // each lane overwrites exactly the pieces it has just read
            *reinterpret_cast<u32x2*>(bufA + o) = u32x2{pack_bf16x2(o1[0], o1[1]), pack_bf16x2(o1[2], o1[3])};
            *reinterpret_cast<u32x2*>(bufB + o) = u32x2{pack_bf16x2(o3[0], o3[1]), pack_bf16x2(o3[2], o3[3])};
            if (g.T2) *reinterpret_cast<u32x2*>(bufC + o) = u32x2{pack_bf16x2(oa[0], oa[1]), pack_bf16x2(oa[2], oa[3])};
          }
        }
#pragma unroll
        for (int t = 0; t < NI; ++t) {
          const int r = t * RPI + cr;
          const uint32_t o = stage_off<ROWB, 8>(r, cc);
          const u32x4 v1 = *reinterpret_cast<const u32x4*>(bufA + o);
          const u32x4 v3 = *reinterpret_cast<const u32x4*>(bufB + o);
          if (mb + r < row_end && cn < g.N) {
            const size_t idx = (size_t)(mb + r) * g.ldc + cn;
            store_out<STREAM_OUT>(reinterpret_cast<u32x4*>(static_cast<bf16_t*>(g.C0) + idx), v1);
            store_out<STREAM_OUT>(reinterpret_cast<u32x4*>(static_cast<bf16_t*>(g.C1) + idx), v3);
          }
        }
        if (g.T2) {
          // The same band once more, transposed, for the dW products: [column][padded grouped row].
          // A pair of transposing reads turns 16 columns x 8 rows per 16-lane group around: lane
          // 4a+b of a group receives element b of what lanes a, a+4, a+8, a+12 fetched, so lane r
          // fetches band row 8*group + r/4 (then +4) at columns 4*(r%4).. and ends up with rows
          // 8*group .. +7 of column r: 16 contiguous bytes of the transposed matrix.  Those are
          // collected over two bands as [column][64 rows] (128 bytes per column, chunks swizzled by
          // column) and read back so that eight consecutive lanes hold one column's 128 bytes: whole,
          // aligned cache lines per store (with 64-byte pieces, one band at a time, these stores moved
          // 3.1 TB/s where the row stores of dh1/dh3 move 5.1; scattered 16-byte stores cost the address
          // unit four times as much again).  Rows past the group's end are zeros (see the gate above) and
          // are written up to the 64-row padding.
          typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
          static_assert(NB % 2 == 0, "bands are turned around in pairs");
          const int o_e = tile.exp_row0;
          const int pad_e = (row_end - o_e + 63) & ~63;
          const int fr = 8 * lane_c + (lane_m >> 2), fa4 = lane_m & 3;
          bf16x8 v[TNH];
#pragma unroll
          for (int pr = 0; pr < TNH; ++pr) {
            const uint32_t o_lo = stage_off<ROWB, 8>(fr, 2 * pr + (fa4 >> 1)) + 8 * (fa4 & 1);
            const uint32_t o_hi = stage_off<ROWB, 8>(fr + 4, 2 * pr + (fa4 >> 1)) + 8 * (fa4 & 1);
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(bufC + o_lo));
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(bufC + o_hi));
            v[pr] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          }
#pragma unroll
          for (int pr = 0; pr < TNH; ++pr) {
            const int tc = 16 * pr + lane_m;             // column; chunk = 8 rows: 4 per band
            *reinterpret_cast<bf16x8*>(bufT + tc * 128 + ((((ib & 1) * 4 + lane_c) ^ ((tc >> 1) & 7)) << 4)) = v[pr];
          }
          if (ib & 1) {
            const int qc = lane >> 3, qg = lane & 7;     // read-back view: column within 8, 8-row chunk of the pair
            const int m8 = mb - 32 + 8 * qg - o_e;       // grouped row of that chunk, relative to the expert
#pragma unroll
            for (int pr = 0; pr < 2 * TNH; ++pr) {
              const int tc = 8 * pr + qc;
              const bf16x8 w = *reinterpret_cast<const bf16x8*>(bufT + tc * 128 + ((qg ^ ((tc >> 1) & 7)) << 4));
              const int col = wcol0 + tc;
              if (col < g.N && m8 < pad_e)
                store_out<STREAM_OUT>(reinterpret_cast<bf16x8*>(g.T2 + (size_t)col * g.ldt + kp_begin + m8), w);
            }
          }
        }
      }
    } else {
      constexpr int NP = MODE == UP ? 3 : (DUAL ? 2 : 1);            // matrices written
      // ET: element type of the output (bf16 bits or float)
      auto staged = [&](auto tag) {
        using ET = decltype(tag);
        constexpr int ES = sizeof(ET);
        constexpr int ROWB = TNH * 16 * ES;
        constexpr int CPR = ROWB / 16, RPI = 64 / CPR, NI = 32 / RPI;
        static_assert(ROWB == 64 || ROWB == 128 || ROWB == 256 || ROWB == 512, "band row");
        static_assert(NP * 32 * ROWB * NW <= LDS_BYTES, "epilogue bands must fit the operand stages");
        char* wb = smem + wave * (NP * 32 * ROWB);
        const int cr = lane / CPR, cc = lane % CPR;
        const int cn = wcol0 + cc * (16 / ES);
        const bool want_h = MODE != UP || g.C0 != nullptr;
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) {
          const int mb = row0 + wm * (TM * 16) + ib * 32;
#pragma unroll
          for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
            for (int j = 0; j < TNH; ++j) {
              const int i = 2 * ib + i2;
              const uint32_t o = piece(std::integral_constant<int, ROWB>{}, std::integral_constant<int, ES>{}, i2, j);
              float v[NP][4];
#pragma unroll
              for (int x = 0; x < 4; ++x) {
                if constexpr (MODE == UP) {
                  v[0][x] = acc[i][j][x];
                  v[1][x] = acc[i][j + TNH][x];
                  v[2][x] = silu_f(v[0][x]) * v[1][x];
                } else {
#pragma unroll
                  for (int pp = 0; pp < NP; ++pp) v[pp][x] = acc[i][j + pp * TNH][x];
                }
              }
#pragma unroll
              for (int pp = 0; pp < NP; ++pp) {
                if (MODE == UP && pp < 2 && !want_h) continue;
                char* dst = wb + pp * (32 * ROWB) + o;
                if constexpr (ES == 2)
                  *reinterpret_cast<u32x2*>(dst) = u32x2{pack_bf16x2(v[pp][0], v[pp][1]), pack_bf16x2(v[pp][2], v[pp][3])};
                else
                  *reinterpret_cast<f32x4*>(dst) = f32x4{v[pp][0], v[pp][1], v[pp][2], v[pp][3]};
              }
            }
#pragma unroll
          for (int pp = 0; pp < NP; ++pp) {
            if (MODE == UP && pp < 2 && !want_h) continue;
            ET* C = static_cast<ET*>(pp == 0 ? g.C0 : (pp == 1 ? g.C1 : g.C2)) + (GROUP_K ? (size_t)e * g.strideC_e : 0);
#pragma unroll
            for (int t = 0; t < NI; ++t) {
              const int r = t * RPI + cr;
              const u32x4 val = swap_halves(
                  *reinterpret_cast<const u32x4*>(wb + pp * (32 * ROWB) + stage_off<ROWB, 4 * ES>(r, cc)),
                  half_flip<ROWB, ES>(r) != 0);
              if (mb + r < row_end && cn < g.N) store_out<STREAM_OUT>(reinterpret_cast<u32x4*>(C + (size_t)(mb + r) * g.ldc + cn), val);
            }
          }
        }
      };
      if constexpr (GROUP_K) {                       // only the weight gradients can be asked for in fp32
        if (g.c_is_f32) staged(float{});
        else staged(bf16_t{});
      } else {
        staged(bf16_t{});
      }
    }
    if (MODE == BWD_ACT) {
      // dg partial of this column tile: lanes l, l^16, l^32, l^48 hold the same row; then the WN
      // wavefronts of a row band are summed in fixed order through LDS.
      __syncthreads();  // all waves are done with the operand tiles
      float* red = reinterpret_cast<float*>(smem);   // [WN][BM]
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        float s = dg_acc[i] + __shfl_xor(dg_acc[i], 16, kWave);
        s += __shfl_xor(s, 32, kWave);
        if (lane_c == 0) red[wn * BM + wm * (TM * 16) + i * 16 + lane_m] = s;
      }
      __syncthreads();
      for (int r = threadIdx.x; r < BM; r += NT) {
        const int m = row0 + r;
        if (m < row_end) {
          float s = 0.f;
#pragma unroll
          for (int w = 0; w < WN; ++w) s += red[w * BM + r];
          g.dg_part[(size_t)m * g.n_part + tile_n] = s;
        }
      }
    }
  }
};

template <int BM, int BN, int BK, int WM, int WN, int NSA, int NSB, int MODE, bool TAIL = false>
__global__ __launch_bounds__(WM* WN* kWave) void mfma_gemm_kernel(MArgs g) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  Gemm<BM, BN, BK, WM, WN, NSA, NSB, MODE, TAIL>::run(g, smem);
}

template <int BM, int BN, int BK, int WM, int WN, int NSA, int NSB, int MODE, bool TAIL = false>
__global__ __launch_bounds__(WM* WN* kWave) void mfma_split_finish_kernel(MArgs g) {
  Gemm<BM, BN, BK, WM, WN, NSA, NSB, MODE, TAIL>::finish(g);
}

// compute units of the current device (looked up once per device)
int compute_units() {
  static int n[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -1;
  if (n[dev] == 0) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 8) return -1;
    n[dev] = v;
  }
  return n[dev];
}

// The kernels use more dynamic LDS than the default limit allows: the limit is raised once per
// device and instantiation (idempotent, so a race between threads is harmless).  This must not
// happen inside a stream capture; mfma_prepare() does it for every instantiation up front.
template <int BM, int BN, int BK, int WM, int WN, int NSA, int NSB, int MODE, bool TAIL = false>
int raise_lds_limit() {
  using G = Gemm<BM, BN, BK, WM, WN, NSA, NSB, MODE, TAIL>;
  static bool attr_set[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return BTX_ERR_HIP;
  if (!attr_set[dev]) {
    auto kern = mfma_gemm_kernel<BM, BN, BK, WM, WN, NSA, NSB, MODE, TAIL>;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            G::LDS_BYTES) != hipSuccess)
      return BTX_ERR_HIP;
    attr_set[dev] = true;
  }
  return BTX_OK;
}

template <int BM, int BN, int BK, int WM, int WN, int NSA, int NSB, int MODE, bool TAIL = false>
int launch(MArgs g, hipStream_t s) {
  using G = Gemm<BM, BN, BK, WM, WN, NSA, NSB, MODE, TAIL>;
  constexpr int BNH = G::DUAL ? BN / 2 : BN;
  g.tiles_n = ceil_div(g.N, BNH);
  g.tiles_m = G::GROUP_K ? ceil_div(g.M, BM) : ceil_div(g.R, BM) + g.E;
  // every tile has exactly one block id below (number of tiles) + 8; see the tile mapping
  g.blocks_per_e = (int)align_up((size_t)g.tiles_m * g.tiles_n, 8) + 8;
  g.total_ids = G::GROUP_K ? g.E * g.blocks_per_e : g.tiles_m * g.tiles_n + 8;
  if (int rc = raise_lds_limit<BM, BN, BK, WM, WN, NSA, NSB, MODE, TAIL>()) return rc;
  int grid = g.total_ids;
  if constexpr (G::SPLIT) {
    // K too short for two slices of the minimum length: split_plan() would never cut
    if (ceil_div(g.K, BK) * (MODE == BWD_DX ? 2 : 1) < 2 * G::kMinSliceTiles) g.partial = nullptr;
    if (g.partial) {                                   // room for the workgroups of slices 1.. of the last round
      g.cus = compute_units();
      if (g.cus <= 0) return BTX_ERR_HIP;
      if (g.cus > kSplitMaxCus) g.partial = nullptr;   // the caller's buffer is sized for that many
      else grid += g.cus + G::kIdHoles * (G::kMaxSlices - 1);   // (left + 8)(S - 1) <= cus + 8 (S - 1) for every left
    }
  } else {
    g.partial = nullptr;
  }
  mfma_gemm_kernel<BM, BN, BK, WM, WN, NSA, NSB, MODE, TAIL><<<grid, G::NT, G::LDS_BYTES, s>>>(g);
  BTX_LAUNCH_CHECK();
  if constexpr (G::SPLIT) {
    if (g.partial) {
      mfma_split_finish_kernel<BM, BN, BK, WM, WN, NSA, NSB, MODE, TAIL>
          <<<(g.cus / 2 + G::kIdHoles) * G::TM, G::NT, 0, s>>>(g);
      BTX_LAUNCH_CHECK();
    }
  }
  return BTX_OK;
}

// The direct-copy loaders need whole 16-byte chunks inside every row and K multiples of 32
// where K is a matrix dimension (half a k tile).
bool fast_ok(const FfShapes& sh) { return sh.d % 32 == 0 && sh.f % 32 == 0 && sh.d >= 64 && sh.f >= 64; }

}  // namespace

constexpr int kActBN = 256;  // column tile of the BWD_ACT kernel = width of one dg partial

// fp32 accumulators of the K slices of the last round of UP / DOWN / BWD_DX: at most cus + 8 * 8 (tile, slice) pairs
// of 256 x 256 floats
size_t mfma_split_bytes() { return (size_t)(kSplitMaxCus + 8 * kSplitMaxSlices) * 256 * 256 * sizeof(float); }

int mfma_prepare() {
  if (compute_units() <= 0) return BTX_ERR_HIP;        // looked up once per device, here rather than in a launch
  int rc = BTX_OK;
  auto both = [&](auto mode_tag, auto bn_tag) {
    constexpr int MODE = decltype(mode_tag)::value, BN = decltype(bn_tag)::value;
    if (!rc) rc = raise_lds_limit<256, BN, 64, 2, 4, 3, 2, MODE, false>();
    if constexpr (MODE != DW13 && MODE != DW2)
      if (!rc) rc = raise_lds_limit<256, BN, 64, 2, 4, 3, 2, MODE, true>();
  };
  both(std::integral_constant<int, UP>{}, std::integral_constant<int, 256>{});
  both(std::integral_constant<int, DOWN>{}, std::integral_constant<int, 256>{});
  both(std::integral_constant<int, BWD_ACT>{}, std::integral_constant<int, kActBN>{});
  both(std::integral_constant<int, BWD_DX>{}, std::integral_constant<int, 256>{});
  both(std::integral_constant<int, DW13>{}, std::integral_constant<int, 256>{});
  both(std::integral_constant<int, DW2>{}, std::integral_constant<int, 256>{});
  return rc;
}
int mfma_bwd_act_partials(int f) { return ceil_div(f, kActBN); }

bool mfma_gather_ok(int T, int d) { return (int64_t)T * d * 2 < ((int64_t)1 << 32); }

int mfma_up_swiglu(const RowSource& xs, const void* W1, const void* W3, const int32_t* off, const FfShapes& sh,
                   void* h1, void* h3, void* act, void* partial, hipStream_t s) {
  if (!fast_ok(sh)) return BTX_ERR_UNSUPPORTED;
  MArgs g{};
  g.A0 = (const bf16_t*)xs.base; g.a_perm = xs.perm; g.a_k = xs.k; g.B0 = (const bf16_t*)W1; g.B1 = (const bf16_t*)W3; g.C0 = h1; g.C1 = h3; g.C2 = act; g.partial = (f32x4*)partial;
  g.offsets = off; g.E = sh.E; g.N = sh.f; g.K = sh.d; g.lda = sh.d; g.ldb = sh.f; g.ldc = sh.f;
  g.strideB_e = sh.s13; g.R = sh.R;
  return sh.d % 64 ? launch<256, 256, 64, 2, 4, 3, 2, UP, true>(g, s) : launch<256, 256, 64, 2, 4, 3, 2, UP>(g, s);
}

int mfma_down(const void* act, const void* W2, const int32_t* off, const FfShapes& sh, void* y, void* partial,
              hipStream_t s) {
  if (!fast_ok(sh)) return BTX_ERR_UNSUPPORTED;
  MArgs g{};
  g.A0 = (const bf16_t*)act; g.B0 = (const bf16_t*)W2; g.C0 = y; g.partial = (f32x4*)partial;
  g.offsets = off; g.E = sh.E; g.N = sh.d; g.K = sh.f; g.lda = sh.f; g.ldb = sh.d; g.ldc = sh.d;
  g.strideB_e = sh.s2; g.R = sh.R;
  return sh.f % 64 ? launch<256, 256, 64, 2, 4, 3, 2, DOWN, true>(g, s) : launch<256, 256, 64, 2, 4, 3, 2, DOWN>(g, s);
}

int mfma_bwd_act(const RowSource& dys, const void* W2, const void* h1, const void* h3, const float* gates,
                 const int32_t* perm, const int32_t* off, const FfShapes& sh, void* dh1, void* dh3, void* gaT,
                 float* dg_part, hipStream_t s) {
  if (!fast_ok(sh)) return BTX_ERR_UNSUPPORTED;
  MArgs g{};
  g.A0 = (const bf16_t*)dys.base; g.a_perm = dys.perm; g.a_k = dys.k;
  g.B0 = (const bf16_t*)W2; g.C0 = dh1; g.C1 = dh3;
  g.T2 = (bf16_t*)gaT; g.ldt = mfma_dw_pitch(sh.R, sh.E);
  g.H1 = (const bf16_t*)h1; g.H3 = (const bf16_t*)h3; g.gates = gates; g.perm = perm; g.dg_part = dg_part;
  g.n_part = mfma_bwd_act_partials(sh.f);
  g.offsets = off; g.E = sh.E; g.N = sh.f; g.K = sh.d; g.lda = sh.d; g.ldb = sh.d; g.ldc = sh.f;
  g.strideB_e = sh.s2; g.R = sh.R;
  return sh.d % 64 ? launch<256, kActBN, 64, 2, 4, 3, 2, BWD_ACT, true>(g, s)
                   : launch<256, kActBN, 64, 2, 4, 3, 2, BWD_ACT>(g, s);
}

int mfma_bwd_dx(const void* dh1, const void* dh3, const void* W1, const void* W3, const int32_t* off,
                const FfShapes& sh, void* dxs, void* partial, hipStream_t s) {
  if (!fast_ok(sh)) return BTX_ERR_UNSUPPORTED;
  MArgs g{};
  g.A0 = (const bf16_t*)dh1; g.A1 = (const bf16_t*)dh3; g.B0 = (const bf16_t*)W1; g.B1 = (const bf16_t*)W3; g.C0 = dxs; g.partial = (f32x4*)partial;
  g.offsets = off; g.E = sh.E; g.N = sh.d; g.K = sh.f; g.lda = sh.f; g.ldb = sh.f; g.ldc = sh.d;
  g.strideB_e = sh.s13; g.R = sh.R;
  return sh.f % 64 ? launch<256, 256, 64, 2, 4, 3, 2, BWD_DX, true>(g, s)
                   : launch<256, 256, 64, 2, 4, 3, 2, BWD_DX>(g, s);
}

int mfma_dw_pitch(int R, int E) { return (int)align_up((size_t)R, 64) + 64 * E; }
bool mfma_rows_ok(int R, int E) { return ((int64_t)align_up((size_t)R, 64) + 64 * E) * 256 * 2 < ((int64_t)1 << 32); }

int mfma_bwd_dw13(int dW_dtype, const void* xsT, const void* dh1, const void* dh3, const int32_t* off,
                  const FfShapes& sh, void* dW1, void* dW3, hipStream_t s) {
  if (!fast_ok(sh)) return BTX_ERR_UNSUPPORTED;
  MArgs g{};
  g.A0 = (const bf16_t*)xsT; g.B0 = (const bf16_t*)dh1; g.B1 = (const bf16_t*)dh3; g.C0 = dW1; g.C1 = dW3;
  g.offsets = off; g.E = sh.E; g.M = sh.d; g.N = sh.f; g.lda = mfma_dw_pitch(sh.R, sh.E); g.ldb = sh.f; g.ldc = sh.f;
  g.strideC_e = sh.s13; g.R = sh.R; g.c_is_f32 = dW_dtype == BTX_F32;
  return launch<256, 256, 64, 2, 4, 3, 2, DW13>(g, s);
}

int mfma_bwd_dw2(int dW_dtype, const void* gaT, const void* dysT, const int32_t* off, const FfShapes& sh, void* dW2,
                 hipStream_t s) {
  if (!fast_ok(sh)) return BTX_ERR_UNSUPPORTED;
  MArgs h{};
  h.A0 = (const bf16_t*)gaT; h.B0 = (const bf16_t*)dysT; h.C0 = dW2;
  h.offsets = off; h.E = sh.E; h.M = sh.f; h.N = sh.d; h.lda = h.ldb = mfma_dw_pitch(sh.R, sh.E); h.ldc = sh.d;
  h.strideC_e = sh.s2; h.R = sh.R; h.c_is_f32 = dW_dtype == BTX_F32;
  return launch<256, 256, 64, 2, 4, 3, 2, DW2>(h, s);
}

}  // namespace btx
