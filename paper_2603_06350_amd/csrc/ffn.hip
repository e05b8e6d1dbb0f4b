// moe_grouped_ffn: the expert computation that dominates the MoE layer (Section 3.2).
// For every expert e and row r of its segment [offsets[e], offsets[e+1]):
//   h[r] = silu(W1_e x_perm[r]) * (W3_e x_perm[r]),   y_perm[r] = W2_e h[r].
// The activation rows come either from a permuted copy x_perm, or straight from x through the
// dispatch's src_assign map (moe_grouped_ffn_gather: row r is x[src_assign[r] / k]); the map only
// changes the per-lane row offset of the activation loads.
//
// Two GEMMs: a gated one (W1 and W3 tiles side by side, SwiGLU applied to the fp32
// accumulators, h stored once) and a plain one for W2.  Both are ragged grouped
// GEMMs: the tile list is derived on the device from `offsets`, so the host never
// learns the expert loads.  With 128 or more rows per expert on average each GEMM is two
// launches over disjoint tile lists:
//   main   block tile 256 x 256 weight rows: every full tile of an expert's segment,
//          and its remainder if that has more than 64 rows;
//   small  block tile 64 x 256: remainders of at most 64 rows.
// A small tile has little arithmetic per weight byte, so it is paced by memory
// latency: it runs a four-stage LDS ring with three stages of loads in flight.  The
// small launches run on a side stream next to the main ones (they stream weights from
// HBM while the main tiles are MFMA/L2 bound).  Below 128 rows per expert (decode and
// small prefill batches: the call is bound by streaming the weights once) every segment
// is cut into 64-row ring tiles, one launch per GEMM.
//
// The main tile keeps its operands in a ring of five 32 KiB half-stage slots (all of the CU's LDS):
// two are being multiplied, up to three are in flight.
//
// moe_grouped_ffn_ws brings a workspace of fp32 partial tiles: a tile takes a whole compute unit,
// so a GEMM runs in rounds of the chip, and when the last round of a GEMM with a long reduction
// is at most half full its tiles are computed as 2 to 4 parts of the K range on the idle units
// and added up, in part order, by a second small launch (ffn_sum_parts_kernel).
//
// bf16 kernels (gfx950): 512 threads = 8 waves, two per SIMD.  K step 64: both
// operands are K-contiguous, so a tile row is 128 B = eight 16-byte chunks.  Tiles go
// global -> LDS with 16-byte-per-lane buffer loads that write LDS directly (no register
// staging); a wave instruction fills 8 rows, and the chunk a lane fetches is
// XOR-swizzled by row so that the 16-byte LDS reads of a 16-row MFMA operand are
// bank-conflict free.  The weight fragment is the MFMA "A" operand and the activation
// fragment "B": a lane then owns 4 consecutive output columns of one output row.
// v_mfma_f32_16x16x32_bf16, fp32 accumulators (on this chip it sustains a higher rate
// than the 32x32x16 form).
//
// Work-group ids are remapped so that each XCD (ids are dealt round-robin to the 8
// XCDs) walks a contiguous range of the tile list with the m-tiles of one weight
// panel adjacent: CUs that share an L2 share weight tiles.
//
// Generic kernel (fp32, or bf16 shapes whose d or F is not a multiple of 64): a plain
// LDS-tiled FMA GEMM with fp32 accumulation.
#include <cstdlib>
#include <mutex>
#include <type_traits>

#include "moe_internal.h"

namespace moe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

enum TileMode { TILES_ALL = 0, TILES_MAIN = 1, TILES_SMALL = 2, TILES_EVEN = 3 };
constexpr int BK_ELEMS = 64;    // K elements per stage of the MFMA kernels
constexpr int SMALL_ROWS = 64;  // remainders up to this many rows go to the small-tile kernel

struct GemmArgs {
  const void* a;    // activations [rows, K]
  const void* b0;   // gated: W1 [E,N,K]   plain: W2 [E,N,K]
  const void* b1;   // gated: W3 [E,N,K]   plain: unused
  void* out;        // [rows, N]
  const int32_t* offsets;
  int E, K, N;
  int n_tiles;      // tiles along N
  int rows;         // T*k; row ranges read from `offsets` are clamped to it
  int mode;         // TileMode
  int bm_main;      // rows of a main tile (also the unit remainders are taken against)
  // Gathered activations: row r of the GEMM is row src_assign[r] / k_div of `a` (the token that
  // assignment r belongs to) instead of row r itself.  nullptr = `a` is already permuted.
  const int32_t* src_assign;
  int k_div;
  int a_rows;       // rows of `a` (gathered row numbers are clamped to it)
  int n_cu;         // compute units of the device (the main/small split is priced in rounds of it)
  // n-tiles and K stages of the up- and the down-projection of the call this GEMM belongs to:
  // both take the main/small decision on the same sum, so they take the same one
  int pair_n_tiles[2], pair_kt[2];
  // Split tiles (kernels built with SPLIT only): fp32 partial tiles, one slot per compute unit.
  // nullptr: no tile is split.  split_phase 0: the GEMM itself; 1: the launch after it that adds
  // up the parts of every split tile and stores it.
  float* split_ws;
  int split_phase;
};

constexpr int SPLIT_SLOT_FLOATS = 320 * 256;   // one partial tile (the largest: 320 x 256 fp32)
constexpr int SPLIT_MAX_PARTS = 4;
constexpr int SPLIT_MIN_STAGES = 8;            // K stages a part must keep

// Row of `a` that holds GEMM row r.
__device__ __forceinline__ int a_row_of(const GemmArgs& p, int r) {
  if (!p.src_assign) return r;
  const int t = p.src_assign[r] / p.k_div;
  return min(max(t, 0), p.a_rows - 1);
}

struct TileCoord {
  int e, m_begin, m_end, n_tile;
  // K split of a tile of the last, partial round (nparts == 1: the whole K range)
  int part, nparts;
  int pslot;   // partial-tile slot of this part; the parts of a tile have consecutive slots
};

// Maps a work-group to (expert, row range, n-tile).  Every wave computes this on its
// own from the device-resident offsets; returns false if the group has no tile.
// An expert with c rows has c / bm_main full tiles and a remainder rem = c % bm_main;
// TILES_ALL lists the full tiles and the remainder, TILES_MAIN drops remainders of at
// most SMALL_ROWS rows, TILES_SMALL lists only those.  Tile order: expert-major, then
// n-tile, then m-tile (m fastest), cut into 8 contiguous ranges, one per XCD.
//
// TILES_MAIN and TILES_SMALL belong to two launches over the same offsets, and both (in both
// GEMMs of a call) take the same decision from them: if carrying the small remainders as (mostly
// empty) main tiles costs no more rounds of the chip, weighted by the K length of each GEMM,
// than the main tiles alone plus the small tiles at 0.6 of a main tile each (a figure that
// reproduces which form measured faster on six layer shapes), the main launches take every
// remainder and the small launches find nothing to do.
// Inclusive prefix sum over the wave by DPP: four shifted adds inside each row of 16 lanes, then
// the totals of rows 0 and 2 go to rows 1 and 3, and the total of rows 0-1 to rows 2 and 3.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ int dpp_add(int x) {
  return x + __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, 0xF, true);
}
__device__ __forceinline__ int wave_scan_add(int x) {
  x = dpp_add<0x111, 0xF>(x);   // row_shr:1
  x = dpp_add<0x112, 0xF>(x);   // row_shr:2
  x = dpp_add<0x114, 0xF>(x);   // row_shr:4
  x = dpp_add<0x118, 0xF>(x);   // row_shr:8
  x = dpp_add<0x142, 0xA>(x);   // row_bcast:15 into rows 1 and 3
  x = dpp_add<0x143, 0xC>(x);   // row_bcast:31 into rows 2 and 3
  return x;
}

template <bool SPLIT = false>
__device__ __forceinline__ bool decode_tile(const GemmArgs& p, TileCoord& tc) {
  const int32_t* __restrict__ offsets = p.offsets;
  const int E = p.E, n_tiles = p.n_tiles, bm = p.bm_main, mode = p.mode;
  const int lane = lane_id();
  const int per = (E + MOE_WAVE - 1) / MOE_WAVE;  // <= 4
  const int e0 = lane * per;
  int mt[4], ob[4], oe[4];                       // tiles, first and end row of this lane's experts
  int t_all[4], t_small[4];
  int n_all = 0, n_small = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int e = e0 + i;
    ob[i] = 0;
    oe[i] = 0;
    t_all[i] = 0;
    t_small[i] = 0;
    if (i < per && e < E) {
      ob[i] = offsets[e];
      oe[i] = offsets[e + 1];
      const int c = max(oe[i] - ob[i], 0);
      const int full = c / bm, rem = c % bm;
      t_all[i] = full + (rem > 0 ? 1 : 0);
      t_small[i] = (rem > 0 && rem <= SMALL_ROWS) ? 1 : 0;
    }
    n_all += t_all[i];
    n_small += t_small[i];
  }
  // prefix sums over the experts (lane order = expert order) of both counts at once; the mode's own
  // list is a combination of the two
  const int incl_all = wave_scan_add(n_all), incl_small = wave_scan_add(n_small);
  bool fold = false;                             // small remainders ride in the main launch
  int small_beside = 0;                          // ... or run as small tiles beside this main launch
  if (mode == TILES_MAIN || mode == TILES_SMALL) {
    n_all = __builtin_amdgcn_readlane(incl_all, MOE_WAVE - 1);
    n_small = __builtin_amdgcn_readlane(incl_small, MOE_WAVE - 1);
    // (tile counts fit 32 bits: the host refuses grids beyond 2^31 - 1 blocks, and a grid is an
    // upper bound of its tile count)
    const uint32_t cu = p.n_cu > 0 ? p.n_cu : 256;
    int64_t cost_fold = 0, cost_split = 0;       // in tenths of a tile-stage on every CU
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const uint32_t tiles_all = static_cast<uint32_t>(n_all) * p.pair_n_tiles[g];
      const uint32_t tiles_small = static_cast<uint32_t>(n_small) * p.pair_n_tiles[g];
      const uint32_t rounds_all = (tiles_all + cu - 1) / cu;
      const uint32_t rounds_main = (tiles_all - tiles_small + cu - 1) / cu;
      cost_fold += static_cast<int64_t>(p.pair_kt[g]) * rounds_all * cu * 10;
      cost_split += static_cast<int64_t>(p.pair_kt[g]) *
                    (static_cast<int64_t>(rounds_main) * cu * 10 + static_cast<int64_t>(tiles_small) * 6);
    }
    fold = cost_fold <= cost_split;
    small_beside = __builtin_amdgcn_readfirstlane((mode == TILES_MAIN && !fold && n_small > 0) ? 1 : 0);
  }
  int local = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int t = t_all[i];
    if (mode == TILES_MAIN) t = fold ? t_all[i] : t_all[i] - t_small[i];
    else if (mode == TILES_SMALL) t = fold ? 0 : t_small[i];
    mt[i] = t;
    local += t;
  }
  int incl = incl_all;
  if (mode == TILES_MAIN) incl = fold ? incl_all : incl_all - incl_small;
  else if (mode == TILES_SMALL) incl = fold ? 0 : incl_small;
  const int total = __builtin_amdgcn_readlane(incl, MOE_WAVE - 1) * n_tiles;
  const int per_xcd = (total + 7) / 8;
  const int xcd = blockIdx.x & 7;
  const int slot = blockIdx.x >> 3;
  int vid = xcd * per_xcd + slot;
  tc.part = 0;
  tc.nparts = 1;
  tc.pslot = 0;
  if (SPLIT && p.split_ws) {
    // The tiles of an XCD's range run in rounds of its compute units.  If the last round is at
    // most half full, its tiles are cut along K into as many parts as fit the idle units (every
    // block of both launches takes the same decision from the same numbers); the grid of the GEMM
    // has a round of extra blocks for the parts.
    const int cus_x = max(1, (p.n_cu > 0 ? p.n_cu : 256) / 8);
    const int full_x = per_xcd / cus_x * cus_x;
    const int tail_x = per_xcd - full_x;
    int parts = 1;
    if (tail_x > 0 && 2 * tail_x <= cus_x)
      parts = min(min(cus_x / tail_x, SPLIT_MAX_PARTS), (p.K / BK_ELEMS) / SPLIT_MIN_STAGES);
    // small tiles in a launch of their own beside this one take the idle units already
    if (parts < 2 || small_beside) parts = 1;
    if (p.split_phase == 1) {
      // the summing launch: block (xcd, t) takes split tile t of the XCD's last round
      if (parts == 1 || slot >= tail_x) return false;
      vid = xcd * per_xcd + full_x + slot;
      tc.nparts = parts;
      tc.pslot = xcd * cus_x + slot * parts;
    } else if (slot >= full_x) {
      const int j = slot - full_x;
      const int t_local = j / parts;
      if (t_local >= tail_x) return false;
      vid = xcd * per_xcd + full_x + t_local;
      tc.part = j - t_local * parts;
      tc.nparts = parts;
      tc.pslot = xcd * cus_x + j;                // j < tail_x * parts <= cus_x
    }
    if (vid >= total) return false;
  } else if (slot >= per_xcd || vid >= total) {
    return false;
  }
  int run = incl - local;
  int found_e = -1, found_local = 0, found_mt = 1, found_ob = 0, found_oe = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int s = run * n_tiles;
    if (mt[i] > 0 && vid >= s && vid < s + mt[i] * n_tiles) {
      found_e = e0 + i;
      found_local = vid - s;
      found_mt = mt[i];
      found_ob = ob[i];
      found_oe = oe[i];
    }
    run += mt[i];
  }
  const unsigned long long who = __ballot(found_e >= 0);
  if (who == 0ull) return false;  // inconsistent offsets: no tile
  const int src = __ffsll(static_cast<long long>(who)) - 1;   // wave-uniform: reads of that lane
  const int e = __builtin_amdgcn_readlane(found_e, src);
  const int loc = __builtin_amdgcn_readlane(found_local, src);
  const int m_tiles = __builtin_amdgcn_readlane(found_mt, src);
  const int m_idx = loc % m_tiles;
  // the lane that owns the expert already holds its row range: no second trip to memory
  const int seg_begin = max(__builtin_amdgcn_readlane(found_ob, src), 0);
  const int seg_end = min(__builtin_amdgcn_readlane(found_oe, src), p.rows);
  tc.e = e;
  tc.n_tile = loc / m_tiles;
  if (mode == TILES_EVEN) {
    // the segment's 16-row sub-tiles are dealt evenly to its ceil(c / bm) tiles
    const int sub = (seg_end - seg_begin + 15) / 16;
    tc.m_begin = seg_begin + (m_idx * sub / m_tiles) * 16;
    tc.m_end = min(seg_end, seg_begin + ((m_idx + 1) * sub / m_tiles) * 16);
  } else if (mode == TILES_SMALL) {
    tc.m_begin = seg_begin + ((seg_end - seg_begin) / bm) * bm;
    tc.m_end = seg_end;
  } else {
    tc.m_begin = seg_begin + m_idx * bm;
    tc.m_end = min(seg_end, tc.m_begin + bm);
  }
  return tc.m_begin < tc.m_end;
}

// silu(g) * u with the hardware exponential and reciprocal (about 1 ulp each; the result is
// rounded to bf16 right after)
__device__ __forceinline__ float silu_mul(float g, float u) {
  return g * u * __builtin_amdgcn_rcpf(1.0f + __expf(-g));
}

// --------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// --------------------------------------------------------------------------------------------
constexpr int BROWS = 256;      // weight rows per block tile
constexpr int BK = BK_ELEMS;    // K elements per stage
constexpr int ROWB = BK * 2;    // bytes per tile row in LDS (eight 16-byte chunks)

// Chunk swizzle of a 128-byte tile row: XOR with the row so that 16 consecutive rows x one
// logical chunk cover a 256-byte bank window exactly once.
__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N <= 20, "vmcnt immediate");
#define MOE_VMCNT_CASE(n) \
  if constexpr (N == n) asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory");
  MOE_VMCNT_CASE(0) MOE_VMCNT_CASE(1) MOE_VMCNT_CASE(2) MOE_VMCNT_CASE(3) MOE_VMCNT_CASE(4)
  MOE_VMCNT_CASE(5) MOE_VMCNT_CASE(6) MOE_VMCNT_CASE(7) MOE_VMCNT_CASE(8) MOE_VMCNT_CASE(9)
  MOE_VMCNT_CASE(10) MOE_VMCNT_CASE(11) MOE_VMCNT_CASE(12) MOE_VMCNT_CASE(13) MOE_VMCNT_CASE(14)
  MOE_VMCNT_CASE(15) MOE_VMCNT_CASE(16) MOE_VMCNT_CASE(17) MOE_VMCNT_CASE(18) MOE_VMCNT_CASE(19)
  MOE_VMCNT_CASE(20)
#undef MOE_VMCNT_CASE
}

// The two-stage form (NSTAGE == 2) keeps its operands in a ring of five half-stage slots (see the
// full-tile path of the kernel), which needs equally large activation and weight halves.
constexpr bool ffn_half_ring(int bm, int nstage) { return nstage == 2 && bm == BROWS; }
constexpr int ffn_lds_bytes(int bm, int nstage) {
  return ffn_half_ring(bm, nstage) ? 5 * bm * ROWB : nstage * (bm + BROWS) * ROWB;
}

// Epilogue of the MFMA kernels.  Accumulator (v, lane) holds out[row = m-sub-tile + lane%16]
// [col = n-sub-tile + 4*(lane/16) + v]: 8-byte pieces scattered over 16 rows.  Each wave turns its
// 16-row sub-tile around in a private LDS region (row pitch = row bytes + 32: the 32-byte runs
// that the four lanes of a row write land in 8 banks, and 8 consecutive rows cover all 64) and
// stores whole rows, 16 bytes per lane, so the L2 sees full-line writes.  Starts with a barrier:
// every wave must be done with whatever else the block kept in LDS.
template <int BM, bool GATED, int WM, int WN, int NSTAGE>
__device__ __forceinline__ void ffn_store_tile(
    const f32x4_t (&acc)[BROWS / WN / 16][BM / WM / 16], const TileCoord& tc, const GemmArgs& p,
    unsigned char* lds, int wave, int lane, int mi_valid, int wave_row0) {
  constexpr int NW = WM * WN;
  constexpr int MI = BM / WM / 16;
  constexpr int NI = BROWS / WN / 16;
  constexpr int NIH = GATED ? NI / 2 : NI;
  constexpr int BN_OUT = GATED ? 128 : 256;
  const int wn = wave % WN;
  const int l16 = lane & 15;
  const int N = p.N;
  const int n0 = tc.n_tile * BN_OUT;
  __builtin_amdgcn_s_barrier();                   // every wave is done with the K-loop stages
  asm volatile("" ::: "memory");
  constexpr int CW = NIH * 16;                    // output columns of this wave
  constexpr int PITCH = CW * 2 + 32;              // bytes
  constexpr int LPR = CW * 2 / 16;                // lanes that store one row
  constexpr int RPI = 64 / LPR;                   // rows per store instruction
  static_assert(16 % RPI == 0 && NW * 16 * PITCH <= ffn_lds_bytes(BM, NSTAGE), "epilogue staging");
  unsigned char* region = lds + wave * (16 * PITCH);
  bf16_t* out = static_cast<bf16_t*>(p.out);
  const int col0 = n0 + wn * CW;                  // first output column of this wave
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    if (mi < mi_valid) {                          // wave-uniform
#pragma unroll
      for (int ni = 0; ni < NIH; ++ni) {
        float o[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (GATED)
            o[u] = silu_mul(acc[ni][mi][u], acc[GATED ? ni + NIH : ni][mi][u]);
          else
            o[u] = acc[ni][mi][u];
        }
        const int c = ni * 16 + 4 * (lane >> 4);
        *reinterpret_cast<uint2*>(region + l16 * PITCH + c * 2) =
            make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // same wave: writes land before the reads
      const int row_base = tc.m_begin + wave_row0 + mi * 16;
#pragma unroll
      for (int it = 0; it < 16 / RPI; ++it) {
        const int r = it * RPI + lane / LPR;
        const int c = (lane % LPR) * 8;           // first column of this lane's 16 bytes
        const uint4 v = *reinterpret_cast<const uint4*>(region + r * PITCH + c * 2);
        const int gr = row_base + r;
        if (gr < tc.m_end && col0 + c < N)
          *reinterpret_cast<uint4*>(out + static_cast<int64_t>(gr) * N + col0 + c) = v;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the region is reused
    }
  }
}

// BM x 256 block tile, WM x WN waves, NSTAGE LDS stages of 64 K-elements.
// NSTAGE == 2: hand-ordered pipeline (large tiles, MFMA/L2 bound).
// NSTAGE  > 2: ring with NSTAGE-1 stages of loads in flight (small tiles, latency bound).
// SPLIT: tiles of the last, partial round may be cut along K (see decode_tile): a part leaves its
// fp32 accumulators in the workspace instead of storing the tile, and ffn_sum_parts_kernel, the
// next launch on the stream, adds the parts in part order and runs the epilogue.
template <int BM, bool GATED, int WM, int WN, int NSTAGE, bool SPLIT = false>
__global__ __launch_bounds__(WM * WN * 64) void ffn_mfma_kernel(GemmArgs p) {
  constexpr int NW = WM * WN;                     // waves per block
  constexpr int KSTEPS = BK / 32;                 // MFMA k-steps per stage
  constexpr int MI = BM / WM / 16;                // 16-row activation sub-tiles per wave
  constexpr int NI = BROWS / WN / 16;             // 16-row weight sub-tiles per wave
  constexpr int NIH = GATED ? NI / 2 : NI;        // gated: sub-tiles per weight matrix
  constexpr int STAGE = (BM + BROWS) * ROWB;      // bytes per stage
  constexpr int NLOAD = (BM + BROWS) / 8 / NW;    // direct-to-LDS instructions per wave per stage
  constexpr int NLA = BM / 8 / NW;                // ... of which load activation rows
  constexpr int NLB = 128 / 8 / NW;               // ... per 128 weight rows
  constexpr int BN_OUT = GATED ? 128 : 256;       // output columns per block tile
  static_assert(NLA * 8 * NW == BM && NLB * 8 * NW == 128 && MI >= 1 && NIH >= 1, "tile shape");
  static_assert(KSTEPS == 2, "the pipelines below are written for two k-steps per stage");
  static_assert(NSTAGE > 2 || ffn_half_ring(BM, NSTAGE), "NSTAGE == 2 means the half-stage ring");
  extern __shared__ __align__(1024) unsigned char lds[];

  TileCoord tc;
  if (!decode_tile<SPLIT>(p, tc)) return;

  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);
  const int wm = wave / WN, wn = wave % WN;
  const int K = p.K, N = p.N;
  int kt_first = 0, kt_count = K / BK;            // this block's K stages
  if (SPLIT && tc.nparts > 1) {
    kt_first = tc.part * kt_count / tc.nparts;
    kt_count = (tc.part + 1) * kt_count / tc.nparts - kt_first;
  }
  const int KT = kt_count;
  const int n0 = tc.n_tile * BN_OUT;
  const bf16_t* A = static_cast<const bf16_t*>(p.a);
  const bf16_t* B0 = static_cast<const bf16_t*>(p.b0) + static_cast<int64_t>(tc.e) * N * K;
  const bf16_t* B1 = GATED ? static_cast<const bf16_t*>(p.b1) + static_cast<int64_t>(tc.e) * N * K
                           : nullptr;
  // 16-row activation sub-tiles of this wave that hold at least one valid row
  const int rows_valid = min(tc.m_end - tc.m_begin, BM);
  const int mi_valid = max(0, min(MI, (rows_valid - wm * (BM / WM) + 15) / 16));

  // ---- global -> LDS assignment: instruction i of this wave fills row group g = i*NW + wave
  //      (8 rows x 8 chunks = 1 KiB).  Which matrix a row group belongs to depends on i alone,
  //      so each instruction has a uniform 64-bit base and a 32-bit per-lane offset.  Rows past
  //      the end of the segment (or of the weight matrix) re-read the last valid row.
  const bool gathered = p.src_assign != nullptr;  // uniform
  const int k_first = kt_first * BK;              // first K element of this block
  const unsigned char* base_a = reinterpret_cast<const unsigned char*>(
      (gathered ? A : A + static_cast<int64_t>(tc.m_begin) * K) + k_first);
  const unsigned char* base_b0 =
      reinterpret_cast<const unsigned char*>(B0 + static_cast<int64_t>(n0) * K + k_first);
  const unsigned char* base_b1 =
      GATED ? reinterpret_cast<const unsigned char*>(B1 + static_cast<int64_t>(n0) * K + k_first)
            : nullptr;
  uint32_t soff[NLOAD];
#pragma unroll
  for (int i = 0; i < NLOAD; ++i) {
    const int g = i * NW + wave;
    const int row = g * 8 + (lane >> 3);          // row in the stage: [0,BM) x rows, then weights
    const int chunk = (lane & 7) ^ swz(row);      // the chunk of the row this lane fetches
    int r;                                        // row relative to the instruction's base
    if (i < NLA) {
      r = min(row, rows_valid - 1);
      // gathered: the offset is taken from the start of `a` (the host checks that it fits 31 bits)
      if (gathered) r = a_row_of(p, tc.m_begin + r);
    } else {
      const int br = row - BM;
      r = GATED ? min(br & 127, N - 1 - n0) : min(br, N - 1 - n0);
    }
    soff[i] = static_cast<uint32_t>(r) * static_cast<uint32_t>(K) * 2u + static_cast<uint32_t>(chunk) * 16u;
  }
  // buffer resources (raw, stride 0) based at the first row of each operand of this tile: the
  // per-lane 32-bit offset and a scalar K offset replace 64-bit per-lane address arithmetic
  const __amdgpu_buffer_rsrc_t rs_a =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(base_a), 0, 0x7FFFFFFF, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_b0 =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(base_b0), 0, 0x7FFFFFFF, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_b1 = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<unsigned char*>(GATED ? base_b1 : base_b0), 0, 0x7FFFFFFF, 0x00020000);
  // instruction i of stage kt, written to LDS byte offset dst (1 KiB per wave instruction)
  auto issue_load_at = [&](int i, int kt, int dst) {
    const __amdgpu_buffer_rsrc_t rs = (i < NLA) ? rs_a : (!GATED || i < NLA + NLB) ? rs_b0 : rs_b1;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        rs, (__attribute__((address_space(3))) void*)(lds + dst), 16,
        static_cast<int>(soff[i]), kt * ROWB, 0, 0);
  };
  auto issue_load = [&](int i, int kt, int stage) {
    issue_load_at(i, kt, stage * STAGE + (i * NW + wave) * 1024);
  };

  // ---- LDS read addresses of the MFMA fragments ------------------------------------------------
  // A lane holds, for row lane%16 of a 16-row sub-tile, the 8 K-elements of one 16-byte chunk of
  // the k-step's four.  Which chunk goes to which lane group is free as long as both operands
  // agree (it only permutes the K order inside the MFMA).  The LDS serves a 16-byte read in
  // passes of lanes {0-7, 32-39}, {8-15, 40-47}, ...: lane groups 0 and 2 therefore take chunks
  // that differ in bit 0 (0 and 1; groups 1 and 3 take 2 and 3), which with the row swizzle
  // makes every pass touch each bank once.
  const int l16 = lane & 15;
  const int f = swz(l16);                         // sub-tile bases are multiples of 16 rows
  const int kgrp = ((lane >> 4) & 1) * 2 + (lane >> 5);
  int koff[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) koff[kk] = (((kk * 4 + kgrp) ^ f) << 4);
  const int x_base = (wm * (BM / WM) + l16) * ROWB;
  // first weight row of sub-tile ni relative to the wave's own first weight row
  auto w_sub = [](int ni) { return GATED ? (ni / NIH) * 128 + (ni % NIH) * 16 : ni * 16; };
  const int w_base = (BM + (GATED ? wn * (NIH * 16) : wn * (NI * 16)) + l16) * ROWB;

  f32x4_t acc[NI][MI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[ni][mi][v] = 0.f;

  // compiler-scheduled stage: used for partial tiles and by the ring pipeline
  auto compute_at = [&](int off_a, int off_w) {
    const unsigned char* sa = lds + off_a;
    const unsigned char* sw = lds + off_w - BM * ROWB;    // w_base counts rows from the stage's first
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      bf16x8_t xf[MI], wf[NI];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        if (mi < mi_valid)
          xf[mi] = *reinterpret_cast<const bf16x8_t*>(sa + x_base + mi * 16 * ROWB + koff[kk]);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        wf[ni] = *reinterpret_cast<const bf16x8_t*>(sw + w_base + w_sub(ni) * ROWB + koff[kk]);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          if (mi < mi_valid)
            acc[ni][mi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[ni], xf[mi], acc[ni][mi], 0, 0, 0);
    }
  };
  auto compute_guarded = [&](int stage) { compute_at(stage * STAGE, stage * STAGE + BM * ROWB); };

  if constexpr (NSTAGE > 2) {
    // ---- ring pipeline: the loads of stage kt+DIST are issued at the start of stage kt -------
    constexpr int DIST = NSTAGE - 1;
#pragma unroll
    for (int s = 0; s < DIST; ++s)
      if (s < KT) {
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) issue_load(i, s, s);
      }
    for (int kt = 0; kt < KT; ++kt) {
      // the loads of stage kt are the oldest outstanding; up to DIST-1 later stages may follow
      const int later = min(DIST - 1, KT - 1 - kt);
      if (later >= 2) wait_vmcnt<2 * NLOAD>();
      else if (later == 1) wait_vmcnt<NLOAD>();
      else wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();     // stage kt landed for all waves; the slot of kt-1 is free
      asm volatile("" ::: "memory");
      if (kt + DIST < KT) {
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) issue_load(i, kt + DIST, (kt + DIST) % NSTAGE);
      }
      if (mi_valid > 0) compute_guarded(kt % NSTAGE);
    }
  } else if (mi_valid < MI) {
    // ---- partial tile in the ring of five half-stage slots: the loads, slots and barriers of the
    //      full-tile path below (waves of one block take either path), compiler-scheduled MFMAs
    constexpr int HALF = BM * ROWB;
    auto issue_act = [&](int kt, int slot) {
#pragma unroll
      for (int j = 0; j < NLA; ++j) issue_load_at(j, kt, slot * HALF + (j * NW + wave) * 1024);
    };
    auto issue_wgt = [&](int kt, int slot) {
#pragma unroll
      for (int j = 0; j < NLA; ++j) issue_load_at(NLA + j, kt, slot * HALF + (j * NW + wave) * 1024);
    };
    issue_act(0, 0);
    issue_wgt(0, 1);
    if (KT > 1) {
      issue_act(1, 2);
      issue_wgt(1, 3);
    }
    if (KT > 2) {
      issue_act(2, 4);
      wait_vmcnt<3 * NLA>();
    } else if (KT > 1) {
      wait_vmcnt<2 * NLA>();
    } else {
      wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    int slot_a = 0;                                 // slot of A(kt); W(kt) sits in the next one
    for (int kt = 0; kt < KT; ++kt) {
      const int slot_w = slot_a == 4 ? 0 : slot_a + 1;
      if (mi_valid > 0) compute_at(slot_a * HALF, slot_w * HALF);
      if (kt + 2 < KT) wait_vmcnt<NLA>();           // A(kt+2) may still fly
      else wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      if (kt + 2 < KT) issue_wgt(kt + 2, slot_a);
      if (kt + 3 < KT) issue_act(kt + 3, slot_w);
      slot_a = slot_w == 4 ? 0 : slot_w + 1;
    }
  } else {
#define MOE_RD(dst, addr, off) \
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "i"(off) : "memory")
#define MOE_MFMA(c, w, x) \
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(w), "v"(x))
#define MOE_W_OFF(ni) ((GATED ? ((ni) / NIH) * 128 + ((ni) % NIH) * 16 : (ni) * 16) * ROWB)
    {
      // ---- full tile, ring of five half-stage slots: hand-ordered pipeline -----------------------
      // A stage is two halves of 32 KiB, the activation rows A(kt) and the weight rows W(kt); half
      // number h = 2*kt (A) or 2*kt + 1 (W) lives in slot h % 5 of a 160 KiB ring.  Two slots are
      // being multiplied, and up to three halves are in flight: the L2 delivers more to a CU that
      // keeps more requests outstanding, and a plain double buffer has at most one stage in flight
      // and none at each barrier.
      //
      // A stage holds two k-steps (32 K-elements each).  Weight fragments live in ONE register
      // set: as soon as the MFMAs that use w[ni] have been issued, w[ni] is re-read for the next
      // k-step, so every LDS read has a whole k-step of MFMAs (its own wave's and the SIMD's other
      // wave's) to land.  Activation fragments alternate between two sets.  LDS reads return in
      // order, so "the fragment I need has landed" is s_waitcnt lgkmcnt(reads issued after it) =
      // NI + MI - 1.  Inline asm pins the order; the compiler does not see these LDS reads, so it
      // inserts no waits of its own.
      // The stage's one barrier sits between its two k-steps.  Before the barrier of stage kt a
      // wave waits until its own loads of W(kt+1) have landed (A(kt+2), issued after them, may
      // still fly) and for its last LDS reads of the stage's two slots; after it, those two slots
      // take W(kt+2) and A(kt+3), and the fragments of stage kt+1 may be read.
      static_assert(BM == BROWS && NLA == 2 * NLB, "halves of equal size");
      constexpr int HALF = BM * ROWB;
      constexpr int NSLOT = 5;
      static_assert(NSLOT * HALF == ffn_lds_bytes(BM, NSTAGE), "ring size");
      // LDS byte addresses of this lane's fragments: per pair of slots (the slot's parity goes into
      // the instruction's 16-bit offset), per k-step
      int xad[3][KSTEPS], wad[3][KSTEPS];
#pragma unroll
      for (int pr = 0; pr < 3; ++pr)
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
          xad[pr][kk] = pr * 2 * HALF + x_base + koff[kk];
          wad[pr][kk] = pr * 2 * HALF + (w_base - BM * ROWB) + koff[kk];
        }
      static_assert(HALF + MOE_W_OFF(NI - 1) < 65536 && HALF + (MI - 1) * 16 * ROWB < 65536,
                    "ds_read offset field");
      bf16x8_t xA[MI], xB[MI], wf[NI];
      constexpr int PEND = NI + MI - 1;
      static_assert(PEND <= 15, "lgkmcnt immediate");
      // the wave's NLA instructions of one half of stage kt into `slot`
      auto issue_half = [&](auto weights_c, int kt, auto slot_c) {
        constexpr int FIRST = decltype(weights_c)::value ? NLA : 0;
        constexpr int SLOT = decltype(slot_c)::value;
#pragma unroll
        for (int j = 0; j < NLA; ++j)
          issue_load_at(FIRST + j, kt, SLOT * HALF + (j * NW + wave) * 1024);
      };
      using ActHalf = std::false_type;
      using WgtHalf = std::true_type;
      auto stage_body = [&](int kt, auto phase_c) {
        constexpr int PH = decltype(phase_c)::value;            // kt % 5
        constexpr int SA = (2 * PH) % NSLOT, SW = (2 * PH + 1) % NSLOT;        // this stage's slots
        constexpr int NA = (2 * PH + 2) % NSLOT, NWT = (2 * PH + 3) % NSLOT;   // the next stage's
        // k-step 0 multiplies (wf, xA) and fetches k-step 1's fragments
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) MOE_RD(xB[mi], xad[SA / 2][1], (SA & 1) * HALF + mi * 16 * ROWB);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
          asm volatile("s_waitcnt lgkmcnt(%0)" ::"i"(PEND) : "memory");
#pragma unroll
          for (int mi = 0; mi < MI; ++mi) MOE_MFMA(acc[ni][mi], wf[ni], xA[mi]);
          MOE_RD(wf[ni], wad[SW / 2][1], (SW & 1) * HALF + MOE_W_OFF(ni));
        }
        if (kt + 2 < KT)                                        // wave-uniform: A(kt+2) is in flight
          asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"i"(NLA) : "memory");
        else
          asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // this stage's slots are free (their last fragments sit in registers)
        if (kt + 2 < KT) issue_half(WgtHalf{}, kt + 2, std::integral_constant<int, SA>{});
        if (kt + 3 < KT) issue_half(ActHalf{}, kt + 3, std::integral_constant<int, SW>{});
        // k-step 1 multiplies (wf, xB) and fetches the first fragments of stage kt+1; after the
        // last stage these reads return stale LDS and go unused
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) MOE_RD(xA[mi], xad[NA / 2][0], (NA & 1) * HALF + mi * 16 * ROWB);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
          for (int mi = 0; mi < MI; ++mi) MOE_MFMA(acc[ni][mi], wf[ni], xB[mi]);
          MOE_RD(wf[ni], wad[NWT / 2][0], (NWT & 1) * HALF + MOE_W_OFF(ni));
        }
      };
      // prologue: A(0), W(0), A(1), W(1), A(2) in this order; stage 0 must have landed
      issue_half(ActHalf{}, 0, std::integral_constant<int, 0>{});
      issue_half(WgtHalf{}, 0, std::integral_constant<int, 1>{});
      if (KT > 1) {
        issue_half(ActHalf{}, 1, std::integral_constant<int, 2>{});
        issue_half(WgtHalf{}, 1, std::integral_constant<int, 3>{});
      }
      if (KT > 2) {
        issue_half(ActHalf{}, 2, std::integral_constant<int, 4>{});
        wait_vmcnt<3 * NLA>();
      } else if (KT > 1) {
        wait_vmcnt<2 * NLA>();
      } else {
        wait_vmcnt<0>();
      }
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) MOE_RD(xA[mi], xad[0][0], mi * 16 * ROWB);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) MOE_RD(wf[ni], wad[0][0], HALF + MOE_W_OFF(ni));
      int kt = 0;
      for (; kt + NSLOT <= KT; kt += NSLOT) {
        stage_body(kt, std::integral_constant<int, 0>{});
        stage_body(kt + 1, std::integral_constant<int, 1>{});
        stage_body(kt + 2, std::integral_constant<int, 2>{});
        stage_body(kt + 3, std::integral_constant<int, 3>{});
        stage_body(kt + 4, std::integral_constant<int, 4>{});
      }
      if (kt < KT) stage_body(kt, std::integral_constant<int, 0>{});
      if (kt + 1 < KT) stage_body(kt + 1, std::integral_constant<int, 1>{});
      if (kt + 2 < KT) stage_body(kt + 2, std::integral_constant<int, 2>{});
      if (kt + 3 < KT) stage_body(kt + 3, std::integral_constant<int, 3>{});
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the unused reads of the last stage
      // the compiler's hazard handling does not see asm MFMAs: let the last results retire
      // before ordinary VALU code reads the accumulators
      asm volatile("s_nop 15\n s_nop 15\n s_nop 15\n s_nop 15" ::: "memory");
    }
#undef MOE_RD
#undef MOE_MFMA
#undef MOE_W_OFF
  }

  if (SPLIT && tc.nparts > 1) {
    // a part of a split tile: the accumulators go to its slot, thread-major so that a thread's
    // 16 bytes sit next to its neighbours'
    constexpr int NT = NW * MOE_WAVE;
    float* mine = p.split_ws + static_cast<int64_t>(tc.pslot) * SPLIT_SLOT_FLOATS;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        *reinterpret_cast<f32x4_t*>(mine + ((ni * MI + mi) * NT + static_cast<int>(threadIdx.x)) * 4) =
            acc[ni][mi];
    return;
  }
  ffn_store_tile<BM, GATED, WM, WN, NSTAGE>(acc, tc, p, lds, wave, lane, mi_valid, wm * (BM / WM));
}

// --------------------------------------------------------------------------------------------
// Even tiles: an expert's c rows are cut into ceil(c / 320) tiles of (nearly) equal height, a
// multiple of 16 rows each, so no segment leaves a small remainder that would have to stream the
// expert's weights once more for a handful of rows: the Mixtral-shaped batch (about 1024 rows
// per expert) runs as four tiles of 256 or 272 rows per expert, whatever the counts are.
// Block tile: up to 320 activation rows x 256 weight rows, K step 64, two LDS stages of 72 KiB.
// 8 waves as 4 (rows) x 2 (weight rows); the tile's 16-row sub-tiles are dealt to the four wave
// rows as evenly as possible (each takes MIV = 0 .. 5 of them, the first wave rows one more than
// the last), so a wave holds up to 5 x 8 accumulator tiles.
//
// Per k-step a wave multiplies in two parts so that ONE register set holds the fragments of both
// operands: part 1 takes the first P1 = ceil(MIV / 2) activation sub-tiles against all eight weight
// sub-tiles; part 2 re-reads those P1 activation fragments for the next k-step, multiplies the
// other MIV - P1 sub-tiles, re-reading each weight fragment right after its last use, and re-reads
// the remaining activation fragments at its end.  Every fragment is requested at least 14 MFMAs
// before it is needed.  LDS reads return in order, so "my fragment has landed" is a count of the
// reads issued after it.  A stage's barrier sits between the two parts of its second k-step:
// by then every fragment of the stage is in registers, the stage's buffer takes the loads of the
// stage after next, and the other buffer (landed: vmcnt(0)) is read from.
constexpr int EVEN_BM = 320;
constexpr int EVEN_STAGE = (EVEN_BM + BROWS) * ROWB;
constexpr int EVEN_LDS = 2 * EVEN_STAGE;

// How the tile's sub-tiles are dealt to wave row wm (of 4): count and first row.
__device__ __forceinline__ void even_wave_rows(int rows_valid, int wm, int& miv, int& row0) {
  const int nsub = (rows_valid + 15) >> 4;
  const int q = nsub >> 2, r = nsub & 3;
  miv = q + (wm < r ? 1 : 0);
  row0 = 16 * (wm * q + min(wm, r));
}

template <bool GATED, bool SPLIT>
__global__ __launch_bounds__(512) void ffn_even_kernel(GemmArgs p) {
  constexpr int NW = 8, WN = 2;
  constexpr int BM = EVEN_BM, MI = 5, NI = 8;
  constexpr int NIH = GATED ? NI / 2 : NI;
  constexpr int STAGE = EVEN_STAGE;
  constexpr int NLA = BM / 8 / NW;                // 5 activation row groups per wave and stage
  constexpr int NLW = BROWS / 8 / NW;             // 4 weight row groups
  constexpr int BN_OUT = GATED ? 128 : 256;
  extern __shared__ __align__(1024) unsigned char lds[];

  TileCoord tc;
  if (!decode_tile<SPLIT>(p, tc)) return;

  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);
  const int wm = wave / WN, wn = wave % WN;
  const int K = p.K, N = p.N;
  int kt_first = 0, kt_count = K / BK;
  if (SPLIT && tc.nparts > 1) {
    kt_first = tc.part * kt_count / tc.nparts;
    kt_count = (tc.part + 1) * kt_count / tc.nparts - kt_first;
  }
  const int KT = kt_count;
  const int n0 = tc.n_tile * BN_OUT;
  const bf16_t* A = static_cast<const bf16_t*>(p.a);
  const bf16_t* B0 = static_cast<const bf16_t*>(p.b0) + static_cast<int64_t>(tc.e) * N * K;
  const bf16_t* B1 = GATED ? static_cast<const bf16_t*>(p.b1) + static_cast<int64_t>(tc.e) * N * K
                           : nullptr;
  const int rows_valid = min(tc.m_end - tc.m_begin, BM);
  int miv, row0;
  even_wave_rows(rows_valid, wm, miv, row0);

  // ---- global -> LDS: 8-row groups of 1 KiB; this wave fills activation groups i*8 + wave
  //      (only those that hold a valid row) and weight groups i*8 + wave
  const bool gathered = p.src_assign != nullptr;
  const int k_first = kt_first * BK;
  const unsigned char* base_a = reinterpret_cast<const unsigned char*>(
      (gathered ? A : A + static_cast<int64_t>(tc.m_begin) * K) + k_first);
  const unsigned char* base_b0 =
      reinterpret_cast<const unsigned char*>(B0 + static_cast<int64_t>(n0) * K + k_first);
  const unsigned char* base_b1 =
      GATED ? reinterpret_cast<const unsigned char*>(B1 + static_cast<int64_t>(n0) * K + k_first)
            : nullptr;
  const int groups_valid = (rows_valid + 7) >> 3;
  const int n_act = min(NLA, max(0, (groups_valid - wave + NW - 1) / NW));   // wave-uniform
  uint32_t soff_a[NLA], soff_w[NLW];
#pragma unroll
  for (int i = 0; i < NLA; ++i) {
    const int row = (i * NW + wave) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ swz(row);
    int r = min(row, rows_valid - 1);
    if (gathered) r = a_row_of(p, tc.m_begin + r);
    soff_a[i] = static_cast<uint32_t>(r) * static_cast<uint32_t>(K) * 2u + static_cast<uint32_t>(chunk) * 16u;
  }
#pragma unroll
  for (int i = 0; i < NLW; ++i) {
    const int br = (i * NW + wave) * 8 + (lane >> 3);          // row of the weight tile (BM % 16 == 0)
    const int chunk = (lane & 7) ^ swz(br);
    const int r = GATED ? min(br & 127, N - 1 - n0) : min(br, N - 1 - n0);
    soff_w[i] = static_cast<uint32_t>(r) * static_cast<uint32_t>(K) * 2u + static_cast<uint32_t>(chunk) * 16u;
  }
  const __amdgpu_buffer_rsrc_t rs_a =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(base_a), 0, 0x7FFFFFFF, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_b0 =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(base_b0), 0, 0x7FFFFFFF, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_b1 = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<unsigned char*>(GATED ? base_b1 : base_b0), 0, 0x7FFFFFFF, 0x00020000);
  auto issue_stage = [&](int kt, int buf) {
#pragma unroll
    for (int i = 0; i < NLA; ++i)
      if (i < n_act)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rs_a, (__attribute__((address_space(3))) void*)(lds + buf * STAGE + (i * NW + wave) * 1024),
            16, static_cast<int>(soff_a[i]), kt * ROWB, 0, 0);
#pragma unroll
    for (int i = 0; i < NLW; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          (!GATED || i < NLW / 2) ? rs_b0 : rs_b1,
          (__attribute__((address_space(3))) void*)(lds + buf * STAGE + BM * ROWB + (i * NW + wave) * 1024),
          16, static_cast<int>(soff_w[i]), kt * ROWB, 0, 0);
  };

  // ---- LDS addresses of this lane's fragments, per buffer and k-step (chunk order as in
  //      ffn_mfma_kernel: lane groups 0..3 take chunks 0, 2, 1, 3 of the k-step)
  const int l16 = lane & 15;
  const int f = swz(l16);
  const int kgrp = ((lane >> 4) & 1) * 2 + (lane >> 5);
  int xa[2][2], wa[2][2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const int ko = ((kk * 4 + kgrp) ^ f) << 4;
      xa[b][kk] = b * STAGE + (row0 + l16) * ROWB + ko;
      wa[b][kk] = b * STAGE + (BM + wn * (NIH * 16) + l16) * ROWB + ko;
    }

  f32x4_t acc[NI][MI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) acc[ni][mi] = f32x4_t{0.f, 0.f, 0.f, 0.f};

#define MOE_RD(dst, addr, off) \
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "i"(off) : "memory")
#define MOE_MFMA(c, w, x) \
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(w), "v"(x))
#define MOE_W_OFF(ni) ((GATED ? ((ni) / NIH) * 128 + ((ni) % NIH) * 16 : (ni) * 16) * ROWB)
  static_assert(MOE_W_OFF(NI - 1) < 65536 && (MI - 1) * 16 * ROWB < 65536, "ds_read offset field");

  auto k_loop = [&](auto miv_c) {
    constexpr int MIV = decltype(miv_c)::value;
    constexpr int P1 = (MIV + 1) / 2, P2 = MIV - P1;
    bf16x8_t x[MI], w[NI];
    // the fragments of a k-step are always requested in the order x[0..P1), w[0..NI), x[P1..MIV)
    auto part1 = [&]() {
      if constexpr (MIV > 0) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
          asm volatile("s_waitcnt lgkmcnt(%0)" ::"i"(NI - 1 - ni + P2) : "memory");
#pragma unroll
          for (int mi = 0; mi < P1; ++mi) MOE_MFMA(acc[ni][mi], w[ni], x[mi]);
        }
      }
    };
    auto part2 = [&](int xn, int wnx) {
      if constexpr (MIV > 0) {
#pragma unroll
        for (int mi = 0; mi < P1; ++mi) MOE_RD(x[mi], xn, mi * 16 * ROWB);
        if constexpr (P2 > 0) asm volatile("s_waitcnt lgkmcnt(%0)" ::"i"(P1) : "memory");
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
          for (int mi = P1; mi < MIV; ++mi) MOE_MFMA(acc[ni][mi], w[ni], x[mi]);
          MOE_RD(w[ni], wnx, MOE_W_OFF(ni));
        }
#pragma unroll
        for (int mi = P1; mi < MIV; ++mi) MOE_RD(x[mi], xn, mi * 16 * ROWB);
      }
    };
    auto stage = [&](int kt, auto par_c) {
      constexpr int PAR = decltype(par_c)::value;
      part1();
      part2(xa[PAR][1], wa[PAR][1]);
      part1();
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      if (kt + 2 < KT) issue_stage(kt + 2, PAR);
      // after the last stage these reads return stale LDS and go unused
      part2(xa[PAR ^ 1][0], wa[PAR ^ 1][0]);
    };
    // prologue: stages 0 and 1 requested; stage 0 must have landed for every wave
    issue_stage(0, 0);
    if (KT > 1) {
      issue_stage(1, 1);
      switch (n_act) {                              // this wave's loads of stage 1 may still fly
        case 0: wait_vmcnt<NLW>(); break;
        case 1: wait_vmcnt<NLW + 1>(); break;
        case 2: wait_vmcnt<NLW + 2>(); break;
        case 3: wait_vmcnt<NLW + 3>(); break;
        case 4: wait_vmcnt<NLW + 4>(); break;
        default: wait_vmcnt<NLW + 5>(); break;
      }
    } else {
      wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if constexpr (MIV > 0) {
#pragma unroll
      for (int mi = 0; mi < P1; ++mi) MOE_RD(x[mi], xa[0][0], mi * 16 * ROWB);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) MOE_RD(w[ni], wa[0][0], MOE_W_OFF(ni));
#pragma unroll
      for (int mi = P1; mi < MIV; ++mi) MOE_RD(x[mi], xa[0][0], mi * 16 * ROWB);
    }
    int kt = 0;
    for (; kt + 2 <= KT; kt += 2) {
      stage(kt, std::integral_constant<int, 0>{});
      stage(kt + 1, std::integral_constant<int, 1>{});
    }
    if (kt < KT) stage(kt, std::integral_constant<int, 0>{});
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // the unused reads of the last stage
    // the compiler's hazard handling does not see asm MFMAs: let the last results retire
    // before ordinary VALU code reads the accumulators
    asm volatile("s_nop 15\n s_nop 15\n s_nop 15\n s_nop 15" ::: "memory");
  };
  switch (miv) {                                    // wave-uniform
    case 0: k_loop(std::integral_constant<int, 0>{}); break;
    case 1: k_loop(std::integral_constant<int, 1>{}); break;
    case 2: k_loop(std::integral_constant<int, 2>{}); break;
    case 3: k_loop(std::integral_constant<int, 3>{}); break;
    case 4: k_loop(std::integral_constant<int, 4>{}); break;
    default: k_loop(std::integral_constant<int, 5>{}); break;
  }
#undef MOE_RD
#undef MOE_MFMA
#undef MOE_W_OFF

  if (SPLIT && tc.nparts > 1) {
    constexpr int NT = NW * MOE_WAVE;
    float* mine = p.split_ws + static_cast<int64_t>(tc.pslot) * SPLIT_SLOT_FLOATS;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        *reinterpret_cast<f32x4_t*>(mine + ((ni * MI + mi) * NT + static_cast<int>(threadIdx.x)) * 4) =
            acc[ni][mi];
    return;
  }
  ffn_store_tile<BM, GATED, 4, WN, 2>(acc, tc, p, lds, wave, lane, miv, row0);
}

// The launch after ffn_even_kernel<.., SPLIT>: adds the parts of every split tile in part order and
// stores it (see ffn_sum_parts_kernel).
template <bool GATED>
__global__ __launch_bounds__(512) void ffn_even_sum_parts_kernel(GemmArgs p) {
  constexpr int NW = 8, WN = 2, MI = 5, NI = 8;
  constexpr int NT = NW * MOE_WAVE;
  extern __shared__ __align__(1024) unsigned char lds[];
  TileCoord tc;
  if (!decode_tile<true>(p, tc)) return;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);
  int miv, row0;
  even_wave_rows(min(tc.m_end - tc.m_begin, EVEN_BM), wave / WN, miv, row0);
  f32x4_t acc[NI][MI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) acc[ni][mi] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const float* first = p.split_ws + static_cast<int64_t>(tc.pslot) * SPLIT_SLOT_FLOATS;
  for (int q = 0; q < tc.nparts; ++q) {
    const float* src = first + static_cast<int64_t>(q) * SPLIT_SLOT_FLOATS;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const f32x4_t v = *reinterpret_cast<const f32x4_t*>(
            src + ((ni * MI + mi) * NT + static_cast<int>(threadIdx.x)) * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[ni][mi][u] += v[u];
      }
  }
  ffn_store_tile<EVEN_BM, GATED, 4, WN, 2>(acc, tc, p, lds, wave, lane, miv, row0);
}

// The launch after a GEMM whose tiles may have been split: block (xcd, t) adds the parts of split
// tile t of the XCD's last round in part order (so the sum does not depend on scheduling) and
// stores the tile.  Finds nothing to do when no tile was split.
template <int BM, bool GATED, int WM, int WN, int NSTAGE>
__global__ __launch_bounds__(WM * WN * 64) void ffn_sum_parts_kernel(GemmArgs p) {
  constexpr int NW = WM * WN;
  constexpr int MI = BM / WM / 16;
  constexpr int NI = BROWS / WN / 16;
  constexpr int NT = NW * MOE_WAVE;
  extern __shared__ __align__(1024) unsigned char lds[];
  TileCoord tc;
  if (!decode_tile<true>(p, tc)) return;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);
  const int wm = wave / WN;
  const int rows_valid = min(tc.m_end - tc.m_begin, BM);
  const int mi_valid = max(0, min(MI, (rows_valid - wm * (BM / WM) + 15) / 16));
  f32x4_t acc[NI][MI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) acc[ni][mi] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const float* first = p.split_ws + static_cast<int64_t>(tc.pslot) * SPLIT_SLOT_FLOATS;
  for (int q = 0; q < tc.nparts; ++q) {
    const float* src = first + static_cast<int64_t>(q) * SPLIT_SLOT_FLOATS;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const f32x4_t v = *reinterpret_cast<const f32x4_t*>(
            src + ((ni * MI + mi) * NT + static_cast<int>(threadIdx.x)) * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[ni][mi][u] += v[u];
      }
  }
  ffn_store_tile<BM, GATED, WM, WN, NSTAGE>(acc, tc, p, lds, wave, lane, mi_valid, wm * (BM / WM));
}

// --------------------------------------------------------------------------------------------
// generic kernel: 64x64 output tile, K step 16, 4x4 outputs per thread, fp32 FMA
// --------------------------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ float ld_elem(const T* p);
template <> __device__ __forceinline__ float ld_elem<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld_elem<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void st_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_elem(bf16_t* p, float v) { *p = f32_to_bf16(v); }

template <typename T, bool GATED>
__global__ __launch_bounds__(256) void ffn_generic_kernel(GemmArgs p) {
  constexpr int TM = 64, TN = 64, TK = 16;
  __shared__ float As[TK][TM + 4];
  __shared__ float Bs[GATED ? 2 : 1][TK][TN + 4];
  TileCoord tc;
  if (!decode_tile(p, tc)) return;
  const int K = p.K, N = p.N;
  const int n0 = tc.n_tile * TN;
  const T* A = static_cast<const T*>(p.a);
  const T* B0 = static_cast<const T*>(p.b0) + static_cast<int64_t>(tc.e) * N * K;
  const T* B1 = GATED ? static_cast<const T*>(p.b1) + static_cast<int64_t>(tc.e) * N * K : nullptr;
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;         // thread's 4 columns / 4 rows
  const int lr = tid >> 2, lk = (tid & 3) * 4;    // loader: row 0..63, k offset 0,4,8,12
  float acc[GATED ? 2 : 1][4][4];
#pragma unroll
  for (int s = 0; s < (GATED ? 2 : 1); ++s)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[s][i][j] = 0.f;
  const int a_row = a_row_of(p, min(tc.m_begin + lr, tc.m_end - 1));
  const int b_row = min(n0 + lr, N - 1);
  for (int k0 = 0; k0 < K; k0 += TK) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int kk = k0 + lk + q;
      As[lk + q][lr] = kk < K ? ld_elem<T>(A + static_cast<int64_t>(a_row) * K + kk) : 0.f;
      Bs[0][lk + q][lr] = kk < K ? ld_elem<T>(B0 + static_cast<int64_t>(b_row) * K + kk) : 0.f;
      if constexpr (GATED)
        Bs[1][lk + q][lr] = kk < K ? ld_elem<T>(B1 + static_cast<int64_t>(b_row) * K + kk) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float av[4], bv[GATED ? 2 : 1][4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int s = 0; s < (GATED ? 2 : 1); ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j) bv[s][j] = Bs[s][kk][tx * 4 + j];
#pragma unroll
      for (int s = 0; s < (GATED ? 2 : 1); ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[s][i][j] = fmaf(av[i], bv[s][j], acc[s][i][j]);
    }
    __syncthreads();
  }
  T* out = static_cast<T*>(p.out);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gr = tc.m_begin + ty * 4 + i;
    if (gr >= tc.m_end) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = n0 + tx * 4 + j;
      if (c < N) {
        float v;
        if (GATED) {
          const float g = acc[0][i][j];
          v = g / (1.0f + expf(-g)) * acc[GATED ? 1 : 0][i][j];
        } else {
          v = acc[0][i][j];
        }
        st_elem(out + static_cast<int64_t>(gr) * N + c, v);
      }
    }
  }
}

// Compute units of the current device, looked up once per device (0 if the query fails: the
// kernels then assume 256).
static int device_cu_count() {
  static int cached[MOE_MAX_DEVICES] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MOE_MAX_DEVICES) return 0;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    cached[dev] = n;
  }
  return cached[dev];
}

// Upper bounds on the number of m-tiles that need no knowledge of the counts: an expert has at
// most floor(c/bm) full tiles (sum <= A/bm) and one remainder.
static int64_t max_m_tiles(int64_t A, int E, int bm, int mode) {
  const int64_t e_cap = E < A ? E : A;
  if (mode == TILES_SMALL) return e_cap;
  return A / bm + e_cap;   // TILES_MAIN may take every remainder: the same bound as TILES_ALL
}

template <int BM, bool GATED, int WM, int WN, int NSTAGE, bool SPLIT>
static int launch_mfma_as(GemmArgs a, int mode, int bm_main, int64_t A, hipStream_t st) {
  constexpr int lds_bytes = ffn_lds_bytes(BM, NSTAGE);
  static LdsOnce once;
  if (ensure_dynamic_lds(once,
                         reinterpret_cast<const void*>(ffn_mfma_kernel<BM, GATED, WM, WN, NSTAGE, SPLIT>),
                         lds_bytes) != MOE_OK)
    return MOE_ERR_HIP;
  a.mode = mode;
  a.bm_main = bm_main;
  a.split_phase = 0;
  if (!SPLIT) a.split_ws = nullptr;
  int64_t grid = max_m_tiles(A, a.E, bm_main, mode) * a.n_tiles;
  if (grid == 0) return MOE_OK;       // no tile of this kind can exist
  grid = (grid + 7) / 8 * 8;
  const int cu8 = (a.n_cu > 0 ? a.n_cu : 256) / 8 * 8;
  if (SPLIT) grid += cu8;             // one more round of blocks for the parts of split tiles
  if (grid > 0x7FFFFFFF) return MOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((ffn_mfma_kernel<BM, GATED, WM, WN, NSTAGE, SPLIT>),
                     dim3(static_cast<unsigned>(grid)), dim3(WM * WN * 64), lds_bytes, st, a);
  int rc = launch_status();
  if (SPLIT && rc == MOE_OK) {
    // the parts meet at the kernel boundary: one block per possible split tile
    static LdsOnce once_sum;
    if (ensure_dynamic_lds(once_sum,
                           reinterpret_cast<const void*>(ffn_sum_parts_kernel<BM, GATED, WM, WN, NSTAGE>),
                           lds_bytes) != MOE_OK)
      return MOE_ERR_HIP;
    a.split_phase = 1;
    hipLaunchKernelGGL((ffn_sum_parts_kernel<BM, GATED, WM, WN, NSTAGE>), dim3(static_cast<unsigned>(cu8)),
                       dim3(WM * WN * 64), lds_bytes, st, a);
    rc = launch_status();
  }
  return rc;
}

template <bool GATED, bool SPLIT>
static int launch_even_as(GemmArgs a, int64_t A, hipStream_t st) {
  static LdsOnce once;
  if (ensure_dynamic_lds(once, reinterpret_cast<const void*>(ffn_even_kernel<GATED, SPLIT>), EVEN_LDS) !=
      MOE_OK)
    return MOE_ERR_HIP;
  a.mode = TILES_EVEN;
  a.bm_main = EVEN_BM;
  a.split_phase = 0;
  if (!SPLIT) a.split_ws = nullptr;
  int64_t grid = max_m_tiles(A, a.E, EVEN_BM, TILES_EVEN) * a.n_tiles;
  if (grid == 0) return MOE_OK;
  grid = (grid + 7) / 8 * 8;
  const int cu8 = (a.n_cu > 0 ? a.n_cu : 256) / 8 * 8;
  if (SPLIT) grid += cu8;
  if (grid > 0x7FFFFFFF) return MOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((ffn_even_kernel<GATED, SPLIT>), dim3(static_cast<unsigned>(grid)), dim3(512),
                     EVEN_LDS, st, a);
  int rc = launch_status();
  if (SPLIT && rc == MOE_OK) {
    static LdsOnce once_sum;
    if (ensure_dynamic_lds(once_sum, reinterpret_cast<const void*>(ffn_even_sum_parts_kernel<GATED>),
                           EVEN_LDS) != MOE_OK)
      return MOE_ERR_HIP;
    a.split_phase = 1;
    hipLaunchKernelGGL((ffn_even_sum_parts_kernel<GATED>), dim3(static_cast<unsigned>(cu8)), dim3(512),
                       EVEN_LDS, st, a);
    rc = launch_status();
  }
  return rc;
}

// `split`: this launch may use the workspace for split tiles if the caller brought one.  Only
// GEMMs with a long reduction do: a part must be worth the exchange (one 256 KiB store per part,
// the summing launch), and a tile of fewer than 96 stages is too short for that (measured: the
// up-projections of the four model shapes gain nothing, their down-projections up to 27 %).
constexpr int SPLIT_MIN_K = 96 * BK_ELEMS;
template <int BM, bool GATED, int WM, int WN, int NSTAGE>
static int launch_mfma(const GemmArgs& a, int mode, int bm_main, int64_t A, hipStream_t st,
                       bool split = false) {
  return split && a.split_ws && a.K >= SPLIT_MIN_K
             ? launch_mfma_as<BM, GATED, WM, WN, NSTAGE, true>(a, mode, bm_main, A, st)
             : launch_mfma_as<BM, GATED, WM, WN, NSTAGE, false>(a, mode, bm_main, A, st);
}

template <typename T, bool GATED>
static int launch_generic(GemmArgs a, int64_t A, hipStream_t st) {
  a.mode = TILES_ALL;
  a.bm_main = 64;
  int64_t grid = max_m_tiles(A, a.E, 64, TILES_ALL) * a.n_tiles;
  grid = (grid + 7) / 8 * 8;
  if (grid > 0x7FFFFFFF) return MOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((ffn_generic_kernel<T, GATED>), dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                     st, a);
  return launch_status();
}

// Main tiles of one grouped GEMM on the MFMA path.
template <bool GATED>
static int mfma_gemm_main(const GemmArgs& g, int64_t A, hipStream_t st) {
  return launch_mfma<256, GATED, 4, 2, 2>(g, TILES_MAIN, 256, A, st, true);
}

// The small remainders of the same GEMM.
template <bool GATED>
static int mfma_gemm_small(const GemmArgs& g, int64_t A, hipStream_t st) {
  return launch_mfma<64, GATED, 2, 4, 4>(g, TILES_SMALL, 256, A, st);
}

// The remainder launches stream whole weight matrices from HBM for a few rows each, while the
// main launches are bound by the matrix pipes and the L2: run side by side they overlap.  One
// side stream per device (default priority, created on first use, kept for the life of the
// process) is forked from the caller's stream with an event and joined back with another, so
// the caller sees ordinary stream semantics; the rows the two chains touch are disjoint (a
// remainder's h rows are written and read by the side chain only, or, when the small remainders
// ride in the main launches, by the main chain only: both GEMMs of a call take that decision
// together).
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
  bool ready = false;
};
static SideStream g_side[MOE_MAX_DEVICES];
static std::mutex g_side_mutex;   // also serialises fork ... join sequences that share the events

static SideStream* side_stream_locked() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MOE_MAX_DEVICES) return nullptr;
  SideStream& s = g_side[dev];
  if (!s.ready) {
    if (hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) != hipSuccess) return nullptr;
    if (hipEventCreateWithFlags(&s.fork, hipEventDisableTiming) != hipSuccess) return nullptr;
    if (hipEventCreateWithFlags(&s.join, hipEventDisableTiming) != hipSuccess) return nullptr;
    s.ready = true;
  }
  return &s;
}

// Both GEMMs (or one of them) on the MFMA path.
static int mfma_ffn(const GemmArgs& g1, const GemmArgs& g2, bool up, bool down, int64_t A,
                    hipStream_t st) {
  int rc = MOE_OK;
  if (A / g1.E < 128) {
    // Few rows per expert (decode, small prefill batches): the call is bound by streaming each
    // expert's weights once, which the latency-hiding ring of the 64-row tiles does best, and a
    // 256-row tile would be mostly padding.  One launch per GEMM.  (Measured at the Mixtral
    // shape: 64 rows per expert 0.85 -> 0.63 ms against 128-row main tiles plus remainders.)
    if (up && (rc = launch_mfma<64, true, 2, 4, 4>(g1, TILES_ALL, 64, A, st, true)) != MOE_OK) return rc;
    if (down) rc = launch_mfma<64, false, 2, 4, 4>(g2, TILES_ALL, 64, A, st, true);
    return rc;
  }
  static const int form = [] { const char* e = getenv("MOE_FFN_FORM"); return e ? atoi(e) : 1; }();
  if (form == 1) {
    auto launch = [&](const GemmArgs& g, auto gated_c) {
      constexpr bool G = decltype(gated_c)::value;
      return g.split_ws && g.K >= SPLIT_MIN_K ? launch_even_as<G, true>(g, A, st)
                                              : launch_even_as<G, false>(g, A, st);
    };
    if (up && (rc = launch(g1, std::true_type{})) != MOE_OK) return rc;
    if (down) rc = launch(g2, std::false_type{});
    return rc;
  }
  std::lock_guard<std::mutex> lock(g_side_mutex);
  SideStream* side = side_stream_locked();
  if (!side) return MOE_ERR_HIP;
  if (hipEventRecord(side->fork, st) != hipSuccess) return MOE_ERR_HIP;
  if (hipStreamWaitEvent(side->stream, side->fork, 0) != hipSuccess) return MOE_ERR_HIP;
  // From here on the side stream must be joined back even if a launch fails.
  if (up) rc = mfma_gemm_small<true>(g1, A, side->stream);
  if (rc == MOE_OK && down) rc = mfma_gemm_small<false>(g2, A, side->stream);
  if (rc == MOE_OK && up) rc = mfma_gemm_main<true>(g1, A, st);
  if (rc == MOE_OK && down) rc = mfma_gemm_main<false>(g2, A, st);
  if (hipEventRecord(side->join, side->stream) != hipSuccess) return MOE_ERR_HIP;
  if (hipStreamWaitEvent(st, side->join, 0) != hipSuccess) return MOE_ERR_HIP;
  return rc;
}

// parts: bit 0 = gated up-projection (h), bit 1 = down-projection (y_perm)
// x_perm [T*k, d] with src_assign == nullptr, or x [T, d] with the src_assign map of the dispatch
static int grouped_ffn_impl(const moe_shape_t* shape, const void* x_perm, const int32_t* src_assign,
                            const int32_t* offsets, const void* w1, const void* w3, const void* w2,
                            void* h, void* y_perm, int parts, void* hip_stream,
                            void* split_ws = nullptr) {
  int rc = check_shape(shape);
  if (rc != MOE_OK) return rc;
  if (shape->T == 0) return MOE_OK;
  if (!x_perm || !offsets || !w1 || !w3 || !w2 || !h || !y_perm) return MOE_ERR_INVALID_ARG;
  // gathered rows are addressed with a 32-bit byte offset from the start of x
  if (src_assign && static_cast<int64_t>(shape->T) * shape->d * elem_bytes(shape->dtype) >=
                        (int64_t(1) << 31))
    return MOE_ERR_UNSUPPORTED;
  if (!aligned16(x_perm) || !aligned16(w1) || !aligned16(w3) || !aligned16(w2) || !aligned16(h) ||
      !aligned16(y_perm))
    return MOE_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int64_t A = static_cast<int64_t>(shape->T) * shape->k;
  const int d = shape->d, F = shape->F, E = shape->E;
  const int n_cu = device_cu_count();
  GemmArgs g1{x_perm, w1, w3, h, offsets, E, d, F, 0, static_cast<int>(A), TILES_ALL, 64,
              src_assign, shape->k, src_assign ? shape->T : static_cast<int>(A), n_cu, {0, 0}, {0, 0},
              static_cast<float*>(split_ws), 0};
  GemmArgs g2{h, w2, nullptr, y_perm, offsets, E, F, d, 0, static_cast<int>(A), TILES_ALL, 64,
              nullptr, 1, static_cast<int>(A), n_cu, {0, 0}, {0, 0}, static_cast<float*>(split_ws), 0};
  const bool up = parts & 1, down = parts & 2;
  if (shape->dtype == MOE_BF16 && d % 64 == 0 && F % 64 == 0) {
    g1.n_tiles = (F + 127) / 128;
    g2.n_tiles = (d + 255) / 256;
    for (GemmArgs* g : {&g1, &g2}) {
      g->pair_n_tiles[0] = g1.n_tiles;
      g->pair_n_tiles[1] = g2.n_tiles;
      g->pair_kt[0] = d / 64;
      g->pair_kt[1] = F / 64;
    }
    return mfma_ffn(g1, g2, up, down, A, st);
  }
  g1.n_tiles = (F + 63) / 64;
  g2.n_tiles = (d + 63) / 64;
  if (shape->dtype == MOE_BF16) {
    if (up) {
      rc = launch_generic<bf16_t, true>(g1, A, st);
      if (rc != MOE_OK) return rc;
    }
    if (down) rc = launch_generic<bf16_t, false>(g2, A, st);
    return rc;
  }
  if (up) {
    rc = launch_generic<float, true>(g1, A, st);
    if (rc != MOE_OK) return rc;
  }
  if (down) rc = launch_generic<float, false>(g2, A, st);
  return rc;
}

}  // namespace moe

extern "C" int moe_grouped_ffn(const moe_shape_t* shape, const void* x_perm, const int32_t* offsets,
                               const void* w1, const void* w3, const void* w2, void* h, void* y_perm,
                               void* hip_stream) {
  return moe::grouped_ffn_impl(shape, x_perm, nullptr, offsets, w1, w3, w2, h, y_perm, 3,
                               hip_stream);
}

// Bytes of the split-tile workspace on the current device: one fp32 partial tile per compute unit.
static size_t ffn_split_workspace_bytes() {
  const int n_cu = moe::device_cu_count();
  return static_cast<size_t>(n_cu > 0 ? n_cu : 256) * moe::SPLIT_SLOT_FLOATS * sizeof(float);
}

extern "C" int moe_ffn_workspace_bytes(const moe_shape_t* shape, size_t* out_bytes) {
  if (!out_bytes) return MOE_ERR_INVALID_ARG;
  const int rc = moe::check_shape(shape);
  if (rc != MOE_OK) return rc;
  *out_bytes = ffn_split_workspace_bytes();
  return MOE_OK;
}

extern "C" int moe_grouped_ffn_ws(const moe_shape_t* shape, const void* x, const int32_t* src_assign,
                                  const int32_t* offsets, const void* w1, const void* w3,
                                  const void* w2, void* h, void* y_perm, int parts, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  if (parts < 1 || parts > 3) return MOE_ERR_INVALID_ARG;
  if (workspace) {
    if (!moe::aligned16(workspace)) return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < ffn_split_workspace_bytes()) return MOE_ERR_WORKSPACE;
  }
  return moe::grouped_ffn_impl(shape, x, src_assign, offsets, w1, w3, w2, h, y_perm, parts,
                               hip_stream, workspace);
}

extern "C" int moe_grouped_ffn_gather(const moe_shape_t* shape, const void* x,
                                      const int32_t* src_assign, const int32_t* offsets,
                                      const void* w1, const void* w3, const void* w2, void* h,
                                      void* y_perm, void* hip_stream) {
  if (!src_assign) return MOE_ERR_INVALID_ARG;
  return moe::grouped_ffn_impl(shape, x, src_assign, offsets, w1, w3, w2, h, y_perm, 3, hip_stream);
}

extern "C" int moe_grouped_ffn_gather_part(const moe_shape_t* shape, const void* x,
                                           const int32_t* src_assign, const int32_t* offsets,
                                           const void* w1, const void* w3, const void* w2, void* h,
                                           void* y_perm, int part, void* hip_stream) {
  if (part != 1 && part != 2) return MOE_ERR_INVALID_ARG;
  if (!src_assign) return MOE_ERR_INVALID_ARG;
  return moe::grouped_ffn_impl(shape, x, src_assign, offsets, w1, w3, w2, h, y_perm, part,
                               hip_stream);
}

extern "C" int moe_grouped_ffn_part(const moe_shape_t* shape, const void* x_perm,
                                    const int32_t* offsets, const void* w1, const void* w3,
                                    const void* w2, void* h, void* y_perm, int part,
                                    void* hip_stream) {
  if (part != 1 && part != 2) return MOE_ERR_INVALID_ARG;
  return moe::grouped_ffn_impl(shape, x_perm, nullptr, offsets, w1, w3, w2, h, y_perm, part,
                               hip_stream);
}
