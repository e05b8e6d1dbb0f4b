// moe_grouped_ffn: the expert computation that dominates the MoE layer (Section 3.2).
// For every expert e and row r of its segment [offsets[e], offsets[e+1]):
//   h[r] = silu(W1_e x_perm[r]) * (W3_e x_perm[r]),   y_perm[r] = W2_e h[r].
// The activation rows come either from a permuted copy x_perm, or straight from x through the
// dispatch's src_assign map (moe_grouped_ffn_gather: row r is x[src_assign[r] / k]); the map only
// changes the per-lane row offset of the activation loads.
//
// Two GEMMs: a gated one (W1 and W3 tiles side by side, SwiGLU applied to the fp32
// accumulators, h stored once) and a plain one for W2.  Both are ragged grouped
// GEMMs, one launch each: the tile list is derived on the device from `offsets`, so the host
// never learns the expert loads.
//   even tiles (128 or more rows per expert on average): an expert's c rows are cut into
//          ceil(c / 320) tiles of nearly equal height (multiples of 16 rows), each against 256
//          weight rows; K step 64, two LDS stages, hand-ordered MFMA pipeline (ffn_even_kernel).
//   ring tiles (decode and small prefill batches, below 128 rows per expert: the call is bound by
//          streaming the weights once): 64-row tiles against 256 weight rows with a four-stage
//          LDS ring, three stages of loads in flight (ffn_ring_kernel).
//
// moe_grouped_ffn_ws brings a workspace of fp32 partial tiles: a tile takes a whole compute unit,
// so a GEMM runs in rounds of the chip, and when the last round of a GEMM with a long reduction
// is at most half full its tiles are computed as 2 to 4 parts of the K range on the idle units
// and added up, in part order, by a second small launch.
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
#include <type_traits>

#include "moe_internal.h"

namespace moe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

enum TileMode { TILES_FIXED = 0, TILES_EVEN = 1 };
constexpr int BK_ELEMS = 64;    // K elements per stage of the MFMA kernels

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
  int bm;           // TILES_FIXED: rows of a tile; TILES_EVEN: most rows of a tile
  // Gathered activations: row r of the GEMM is row src_assign[r] / k_div of `a` (the token that
  // assignment r belongs to) instead of row r itself.  nullptr = `a` is already permuted.
  const int32_t* src_assign;
  int k_div;
  int a_rows;       // rows of `a` (gathered row numbers are clamped to it)
  int n_cu;         // compute units of the device (tiles are split by rounds of it)
  // Split tiles (kernels built with SPLIT only): fp32 partial tiles, one slot per compute unit.
  // nullptr: no tile is split.  split_phase 0: the GEMM itself; 1: the launch after it that adds
  // up the parts of every split tile and stores it.
  float* split_ws;
  int split_phase;
  // Scattered, scaled output (plain GEMM of a k = 1 layer: the combine folded into the store):
  // GEMM row r goes to row out_map[r] of `out`, multiplied by out_scale[out_map[r]] before the
  // one rounding.  nullptr = row r of `out`, unscaled.
  const int32_t* out_map;
  const float* out_scale;
  int out_rows;     // rows of `out` (mapped row numbers are clamped to it)
  // TILES_EVEN launches without split_ws: tiles of a last round that is at most half full are cut
  // along their rows into pieces for the idle units (the grid has a round of extra blocks).
  int m_split;
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
  int sharers; // tiles and pieces of tiles of this expert that read the same weight rows
};
constexpr int MSPLIT_MAX_PIECES = 4;
constexpr int WGT_NT_MAX_SHARERS = 2;

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

// Maps a work-group to (expert, row range, n-tile).  Every wave computes this on its
// own from the device-resident offsets; returns false if the group has no tile.
// An expert with c rows has ceil(c / bm) tiles: TILES_FIXED cuts them at multiples of bm (the last
// one holds the remainder), TILES_EVEN deals the segment's 16-row sub-tiles evenly to them.
// Tile order: expert-major, then n-tile, then m-tile (m fastest), cut into 8 contiguous ranges,
// one per XCD.
template <bool SPLIT = false>
__device__ __forceinline__ bool decode_tile(const GemmArgs& p, TileCoord& tc) {
  const int32_t* __restrict__ offsets = p.offsets;
  const int E = p.E, n_tiles = p.n_tiles, bm = p.bm;
  const int lane = lane_id();
  const int per = (E + MOE_WAVE - 1) / MOE_WAVE;  // <= 4
  const int e0 = lane * per;
  int mt[4], ob[4], oe[4];                       // tiles, first and end row of this lane's experts
  int local = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int e = e0 + i;
    ob[i] = 0;
    oe[i] = 0;
    mt[i] = 0;
    if (i < per && e < E) {
      ob[i] = offsets[e];
      oe[i] = offsets[e + 1];
      mt[i] = (max(oe[i] - ob[i], 0) + bm - 1) / bm;
    }
    local += mt[i];
  }
  // prefix sum over the experts (lane order = expert order)
  const int incl = wave_scan_add(local);
  // (tile counts fit 32 bits: the host refuses grids beyond 2^31 - 1 blocks, and a grid is an
  // upper bound of its tile count)
  const int total = __builtin_amdgcn_readlane(incl, MOE_WAVE - 1) * n_tiles;
  const int per_xcd = (total + 7) / 8;
  const int xcd = blockIdx.x & 7;
  const int slot = blockIdx.x >> 3;
  int vid = xcd * per_xcd + slot;
  tc.part = 0;
  tc.nparts = 1;
  tc.pslot = 0;
  int m_pieces = 1, m_piece = 0;
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
    if (parts < 2) parts = 1;
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
  } else if (p.m_split && slot + max(1, (p.n_cu > 0 ? p.n_cu : 256) / 8) >= per_xcd) {
    // No workspace: the tiles of a last round that is at most half full are cut along their rows
    // instead, each piece a tile of its own that streams the whole weight tile (out of the L2, which
    // its sister pieces fill at the same time).  The outputs are the same bits: a row's sums do not
    // depend on which rows share its tile.  (Only blocks of the last two rounds come here: the
    // integer divisions below cost a tile of the rounds before them half a percent of its time.)
    const int cus_x = max(1, (p.n_cu > 0 ? p.n_cu : 256) / 8);
    const int full_x = per_xcd / cus_x * cus_x;
    const int tail_x = per_xcd - full_x;
    if (slot >= full_x) {
      if (tail_x > 0 && 2 * tail_x <= cus_x) m_pieces = min(cus_x / tail_x, MSPLIT_MAX_PIECES);
      const int j = slot - full_x;
      const int t_local = j / m_pieces;
      if (t_local >= tail_x) return false;
      vid = xcd * per_xcd + full_x + t_local;
      m_piece = j - t_local * m_pieces;
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
  tc.sharers = m_tiles;
  if (p.mode == TILES_EVEN) {
    // The segment's 16-row sub-tiles are dealt in pairs: a tile's sub-tiles go to four wave rows,
    // and wave rows 0, 2 and 1, 3 share their SIMDs, so a tile with an odd number of sub-tiles is
    // as slow as one with the next even number.  67 sub-tiles become 17, 16, 16, 18 (9 + 8 + 8 + 9
    // per SIMD pair), not 16, 17, 17, 17 (8 + 9 + 9 + 9).  An odd one out goes to the first tile,
    // which has the fewest pairs (so no tile exceeds 20 sub-tiles).
    const int sub = (seg_end - seg_begin + 15) / 16;
    const int pairs = sub >> 1, odd = sub & 1;
    const int b0 = m_idx == 0 ? 0 : 2 * (m_idx * pairs / m_tiles) + odd;
    const int b1 = 2 * ((m_idx + 1) * pairs / m_tiles) + odd;
    int s0 = b0, s1 = b1;
    if (m_pieces > 1) {
      const int n_sub = b1 - b0;
      const int pieces = min(m_pieces, max(1, n_sub / 4));    // a piece keeps 64 rows or more
      if (m_piece >= pieces) return false;
      tc.sharers = m_tiles + pieces - 1;
      s0 = b0 + m_piece * n_sub / pieces;
      s1 = b0 + (m_piece + 1) * n_sub / pieces;
    }
    tc.m_begin = seg_begin + s0 * 16;
    tc.m_end = min(seg_end, seg_begin + s1 * 16);
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
// bf16 MFMA kernels
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

// Store of a wave's outputs.  Accumulator (v, lane) holds out[row = m-sub-tile + lane%16]
// [col = n-sub-tile + 4*(lane/16) + v]: 8-byte pieces scattered over 16 rows.  Each wave turns its
// 16-row sub-tile around in a private LDS region (row pitch = row bytes + 32: the 32-byte runs
// that the four lanes of a row write land in 8 banks, and 8 consecutive rows cover all 64) and
// stores whole rows, 16 bytes per lane, so the L2 sees full-line writes.  Starts with a barrier:
// every wave must be done with whatever else the block kept in that LDS.
// MI, NI: accumulator sub-tiles of a wave; WN: waves along the weight rows; the wave's first
// mi_valid sub-tiles are stored, the first one starting at row wave_row0 of the tile.
template <bool GATED, int MI, int NI, int WN, int NW>
__device__ __forceinline__ void ffn_store_tile(const f32x4_t (&acc)[NI][MI], const TileCoord& tc,
                                               const GemmArgs& p, unsigned char* lds, int wave, int lane,
                                               int mi_valid, int wave_row0) {
  constexpr int NIH = GATED ? NI / 2 : NI;
  constexpr int BN_OUT = GATED ? 128 : 256;
  const int wn = wave % WN;
  const int l16 = lane & 15;
  const int N = p.N;
  const int n0 = tc.n_tile * BN_OUT;
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  constexpr int CW = NIH * 16;                    // output columns of this wave
  constexpr int PITCH = CW * 2 + 32;              // bytes
  constexpr int LPR = CW * 2 / 16;                // lanes that store one row
  constexpr int RPI = 64 / LPR;                   // rows per store instruction
  static_assert(16 % RPI == 0 && NW * 16 * PITCH <= 40 * 1024, "staging fits the smallest LDS buffer it is given");
  unsigned char* region = lds + wave * (16 * PITCH);
  bf16_t* out = static_cast<bf16_t*>(p.out);
  const int col0 = n0 + wn * CW;                  // first output column of this wave
  const int32_t* out_map = GATED ? nullptr : p.out_map;   // uniform
  auto mapped_row = [&](int gr) { return min(max(out_map[min(gr, tc.m_end - 1)], 0), p.out_rows - 1); };
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    if (mi < mi_valid) {                          // wave-uniform
      const int row_base = tc.m_begin + wave_row0 + mi * 16;
      // this lane's accumulators belong to row lane%16 of the sub-tile
      const float scale = out_map ? p.out_scale[mapped_row(row_base + l16)] : 1.f;
#pragma unroll
      for (int ni = 0; ni < NIH; ++ni) {
        float o[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (GATED)
            o[u] = silu_mul(acc[ni][mi][u], acc[GATED ? ni + NIH : ni][mi][u]);
          else
            o[u] = out_map ? acc[ni][mi][u] * scale : acc[ni][mi][u];
        }
        const int c = ni * 16 + 4 * (lane >> 4);
        *reinterpret_cast<uint2*>(region + l16 * PITCH + c * 2) =
            make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // same wave: writes land before the reads
#pragma unroll
      for (int it = 0; it < 16 / RPI; ++it) {
        const int r = it * RPI + lane / LPR;
        const int c = (lane % LPR) * 8;           // first column of this lane's 16 bytes
        const uint4 v = *reinterpret_cast<const uint4*>(region + r * PITCH + c * 2);
        const int gr = row_base + r;
        if (gr < tc.m_end && col0 + c < N) {
          const int dst = out_map ? mapped_row(gr) : gr;
          *reinterpret_cast<uint4*>(out + static_cast<int64_t>(dst) * N + col0 + c) = v;
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the region is reused
    }
  }
}

// A part of a split tile leaves its accumulators in its workspace slot, thread-major so that a
// thread's 16 bytes sit next to its neighbours'; the summing launch reads them back the same way.
template <int MI, int NI, int NT>
__device__ __forceinline__ void ffn_store_part(const f32x4_t (&acc)[NI][MI], const TileCoord& tc,
                                               const GemmArgs& p) {
  static_assert(NI * MI * NT * 4 <= SPLIT_SLOT_FLOATS, "slot size");
  float* mine = p.split_ws + static_cast<int64_t>(tc.pslot) * SPLIT_SLOT_FLOATS;
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
      *reinterpret_cast<f32x4_t*>(mine + ((ni * MI + mi) * NT + static_cast<int>(threadIdx.x)) * 4) =
          acc[ni][mi];
}
template <int MI, int NI, int NT>
__device__ __forceinline__ void ffn_sum_parts(f32x4_t (&acc)[NI][MI], const TileCoord& tc,
                                              const GemmArgs& p) {
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) acc[ni][mi] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const float* first = p.split_ws + static_cast<int64_t>(tc.pslot) * SPLIT_SLOT_FLOATS;
  for (int q = 0; q < tc.nparts; ++q) {           // in part order: the sum does not depend on scheduling
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
}

// --------------------------------------------------------------------------------------------
// Ring tiles: BM x 256 block tile, WM x WN waves, NSTAGE LDS stages of 64 K-elements with
// NSTAGE - 1 stages of loads in flight (little arithmetic per weight byte: paced by memory
// latency).  SPLIT: tiles of the last, partial round may be cut along K (see decode_tile): a part
// leaves its fp32 accumulators in the workspace instead of storing the tile, and
// ffn_ring_sum_parts_kernel, the next launch on the stream, adds the parts and stores the tile.
// --------------------------------------------------------------------------------------------
constexpr int ffn_ring_lds_bytes(int bm, int nstage) { return nstage * (bm + BROWS) * ROWB; }

template <int BM, bool GATED, int WM, int WN, int NSTAGE, bool SPLIT>
__device__ __forceinline__ void ffn_ring_tile(const GemmArgs& p, const TileCoord& tc, unsigned char* lds) {
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
  static_assert(NSTAGE > 2, "a ring keeps at least two stages of loads in flight");

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
  // The weight rows of an expert that is this one tile are read once by the whole chip: requested
  // with the non-temporal hint they do not displace what other blocks still share in the L2.
  // (Measured with the hint on every ring tile: decode-shaped layer 0.79 -> 0.72 ms, Mixtral shape
  // at 16 tokens 0.51 -> 0.48 ms, its weights then stream at 5.9 TB/s; with two tiles per expert,
  // Mixtral shape at 256 and 448 tokens, 1 to 5 % slower, hence the condition.  Only in launches
  // of ring tiles alone: for the small experts of a skewed batch, inside a launch of even tiles,
  // the hint gained nothing measurable.)
  const bool wgt_nt = p.mode == TILES_FIXED && tc.sharers <= 1;   // block-uniform
  // instruction i of stage kt into LDS stage `stage` (1 KiB per wave instruction)
  auto issue_load = [&](int i, int kt, int stage) {
    const __amdgpu_buffer_rsrc_t rs = (i < NLA) ? rs_a : (!GATED || i < NLA + NLB) ? rs_b0 : rs_b1;
    if (i < NLA || !wgt_nt)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rs, (__attribute__((address_space(3))) void*)(lds + stage * STAGE + (i * NW + wave) * 1024), 16,
          static_cast<int>(soff[i]), kt * ROWB, 0, 0);
    else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rs, (__attribute__((address_space(3))) void*)(lds + stage * STAGE + (i * NW + wave) * 1024), 16,
          static_cast<int>(soff[i]), kt * ROWB, 0, 2);             // aux bit 1: nt
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
    for (int mi = 0; mi < MI; ++mi) acc[ni][mi] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](int stage) {                 // compiler-scheduled
    const unsigned char* s = lds + stage * STAGE;
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      bf16x8_t xf[MI], wf[NI];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        if (mi < mi_valid)
          xf[mi] = *reinterpret_cast<const bf16x8_t*>(s + x_base + mi * 16 * ROWB + koff[kk]);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        wf[ni] = *reinterpret_cast<const bf16x8_t*>(s + w_base + w_sub(ni) * ROWB + koff[kk]);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          if (mi < mi_valid)
            acc[ni][mi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[ni], xf[mi], acc[ni][mi], 0, 0, 0);
    }
  };

  // ---- ring pipeline: the loads of stage kt+DIST are issued at the start of stage kt -----------
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
    if (mi_valid > 0) compute(kt % NSTAGE);
  }

  if (SPLIT && tc.nparts > 1) {
    ffn_store_part<MI, NI, NW * MOE_WAVE>(acc, tc, p);
    return;
  }
  ffn_store_tile<GATED, MI, NI, WN, NW>(acc, tc, p, lds, wave, lane, mi_valid, wm * (BM / WM));
}

template <int BM, bool GATED, int WM, int WN, int NSTAGE, bool SPLIT = false>
__global__ __launch_bounds__(WM * WN * 64) void ffn_ring_kernel(GemmArgs p) {
  extern __shared__ __align__(1024) unsigned char lds[];
  TileCoord tc;
  if (!decode_tile<SPLIT>(p, tc)) return;
  ffn_ring_tile<BM, GATED, WM, WN, NSTAGE, SPLIT>(p, tc, lds);
}

// Adds the parts of a split ring tile and stores it.
template <int BM, bool GATED, int WM, int WN>
__device__ __forceinline__ void ffn_ring_sum_tile(const GemmArgs& p, const TileCoord& tc, unsigned char* lds) {
  constexpr int NW = WM * WN;
  constexpr int MI = BM / WM / 16;
  constexpr int NI = BROWS / WN / 16;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);
  const int wm = wave / WN;
  const int rows_valid = min(tc.m_end - tc.m_begin, BM);
  const int mi_valid = max(0, min(MI, (rows_valid - wm * (BM / WM) + 15) / 16));
  f32x4_t acc[NI][MI];
  ffn_sum_parts<MI, NI, NW * MOE_WAVE>(acc, tc, p);
  ffn_store_tile<GATED, MI, NI, WN, NW>(acc, tc, p, lds, wave, lane, mi_valid, wm * (BM / WM));
}

// The launch after a ring GEMM whose tiles may have been split: block (xcd, t) adds the parts of
// split tile t of the XCD's last round and stores the tile.  Finds nothing to do when no tile was split.
template <int BM, bool GATED, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void ffn_ring_sum_parts_kernel(GemmArgs p) {
  extern __shared__ __align__(1024) unsigned char lds[];
  TileCoord tc;
  if (!decode_tile<true>(p, tc)) return;
  ffn_ring_sum_tile<BM, GATED, WM, WN>(p, tc, lds);
}

// --------------------------------------------------------------------------------------------
// Even tiles: an expert's c rows are cut into ceil(c / 320) tiles of (nearly) equal height, a
// multiple of 16 rows each, so no segment leaves a small remainder that would have to stream the
// expert's weights once more for a handful of rows: the Mixtral-shaped batch (about 1024 rows
// per expert) runs as four tiles of 256 or 272 rows per expert, whatever the counts are.
// Block tile: up to 320 activation rows x 256 weight rows, K step 64, two LDS stages of 72 KiB
// (the two activation buffers first, then the two weight buffers, so that a fragment read
// selects the buffer with its 16-bit offset field).
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
// reads issued after it.  Inline asm pins the order; the compiler does not see these LDS reads, so
// it inserts no waits of its own.  A stage's barrier sits between the two parts of its second
// k-step: by then every fragment of the stage is in registers, the stage's buffer takes the loads
// of the stage after next, and the other buffer (landed: vmcnt(0)) is read from.
//
// Who issues the loads (ALTERNATE).  A wave that issues a burst of direct-to-LDS loads is held at every one of
// them until the address unit takes it, and issues no MFMA meanwhile.  If all eight waves load
// their eighth of a stage right after the barrier, both waves of every SIMD are held at once and
// the matrix pipe idles.  With ALTERNATE the waves form two sets of four, {0-3} and {4-7}
// (waves w and w + 4 share a SIMD), that take turns: set (stage & 1) issues the whole stage while
// the other set goes straight on with its MFMAs, so every SIMD always has a wave that multiplies.
// Measured on the Mixtral shape: up-projection 6 % faster.  Calls whose experts hold a single tile
// each (nothing shares a weight tile through the L2, the call waits on HBM) are faster with every
// wave loading; the host chooses by the mean rows per expert.
constexpr int EVEN_BM = 320;
constexpr int EVEN_ACT = EVEN_BM * ROWB;                     // one activation buffer
constexpr int EVEN_WGT = BROWS * ROWB;                       // one weight buffer
// Tiles of at most RING_ROWS rows (a small expert of a skewed batch, beside experts that hold several
// full tiles) run the ring pipeline inside the same launch: they have little arithmetic per weight
// byte and are paced by memory latency, which the ring's three stages in flight hide best.
constexpr int RING_ROWS = 64;
constexpr int EVEN_LDS = ffn_ring_lds_bytes(RING_ROWS, 4) > 2 * (EVEN_ACT + EVEN_WGT)
                             ? ffn_ring_lds_bytes(RING_ROWS, 4) : 2 * (EVEN_ACT + EVEN_WGT);

// How the tile's sub-tiles are dealt to wave row wm (of 4): count and first row.
__device__ __forceinline__ void even_wave_rows(int rows_valid, int wm, int& miv, int& row0) {
  const int nsub = (rows_valid + 15) >> 4;
  const int q = nsub >> 2, r = nsub & 3;
  miv = q + (wm < r ? 1 : 0);
  row0 = 16 * (wm * q + min(wm, r));
}

// MI: 16-row sub-tiles a wave can hold.  MI = 5: tiles of up to 320 rows, two activation and two weight
// buffers (144 KiB).  MI = 4: tiles of up to 256 rows; the 16 KiB the activation buffers give back
// make a third weight buffer (160 KiB), and the weight rows are requested a stage earlier than the
// activation rows: they are the operand that misses the L2 (an XCD's tiles share activation
// rows far more often than weight rows), so their requests take longest to return.
template <bool GATED, bool SPLIT, bool ALTERNATE, bool WNT, int MI>
__device__ __forceinline__ void ffn_even_tile(const GemmArgs& p, const TileCoord& tc, unsigned char* lds) {
  constexpr int NW = 8, WN = 2;
  constexpr int BM = MI * 64, NI = 8;
  constexpr int NIH = GATED ? NI / 2 : NI;
  constexpr int NLA = BM / 8 / 4;                 // up to 10 activation row groups per loading wave and stage
  constexpr int NLW = BROWS / 8 / 4;              // up to 8 weight row groups
  constexpr int BN_OUT = GATED ? 128 : 256;
  constexpr int ACT = BM * ROWB;                  // one activation buffer
  constexpr int NWB = MI == 4 ? 3 : 2;            // weight buffers
  constexpr int W_BASE = 2 * ACT;                 // LDS offset of the weight buffers
  static_assert(MI == 4 || MI == 5, "wave tile");
  static_assert(W_BASE + NWB * EVEN_WGT <= EVEN_LDS, "LDS budget");

  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);
  const int wm = wave / WN, wn = wave % WN;
  constexpr bool alternate = ALTERNATE;
  constexpr int ns = alternate ? 4 : 8;           // waves that share a stage's loads
  const int lw = alternate ? (wave & 3) : wave;   // this wave's place among them
  const int lset = alternate ? (wave >> 2) : 0;   // ... and the stages it loads: stage & 1 == lset
  const int K = p.K, N = p.N;
  int KT = K / BK, k_first = 0;                   // this block's K stages
  if (SPLIT && tc.nparts > 1) {
    const int kt_first = tc.part * KT / tc.nparts;
    KT = (tc.part + 1) * KT / tc.nparts - kt_first;
    k_first = kt_first * BK;
  }
  const int n0 = tc.n_tile * BN_OUT;
  const int rows_valid = min(tc.m_end - tc.m_begin, BM);
  int miv, row0;
  even_wave_rows(rows_valid, wm, miv, row0);

  // ---- global -> LDS.  A wave instruction fills an 8-row group of 1 KiB.  A loading wave takes
  //      activation groups i * ns + lw (only those that hold a valid row) and weight groups
  //      i * ns + lw (only those inside the weight matrix: N - n0 is a multiple of 64, so a group
  //      is inside or outside as a whole).  The rows of a wave's weight groups are multiples of
  //      32 rows apart (same swizzle): one per-lane offset, the rest is a scalar.  Activation rows
  //      past the end of the segment re-read its last row.
  const bool gathered = p.src_assign != nullptr;
  const bf16_t* A = static_cast<const bf16_t*>(p.a) + k_first;
  const bf16_t* B0 = static_cast<const bf16_t*>(p.b0) + static_cast<int64_t>(tc.e) * N * K + k_first;
  const bf16_t* B1 =
      GATED ? static_cast<const bf16_t*>(p.b1) + static_cast<int64_t>(tc.e) * N * K + k_first : B0;
  // buffer resources (raw, stride 0) based at the first row of each operand of this tile: the
  // per-lane 32-bit offset and a scalar offset replace 64-bit per-lane address arithmetic
  // (gathered rows: the offset is taken from the start of `a`; the host checks that it fits 31 bits)
  const __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(gathered ? A : A + static_cast<int64_t>(tc.m_begin) * K), 0, 0x7FFFFFFF, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_b0 = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(B0 + static_cast<int64_t>(n0) * K), 0, 0x7FFFFFFF, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_b1 = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(B1 + static_cast<int64_t>(n0) * K), 0, 0x7FFFFFFF, 0x00020000);
  const int n_act = min(BM / 8 / ns, max(0, (((rows_valid + 7) >> 3) - lw + ns - 1) / ns));
  const int w_rows = min(GATED ? 128 : 256, N - n0);          // weight rows of this tile per matrix
  uint32_t soff_a[NLA], soff_w;
  {
    const int br = lw * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ swz(br);
    soff_w = static_cast<uint32_t>(br) * static_cast<uint32_t>(K) * 2u + static_cast<uint32_t>(chunk) * 16u;
  }
  // The activation rows of stage kt go to activation buffer kt % 2 and are requested two stages
  // ahead, the weight rows to weight buffer kt % NWB, NWB stages ahead.  With ALTERNATE the requests
  // made after the barrier of stage j (activations of j + 2, weights of j + NWB) all come from
  // wave set j & 1.
  auto issue_act = [&](int kt) {
    if (alternate && lset != (kt & 1)) return;
#pragma unroll
    for (int i = 0; i < NLA; ++i)
      if (i < n_act)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rs_a, (__attribute__((address_space(3))) void*)(lds + (kt & 1) * ACT + (i * ns + lw) * 1024),
            16, static_cast<int>(soff_a[i]), kt * ROWB, 0, 0);
  };
  // Every wave makes the same number of weight requests per stage (W_LOADS), so that a wait can
  // leave exactly one stage's weight requests outstanding: a group outside the weight matrix (the
  // last n-tile of a matrix whose row count is not a multiple of the tile) re-reads the tile's
  // first rows; its products are never stored.
  constexpr int W_LOADS = 32 / ns;
  // WNT: weight rows that at most two tiles read (an expert of one or two tiles) are requested with
  // the non-temporal hint: nothing will ask for them again, and they stop displacing the activation
  // rows, which the other n-tiles of the round and the later rounds re-read, from the L2.  Weight
  // rows shared by more tiles keep the default policy (measured with the hint on every tile: the
  // Mixtral shape, four tiles per expert, up-projection 4 % slower; llama4 and phi shapes, one and
  // two tiles per expert, both GEMMs 4 to 7 % faster).  The branch per stage costs a launch whose
  // tiles all keep the default policy about 1 %, so the host builds it in (WNT) only for calls with
  // few rows per expert.
  const bool wgt_nt = WNT && tc.sharers <= WGT_NT_MAX_SHARERS;       // block-uniform
  auto issue_wgt_with = [&](int kt, int wb, auto aux_c) {
    constexpr int AUX = decltype(aux_c)::value;
#pragma unroll
    for (int i = 0; i < W_LOADS; ++i) {
      // group i * ns + lw of the 32 weight row groups; gated: groups 0-15 are W1 rows 0-127 of the
      // tile, groups 16-31 the same rows of W3
      const int g0 = i * ns * 8;                  // first row of the step (lw = 0)
      int jr = GATED ? (g0 & 127) : g0;           // ... inside its matrix
      if (jr >= w_rows) jr = 0;
      if (!GATED || g0 < 128)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rs_b0, (__attribute__((address_space(3))) void*)(lds + W_BASE + wb * EVEN_WGT + (i * ns + lw) * 1024),
            16, static_cast<int>(soff_w), kt * ROWB + jr * K * 2, 0, AUX);
      else
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rs_b1, (__attribute__((address_space(3))) void*)(lds + W_BASE + wb * EVEN_WGT + (i * ns + lw) * 1024),
            16, static_cast<int>(soff_w), kt * ROWB + jr * K * 2, 0, AUX);
    }
  };
  auto issue_wgt = [&](int kt, int wb) {
    if (alternate && lset != ((kt + NWB) & 1)) return;
    if (wgt_nt)
      issue_wgt_with(kt, wb, std::integral_constant<int, 2>{});    // aux bit 1: nt
    else
      issue_wgt_with(kt, wb, std::integral_constant<int, 0>{});
  };

  // ---- LDS addresses of this lane's fragments per k-step.  A lane holds, for row lane%16 of a
  //      16-row sub-tile, the 8 K-elements of one 16-byte chunk of the k-step's four.  Which chunk
  //      goes to which lane group is free as long as both operands agree (it only permutes the K
  //      order inside the MFMA).  The LDS serves a 16-byte read in passes of lanes {0-7, 32-39},
  //      {8-15, 40-47}, ...: lane groups 0 and 2 therefore take chunks that differ in bit 0 (0 and
  //      1; groups 1 and 3 take 2 and 3), which with the row swizzle makes every pass touch each
  //      bank once.
  const int l16 = lane & 15;
  const int f = swz(l16);                         // sub-tile bases are multiples of 16 rows
  const int kgrp = ((lane >> 4) & 1) * 2 + (lane >> 5);
  int xa[2], wa[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    const int ko = ((kk * 4 + kgrp) ^ f) << 4;
    xa[kk] = (row0 + l16) * ROWB + ko;
    wa[kk] = W_BASE + (wn * (NIH * 16) + l16) * ROWB + ko;
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
#define MOE_X_OFF(buf, mi) ((buf) * ACT + (mi) * 16 * ROWB)
#define MOE_W_OFF(ni) ((GATED ? ((ni) / NIH) * 128 + ((ni) % NIH) * 16 : (ni) * 16) * ROWB)
  static_assert(MOE_W_OFF(NI - 1) < 65536 && MOE_X_OFF(1, MI - 1) < 65536, "ds_read offset field");

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
    // kk, buf: the k-step and activation buffer the next fragments come from; wv: this lane's
    // address in the weight buffer they come from
    auto part2 = [&](auto kk_c, auto buf_c, int wv) {
      constexpr int KK = decltype(kk_c)::value, BUF = decltype(buf_c)::value;
      if constexpr (MIV > 0) {
#pragma unroll
        for (int mi = 0; mi < P1; ++mi) MOE_RD(x[mi], xa[KK], MOE_X_OFF(BUF, mi));
        if constexpr (P2 > 0) asm volatile("s_waitcnt lgkmcnt(%0)" ::"i"(P1) : "memory");
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
          for (int mi = P1; mi < MIV; ++mi) MOE_MFMA(acc[ni][mi], w[ni], x[mi]);
          MOE_RD(w[ni], wv, MOE_W_OFF(ni));
        }
#pragma unroll
        for (int mi = P1; mi < MIV; ++mi) MOE_RD(x[mi], xa[KK], MOE_X_OFF(BUF, mi));
      }
    };
    using K0 = std::integral_constant<int, 0>;
    using K1 = std::integral_constant<int, 1>;
    int wb = 0;                                   // weight buffer of the current stage (uniform)
    auto stage = [&](int kt, auto par_c) {
      constexpr int PAR = decltype(par_c)::value;
      const int wb_next = wb + 1 == NWB ? 0 : wb + 1;
      part1();
      part2(K1{}, std::integral_constant<int, PAR>{}, wa[1] + wb * EVEN_WGT);
      part1();
      // Stage kt + 1 must have landed.  Requests return in order, and the last ones this wave made
      // (after the barrier of stage kt - 1, if it was its turn) were the activation rows of kt + 1,
      // then, with three weight buffers, the weight rows of kt + 2: those may stay in flight.
      if (NWB == 3 && kt >= 1 && kt + 2 < KT && (!alternate || lset == ((kt - 1) & 1)))
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"i"(W_LOADS) : "memory");
      else
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      if (kt + 2 < KT) issue_act(kt + 2);
      if (kt + NWB < KT) issue_wgt(kt + NWB, wb);
      // (after the tile's last stage these reads return whatever the buffer holds and go unused)
      part2(K0{}, std::integral_constant<int, PAR ^ 1>{}, wa[0] + wb_next * EVEN_WGT);
      wb = wb_next;
    };
    if constexpr (MIV > 0) {
#pragma unroll
      for (int mi = 0; mi < P1; ++mi) MOE_RD(x[mi], xa[0], MOE_X_OFF(0, mi));
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) MOE_RD(w[ni], wa[0], MOE_W_OFF(ni));
#pragma unroll
      for (int mi = P1; mi < MIV; ++mi) MOE_RD(x[mi], xa[0], MOE_X_OFF(0, mi));
    }
    int kt = 0;
    for (; kt + 2 <= KT; kt += 2) {
      stage(kt, K0{});
      stage(kt + 1, K1{});
    }
    if (kt < KT) stage(kt, K0{});
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // the unused reads of the last stage
    // the compiler's hazard handling does not see asm MFMAs: let the last results retire
    // before ordinary VALU code reads the accumulators
    asm volatile("s_nop 15\n s_nop 15\n s_nop 15\n s_nop 15" ::: "memory");
  };

  // prologue: stages 0 and 1 requested, the weight rows first: their addresses need no memory, while
  // the activation rows of a call that reads x through the map wait for the map entries, a trip to
  // memory that now overlaps the weights'.  Everything this wave requested has landed before the
  // first barrier (a count that spared stage 1 would depend on how many groups the wave skipped).
#pragma unroll
  for (int s = 0; s < NWB; ++s)
    if (s < KT) issue_wgt(s, s);
#pragma unroll
  for (int i = 0; i < NLA; ++i) {
    const int row = (i * ns + lw) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ swz(row);      // the chunk of the row this lane fetches
    int r = min(row, rows_valid - 1);
    if (gathered) r = a_row_of(p, tc.m_begin + r);
    soff_a[i] = static_cast<uint32_t>(r) * static_cast<uint32_t>(K) * 2u + static_cast<uint32_t>(chunk) * 16u;
  }
  issue_act(0);
  if (KT > 1) issue_act(1);
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  switch (miv) {                                  // wave-uniform
    case 0: k_loop(std::integral_constant<int, 0>{}); break;
    case 1: k_loop(std::integral_constant<int, 1>{}); break;
    case 2: k_loop(std::integral_constant<int, 2>{}); break;
    case 3: k_loop(std::integral_constant<int, 3>{}); break;
    case 4: k_loop(std::integral_constant<int, 4>{}); break;
    default:
      if constexpr (MI >= 5) k_loop(std::integral_constant<int, 5>{});
      break;
  }
#undef MOE_RD
#undef MOE_MFMA
#undef MOE_X_OFF
#undef MOE_W_OFF

  if (SPLIT && tc.nparts > 1) {
    ffn_store_part<MI, NI, NW * MOE_WAVE>(acc, tc, p);
    return;
  }
  // the store turns the sub-tiles around in activation buffer 0 (every wave has read its last
  // fragments before the store's barrier)
  ffn_store_tile<GATED, MI, NI, WN, NW>(acc, tc, p, lds, wave, lane, miv, row0);
}

// Tiles of at most this many rows of the down-projection take the form with three weight buffers.
// (Measured on uniform batches at the Mixtral shape, 768 and 1024 rows per expert: the
// down-projection, whose reduction is 14336 long, 11 % and 4.5 % faster; the up-projection, 4096
// long, 1 % slower, so it keeps two weight buffers for every tile.)
constexpr int EVEN_ROWS_3WB = 256;

template <bool GATED, bool SPLIT, bool ALTERNATE, bool WNT>
__global__ __launch_bounds__(512) void ffn_even_kernel(GemmArgs p) {
  extern __shared__ __align__(1024) unsigned char lds[];
  TileCoord tc;
  if (!decode_tile<SPLIT>(p, tc)) return;
  const int rows = tc.m_end - tc.m_begin;         // block-uniform
  if (rows <= RING_ROWS)
    ffn_ring_tile<RING_ROWS, GATED, 2, 4, 4, SPLIT>(p, tc, lds);
  else if (!GATED && rows <= EVEN_ROWS_3WB)
    ffn_even_tile<GATED, SPLIT, ALTERNATE, WNT, 4>(p, tc, lds);
  else
    ffn_even_tile<GATED, SPLIT, ALTERNATE, WNT, 5>(p, tc, lds);
}

// The launch after ffn_even_kernel<.., SPLIT>: adds the parts of every split tile and stores it.
template <bool GATED, int MI>
__device__ __forceinline__ void ffn_even_sum_tile(const GemmArgs& p, const TileCoord& tc, unsigned char* lds) {
  constexpr int NW = 8, WN = 2, NI = 8;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);
  int miv, row0;
  even_wave_rows(min(tc.m_end - tc.m_begin, MI * 64), wave / WN, miv, row0);
  f32x4_t acc[NI][MI];
  ffn_sum_parts<MI, NI, NW * MOE_WAVE>(acc, tc, p);
  ffn_store_tile<GATED, MI, NI, WN, NW>(acc, tc, p, lds, wave, lane, miv, row0);
}
template <bool GATED>
__global__ __launch_bounds__(512) void ffn_even_sum_parts_kernel(GemmArgs p) {
  extern __shared__ __align__(1024) unsigned char lds[];
  TileCoord tc;
  if (!decode_tile<true>(p, tc)) return;
  const int rows = tc.m_end - tc.m_begin;
  if (rows <= RING_ROWS)                          // its parts came from the ring pipeline
    ffn_ring_sum_tile<RING_ROWS, GATED, 2, 4>(p, tc, lds);
  else if (!GATED && rows <= EVEN_ROWS_3WB)
    ffn_even_sum_tile<GATED, 4>(p, tc, lds);
  else
    ffn_even_sum_tile<GATED, 5>(p, tc, lds);
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
  const int32_t* out_map = GATED ? nullptr : p.out_map;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int gr = tc.m_begin + ty * 4 + i;
    if (gr >= tc.m_end) continue;
    float scale = 1.f;
    if (out_map) {
      gr = min(max(out_map[gr], 0), p.out_rows - 1);
      scale = p.out_scale[gr];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = n0 + tx * 4 + j;
      if (c < N) {
        float v;
        if (GATED) {
          const float g = acc[0][i][j];
          v = g / (1.0f + expf(-g)) * acc[GATED ? 1 : 0][i][j];
        } else {
          v = out_map ? acc[0][i][j] * scale : acc[0][i][j];
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

// Upper bound on the number of m-tiles that needs no knowledge of the counts: an expert with c rows
// has ceil(c / bm) <= c / bm + 1 tiles, and at most min(E, A) experts have any.
static int64_t max_m_tiles(int64_t A, int E, int bm) { return A / bm + (E < A ? E : A); }

// `split`: the launch may use the workspace for split tiles if the caller brought one.  Only
// GEMMs with a long reduction do: a part must be worth the exchange (one 256 to 320 KiB store per
// part, the summing launch), and a tile of fewer than 96 stages is too short for that (measured:
// the up-projections of the four model shapes gain nothing, their down-projections up to 27 %).
constexpr int SPLIT_MIN_K = 96 * BK_ELEMS;

// One grouped GEMM.  main_kernel: void (*)(GemmArgs); the grid is an upper bound of the tile count
// (surplus blocks exit at once), plus a round of blocks for the parts when tiles may be split; the
// summing kernel (one block per possible split tile) follows on the same stream.
static int launch_grouped_gemm(GemmArgs a, int mode, int bm, int64_t A, int threads, int lds_bytes,
                               void (*main_kernel)(GemmArgs), LdsOnce& once_main,
                               void (*sum_kernel)(GemmArgs), LdsOnce& once_sum, hipStream_t st) {
  if (ensure_dynamic_lds(once_main, reinterpret_cast<const void*>(main_kernel), lds_bytes) != MOE_OK)
    return MOE_ERR_HIP;
  a.mode = mode;
  a.bm = bm;
  a.split_phase = 0;
  if (!sum_kernel) a.split_ws = nullptr;
  int64_t grid = max_m_tiles(A, a.E, bm) * a.n_tiles;
  if (grid == 0) return MOE_OK;
  grid = (grid + 7) / 8 * 8;
  const int cu8 = (a.n_cu > 0 ? a.n_cu : 256) / 8 * 8;
  if (sum_kernel || a.m_split) grid += cu8;
  if (grid > 0x7FFFFFFF) return MOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(main_kernel, dim3(static_cast<unsigned>(grid)), dim3(threads), lds_bytes, st, a);
  int rc = launch_status();
  if (sum_kernel && rc == MOE_OK) {
    if (ensure_dynamic_lds(once_sum, reinterpret_cast<const void*>(sum_kernel), lds_bytes) != MOE_OK)
      return MOE_ERR_HIP;
    a.split_phase = 1;
    hipLaunchKernelGGL(sum_kernel, dim3(static_cast<unsigned>(cu8)), dim3(threads), lds_bytes, st, a);
    rc = launch_status();
  }
  return rc;
}

template <bool GATED, bool ALTERNATE, bool WNT>
static int launch_even(const GemmArgs& a, int64_t A, bool row_split, hipStream_t st) {
  static LdsOnce once[2], once_sum;
  if (a.split_ws && a.K >= SPLIT_MIN_K)
    return launch_grouped_gemm(a, TILES_EVEN, EVEN_BM, A, 512, EVEN_LDS, ffn_even_kernel<GATED, true, ALTERNATE, WNT>,
                               once[1], ffn_even_sum_parts_kernel<GATED>, once_sum, st);
  GemmArgs b = a;
  b.m_split = row_split ? 1 : 0;
  return launch_grouped_gemm(b, TILES_EVEN, EVEN_BM, A, 512, EVEN_LDS, ffn_even_kernel<GATED, false, ALTERNATE, WNT>,
                             once[0], nullptr, once_sum, st);
}

template <bool GATED>
static int launch_ring(const GemmArgs& a, int64_t A, hipStream_t st) {
  constexpr int BM = 64, WM = 2, WN = 4, NSTAGE = 4;
  constexpr int lds_bytes = ffn_ring_lds_bytes(BM, NSTAGE);
  static LdsOnce once[2], once_sum;
  if (a.split_ws && a.K >= SPLIT_MIN_K)
    return launch_grouped_gemm(a, TILES_FIXED, BM, A, WM * WN * 64, lds_bytes,
                               ffn_ring_kernel<BM, GATED, WM, WN, NSTAGE, true>, once[1],
                               ffn_ring_sum_parts_kernel<BM, GATED, WM, WN>, once_sum, st);
  return launch_grouped_gemm(a, TILES_FIXED, BM, A, WM * WN * 64, lds_bytes,
                             ffn_ring_kernel<BM, GATED, WM, WN, NSTAGE, false>, once[0], nullptr, once_sum, st);
}

template <typename T, bool GATED>
static int launch_generic(GemmArgs a, int64_t A, hipStream_t st) {
  a.mode = TILES_FIXED;
  a.bm = 64;
  int64_t grid = max_m_tiles(A, a.E, 64) * a.n_tiles;
  grid = (grid + 7) / 8 * 8;
  if (grid > 0x7FFFFFFF) return MOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((ffn_generic_kernel<T, GATED>), dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                     st, a);
  return launch_status();
}

// Mean rows per expert from which the even tiles take over from the ring tiles, and from which the
// waves of a SIMD take turns loading (two or more tiles of an expert then share each weight tile
// through the L2; measured on five layer shapes: 4 to 6 % faster from 512 rows per expert on, 2 %
// slower at 256, where each expert is a single tile).
constexpr int EVEN_MIN_ROWS = 128;
constexpr int ALTERNATE_MIN_ROWS = 384;
// Mean rows per expert below which the kernels are built with the per-tile choice of the
// non-temporal hint for weight rows (experts of at most two tiles are then the rule).
constexpr int WGT_NT_ROWS = 2 * EVEN_BM;

// Both GEMMs (or one of them) on the MFMA path: one launch each on the caller's stream.
static int mfma_ffn(GemmArgs g1, GemmArgs g2, bool up, bool down, int64_t A, bool row_split,
                    hipStream_t st) {
  int rc = MOE_OK;
  if (A / g1.E < EVEN_MIN_ROWS) {
    // Few rows per expert (decode, small prefill batches): the call is bound by streaming each
    // expert's weights once, which the latency-hiding ring of the 64-row tiles does best.
    // (Measured, whole layer, ring tiles against even tiles for every expert: Mixtral shape 64 / 96
    // rows per expert 0.60 / 0.63 ms against 0.70 / 0.74; skewed 64-expert layer at 256 ... 1280
    // tokens, where a hot expert holds ten times the mean, 0.22 ... 0.39 ms against 0.27 ... 0.41;
    // only the fine-grained layer at 96 rows per expert is faster with even tiles, 0.28 against 0.33 ms.)
    if (up && (rc = launch_ring<true>(g1, A, st)) != MOE_OK) return rc;
    if (down) rc = launch_ring<false>(g2, A, st);
    return rc;
  }
  if (A / g1.E >= WGT_NT_ROWS) {
    if (up && (rc = launch_even<true, true, false>(g1, A, row_split, st)) != MOE_OK) return rc;
    if (down) rc = launch_even<false, true, false>(g2, A, row_split, st);
  } else if (A / g1.E >= ALTERNATE_MIN_ROWS) {
    if (up && (rc = launch_even<true, true, true>(g1, A, row_split, st)) != MOE_OK) return rc;
    if (down) rc = launch_even<false, true, true>(g2, A, row_split, st);
  } else {
    if (up && (rc = launch_even<true, false, true>(g1, A, row_split, st)) != MOE_OK) return rc;
    if (down) rc = launch_even<false, false, true>(g2, A, row_split, st);
  }
  return rc;
}

// parts: bit 0 = gated up-projection (h), bit 1 = down-projection (y_perm)
// x_perm [T*k, d] with src_assign == nullptr, or x [T, d] with the src_assign map of the dispatch
// combine_w != nullptr (k = 1 layers only): y_perm is y [T, d]; row r of the down-projection is
// stored to y[src_assign[r]] times combine_w[src_assign[r]]
static int grouped_ffn_impl(const moe_shape_t* shape, const void* x_perm, const int32_t* src_assign,
                            const int32_t* offsets, const void* w1, const void* w3, const void* w2,
                            void* h, void* y_perm, int parts, void* hip_stream,
                            void* split_ws = nullptr, const float* combine_w = nullptr,
                            bool row_split = true) {
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
  GemmArgs g1{x_perm, w1, w3, h, offsets, E, d, F, 0, static_cast<int>(A), TILES_FIXED, 64,
              src_assign, shape->k, src_assign ? shape->T : static_cast<int>(A), n_cu,
              static_cast<float*>(split_ws), 0, nullptr, nullptr, 0};
  GemmArgs g2{h, w2, nullptr, y_perm, offsets, E, F, d, 0, static_cast<int>(A), TILES_FIXED, 64,
              nullptr, 1, static_cast<int>(A), n_cu, static_cast<float*>(split_ws), 0,
              combine_w ? src_assign : nullptr, combine_w, shape->T};
  const bool up = parts & 1, down = parts & 2;
  if (shape->dtype == MOE_BF16 && d % 64 == 0 && F % 64 == 0) {
    g1.n_tiles = (F + 127) / 128;
    g2.n_tiles = (d + 255) / 256;
    return mfma_ffn(g1, g2, up, down, A, row_split, st);
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
  const bool whole_tiles = (parts & 4) != 0;
  parts &= ~4;
  if (parts < 1 || parts > 3) return MOE_ERR_INVALID_ARG;
  if (workspace) {
    if (!moe::aligned16(workspace)) return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < ffn_split_workspace_bytes()) return MOE_ERR_WORKSPACE;
  }
  return moe::grouped_ffn_impl(shape, x, src_assign, offsets, w1, w3, w2, h, y_perm, parts,
                               hip_stream, workspace, nullptr, !whole_tiles);
}

extern "C" int moe_grouped_ffn_gather(const moe_shape_t* shape, const void* x,
                                      const int32_t* src_assign, const int32_t* offsets,
                                      const void* w1, const void* w3, const void* w2, void* h,
                                      void* y_perm, void* hip_stream) {
  if (!src_assign) return MOE_ERR_INVALID_ARG;
  return moe::grouped_ffn_impl(shape, x, src_assign, offsets, w1, w3, w2, h, y_perm, 3, hip_stream);
}

extern "C" int moe_grouped_ffn_combine_k1(const moe_shape_t* shape, const void* x,
                                          const int32_t* src_assign, const int32_t* offsets,
                                          const void* w1, const void* w3, const void* w2,
                                          const float* topk_w, void* h, void* y, void* hip_stream) {
  if (!shape) return MOE_ERR_INVALID_ARG;
  if (shape->k != 1) return MOE_ERR_UNSUPPORTED;
  if (!src_assign || !topk_w) return MOE_ERR_INVALID_ARG;
  return moe::grouped_ffn_impl(shape, x, src_assign, offsets, w1, w3, w2, h, y, 3, hip_stream, nullptr,
                               topk_w);
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
