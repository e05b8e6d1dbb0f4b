// moe_grouped_ffn: the expert computation that dominates the MoE layer (Section 3.2).
// For every expert e and row r of its segment [offsets[e], offsets[e+1]):
//   h[r] = silu(W1_e x_perm[r]) * (W3_e x_perm[r]),   y_perm[r] = W2_e h[r].
//
// Two launches: a gated GEMM (W1 and W3 tiles side by side, SwiGLU applied to the
// fp32 accumulators, h stored once) and a plain GEMM for W2.  Both are ragged
// grouped GEMMs: the tile list is derived on the device from `offsets`, so the host
// never learns the expert loads.
//
// bf16 kernel (gfx950): 512 threads = 8 waves (two per SIMD, so one wave's LDS
// waits hide behind the other's MFMAs); block tile BM rows x 256 weight rows,
// K step 64.  Both operands are K-contiguous in memory, so a tile
// row is 128 B = eight 16-byte chunks.  Tiles go global -> LDS with the direct
// 16-byte-per-lane loads (no register staging), double buffered; a wave
// instruction fills 8 rows, and the chunk a lane fetches is XOR-swizzled by row so
// that the later 16-byte LDS reads of a 32-row MFMA operand spread over all banks.
// The weight fragment is fed as the MFMA "A" operand and the activation fragment
// as "B": each lane then owns 4 consecutive output columns of one output row and
// stores them as one 8-byte word.  v_mfma_f32_32x32x16_bf16, fp32 accumulators.
//
// Work-group ids are remapped so that each XCD (ids are dealt round-robin to the 8
// XCDs) walks a contiguous range of the tile list with the m-tiles of one weight
// panel adjacent: CUs that share an L2 share weight tiles.
//
// Generic kernel (fp32, or bf16 shapes whose d or F is not a multiple of 64): a
// plain LDS-tiled FMA GEMM with fp32 accumulation.
#include "moe_internal.h"

namespace moe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

struct GemmArgs {
  const void* a;    // activations [rows, K]
  const void* b0;   // gated: W1 [E,N,K]   plain: W2 [E,N,K]
  const void* b1;   // gated: W3 [E,N,K]   plain: unused
  void* out;        // [rows, N]
  const int32_t* offsets;
  int E, K, N;
  int n_tiles;      // tiles along N
  int rows;         // T*k; row ranges read from `offsets` are clamped to it
};

struct TileCoord {
  int e, m_begin, m_end, n_tile;
};

// Maps a work-group to (expert, row range, n-tile).  Every wave computes this on
// its own from the device-resident offsets; returns false if the group has no tile.
// Tile order: expert-major, then n-tile, then m-tile (m fastest), cut into 8
// contiguous ranges, one per XCD.
__device__ __forceinline__ bool decode_tile(const int32_t* __restrict__ offsets, int E, int BM,
                                            int n_tiles, int rows, TileCoord& tc) {
  const int lane = lane_id();
  const int per = (E + MOE_WAVE - 1) / MOE_WAVE;  // <= 4
  const int e0 = lane * per;
  int mt[4];
  int local = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int e = e0 + i;
    int c = 0;
    if (i < per && e < E) c = (offsets[e + 1] - offsets[e] + BM - 1) / BM;
    c = max(c, 0);
    mt[i] = c;
    local += c;
  }
  int incl = local;
#pragma unroll
  for (int off = 1; off < MOE_WAVE; off <<= 1) {
    const int up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  const int total = __builtin_amdgcn_readfirstlane(__shfl(incl, MOE_WAVE - 1)) * n_tiles;
  const int per_xcd = (total + 7) / 8;
  const int xcd = blockIdx.x & 7;
  const int slot = blockIdx.x >> 3;
  const int vid = xcd * per_xcd + slot;
  if (slot >= per_xcd || vid >= total) return false;
  int run = incl - local;
  int found_e = -1, found_local = 0, found_mt = 1;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int s = run * n_tiles;
    if (mt[i] > 0 && vid >= s && vid < s + mt[i] * n_tiles) {
      found_e = e0 + i;
      found_local = vid - s;
      found_mt = mt[i];
    }
    run += mt[i];
  }
  const unsigned long long who = __ballot(found_e >= 0);
  if (who == 0ull) return false;  // inconsistent offsets: no tile
  const int src = __ffsll(static_cast<long long>(who)) - 1;
  // readfirstlane: the results are wave-uniform; tell the compiler so they live in SGPRs
  const int e = __builtin_amdgcn_readfirstlane(__shfl(found_e, src));
  const int loc = __builtin_amdgcn_readfirstlane(__shfl(found_local, src));
  const int m_tiles = __builtin_amdgcn_readfirstlane(__shfl(found_mt, src));
  const int m_idx = loc % m_tiles;
  tc.e = e;
  tc.n_tile = loc / m_tiles;
  tc.m_begin = max(offsets[e], 0) + m_idx * BM;
  tc.m_end = min(offsets[e + 1], rows);
  return tc.m_begin < tc.m_end;
}

__device__ __forceinline__ float silu_mul(float g, float u) {
  return g * u * __frcp_rn(1.0f + __expf(-g));
}

// --------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// --------------------------------------------------------------------------------------------
constexpr int BK = 64;          // K elements per stage
constexpr int ROWB = BK * 2;    // bytes per tile row in LDS
constexpr int BROWS = 256;      // weight rows per block tile

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

template <int BM, bool GATED, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void ffn_mfma_kernel(GemmArgs p) {
  constexpr int NW = WM * WN;                     // waves per block
  constexpr int MI = BM / WM / 32;                // 32-row activation sub-tiles per wave
  constexpr int NI = BROWS / WN / 32;             // 32-row weight sub-tiles per wave
  constexpr int NIH = GATED ? NI / 2 : NI;        // gated: sub-tiles per weight matrix
  constexpr int STAGE = (BM + BROWS) * ROWB;      // bytes per stage
  constexpr int NLOAD = (BM + BROWS) / 8 / NW;    // direct-to-LDS instructions per wave per stage
  constexpr int NLA = BM / 8 / NW;                // ... of which load activation rows
  constexpr int NLB = 128 / 8 / NW;               // ... per 128 weight rows
  constexpr int BN_OUT = GATED ? 128 : 256;       // output columns per block tile
  static_assert(NLA * 8 * NW == BM && NLB * 8 * NW == 128 && MI >= 1 && NIH >= 1, "tile shape");
  extern __shared__ __align__(1024) unsigned char lds[];

  TileCoord tc;
  if (!decode_tile(p.offsets, p.E, BM, p.n_tiles, p.rows, tc)) return;

  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);
  const int wm = wave / WN, wn = wave % WN;
  const int K = p.K, N = p.N;
  const int n0 = tc.n_tile * BN_OUT;
  const bf16_t* A = static_cast<const bf16_t*>(p.a);
  const bf16_t* B0 = static_cast<const bf16_t*>(p.b0) + static_cast<int64_t>(tc.e) * N * K;
  const bf16_t* B1 = GATED ? static_cast<const bf16_t*>(p.b1) + static_cast<int64_t>(tc.e) * N * K
                           : nullptr;

  // ---- global -> LDS assignment: instruction i of this wave fills row group g = i*NW + wave.
  //      Which matrix a row group belongs to depends on i alone, so each instruction has a
  //      uniform 64-bit base and a 32-bit per-lane offset.
  const unsigned char* base_a =
      reinterpret_cast<const unsigned char*>(A + static_cast<int64_t>(tc.m_begin) * K);
  const unsigned char* base_b0 =
      reinterpret_cast<const unsigned char*>(B0 + static_cast<int64_t>(n0) * K);
  const unsigned char* base_b1 =
      GATED ? reinterpret_cast<const unsigned char*>(B1 + static_cast<int64_t>(n0) * K) : nullptr;
  uint32_t soff[NLOAD];
#pragma unroll
  for (int i = 0; i < NLOAD; ++i) {
    const int g = i * NW + wave;
    const int row = g * 8 + (lane >> 3);          // row in the stage: [0,BM) x rows, then weights
    const int chunk = (lane & 7) ^ swz(row);      // the 16 B chunk of the row this lane fetches
    int r;                                        // row relative to the instruction's base
    if (i < NLA) {
      r = min(row, tc.m_end - 1 - tc.m_begin);
    } else {
      const int br = row - BM;
      r = GATED ? min(br & 127, N - 1 - n0) : min(br, N - 1 - n0);
    }
    soff[i] = static_cast<uint32_t>(r) * static_cast<uint32_t>(K) * 2u + static_cast<uint32_t>(chunk) * 16u;
  }
  auto issue_loads = [&](int kt, int stage) {
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int g = i * NW + wave;
      const unsigned char* base =
          (i < NLA) ? base_a : (!GATED || i < NLA + NLB) ? base_b0 : base_b1;
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(base + static_cast<int64_t>(kt) * ROWB + soff[i]),
          (__attribute__((address_space(3))) void*)(lds + stage * STAGE + g * 1024), 16, 0, 0);
    }
  };

  // ---- LDS read addresses of the MFMA fragments ------------------------------------------------
  const int l32 = lane & 31;
  const int f = swz(lane);                        // sub-tile bases are multiples of 32 rows
  int koff[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) koff[kk] = (((kk * 2 + (lane >> 5)) ^ f) << 4);
  const int x_base = (wm * (BM / WM) + l32) * ROWB;
  int w_sub[NI];                                  // first weight row of sub-tile ni in the stage
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
    w_sub[ni] = GATED ? (ni / NIH) * 128 + wn * (NIH * 32) + (ni % NIH) * 32
                      : wn * (NI * 32) + ni * 32;
  const int w_base = (BM + l32) * ROWB;

  f32x16_t acc[NI][MI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.f;

  auto load_frags = [&](const unsigned char* sb, int kk, bf16x8_t (&xf)[MI], bf16x8_t (&wf)[NI]) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
      xf[mi] = *reinterpret_cast<const bf16x8_t*>(sb + x_base + mi * 32 * ROWB + koff[kk]);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
      wf[ni] = *reinterpret_cast<const bf16x8_t*>(sb + w_base + w_sub[ni] * ROWB + koff[kk]);
  };
  auto mma = [&](const bf16x8_t (&xf)[MI], const bf16x8_t (&wf)[NI]) {
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ni], xf[mi], acc[ni][mi], 0, 0, 0);
  };
  // one stage = 4 MFMA k-steps; the fragments of step kk+1 are read while step kk multiplies
  auto compute = [&](int stage) {
    const unsigned char* sb = lds + stage * STAGE;
    bf16x8_t xa[MI], wa[NI], xb[MI], wb[NI];
    load_frags(sb, 0, xa, wa);
    load_frags(sb, 1, xb, wb);
    mma(xa, wa);
    load_frags(sb, 2, xa, wa);
    mma(xb, wb);
    load_frags(sb, 3, xb, wb);
    mma(xa, wa);
    mma(xb, wb);
  };

  const int KT = K / BK;
  issue_loads(0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  for (int kt = 0; kt < KT; kt += 2) {
    if (kt + 1 < KT) issue_loads(kt + 1, 1);
    compute(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (kt + 1 < KT) {
      if (kt + 2 < KT) issue_loads(kt + 2, 0);
      compute(1);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    }
  }

  // ---- epilogue: accumulator (v, lane) holds out[row = m-sub-tile + lane%32]
  //      [col = n-sub-tile + 8*(v/4) + 4*(lane/32) + v%4] -------------------------------------
  bf16_t* out = static_cast<bf16_t*>(p.out);
  const int row_l = wm * (BM / WM) + l32;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int gr = tc.m_begin + row_l + mi * 32;
    if (gr >= tc.m_end) continue;
    bf16_t* orow = out + static_cast<int64_t>(gr) * N;
#pragma unroll
    for (int ni = 0; ni < NIH; ++ni) {
      const int cb = n0 + wn * (NIH * 32) + ni * 32 + 4 * (lane >> 5);
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const int c = cb + 8 * vq;
        if (c < N) {
          float o[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            if (GATED)
              o[u] = silu_mul(acc[ni][mi][4 * vq + u], acc[GATED ? ni + NIH : ni][mi][4 * vq + u]);
            else
              o[u] = acc[ni][mi][4 * vq + u];
          }
          *reinterpret_cast<uint2*>(orow + c) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
        }
      }
    }
  }
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
  if (!decode_tile(p.offsets, p.E, TM, p.n_tiles, p.rows, tc)) return;
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
  const int a_row = min(tc.m_begin + lr, tc.m_end - 1);
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

// Upper bound on sum_e ceil(count_e / BM) that needs no knowledge of the counts.
static int64_t max_m_tiles(int64_t A, int E, int BM) {
  const int64_t ub = A / BM + E;
  return ub < A ? ub : A;
}

template <int BM, bool GATED, int WM, int WN>
static int launch_mfma(const GemmArgs& a, int64_t A, hipStream_t st) {
  constexpr int lds_bytes = 2 * (BM + BROWS) * ROWB;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_mfma_kernel<BM, GATED, WM, WN>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
      return MOE_ERR_HIP;
    attr_set = true;
  }
  int64_t grid = max_m_tiles(A, a.E, BM) * a.n_tiles;
  grid = (grid + 7) / 8 * 8;
  if (grid > 0x7FFFFFFF) return MOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((ffn_mfma_kernel<BM, GATED, WM, WN>), dim3(static_cast<unsigned>(grid)),
                     dim3(WM * WN * 64), lds_bytes, st, a);
  return launch_status();
}

template <typename T, bool GATED>
static int launch_generic(const GemmArgs& a, int64_t A, hipStream_t st) {
  int64_t grid = max_m_tiles(A, a.E, 64) * a.n_tiles;
  grid = (grid + 7) / 8 * 8;
  if (grid > 0x7FFFFFFF) return MOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((ffn_generic_kernel<T, GATED>), dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                     st, a);
  return launch_status();
}

}  // namespace moe

// parts: bit 0 = gated up-projection (h), bit 1 = down-projection (y_perm)
static int grouped_ffn_impl(const moe_shape_t* shape, const void* x_perm, const int32_t* offsets,
                            const void* w1, const void* w3, const void* w2, void* h, void* y_perm,
                            int parts, void* hip_stream) {
  using namespace moe;
  int rc = check_shape(shape);
  if (rc != MOE_OK) return rc;
  if (shape->T == 0) return MOE_OK;
  if (!x_perm || !offsets || !w1 || !w3 || !w2 || !h || !y_perm) return MOE_ERR_INVALID_ARG;
  if (!aligned16(x_perm) || !aligned16(w1) || !aligned16(w3) || !aligned16(w2) || !aligned16(h) ||
      !aligned16(y_perm))
    return MOE_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int64_t A = static_cast<int64_t>(shape->T) * shape->k;
  const int d = shape->d, F = shape->F, E = shape->E;
  GemmArgs g1{x_perm, w1, w3, h, offsets, E, d, F, 0, static_cast<int>(A)};
  GemmArgs g2{h, w2, nullptr, y_perm, offsets, E, F, d, 0, static_cast<int>(A)};
  const bool up = parts & 1, down = parts & 2;
  if (shape->dtype == MOE_BF16 && d % 64 == 0 && F % 64 == 0) {
    g1.n_tiles = (F + 127) / 128;
    g2.n_tiles = (d + 255) / 256;
    const bool big = A / E >= 512;
    if (up) {
      rc = big ? launch_mfma<256, true, 4, 2>(g1, A, st) : launch_mfma<128, true, 2, 4>(g1, A, st);
      if (rc != MOE_OK) return rc;
    }
    if (down)
      rc = big ? launch_mfma<256, false, 4, 2>(g2, A, st) : launch_mfma<128, false, 2, 4>(g2, A, st);
    return rc;
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

extern "C" int moe_grouped_ffn(const moe_shape_t* shape, const void* x_perm, const int32_t* offsets,
                               const void* w1, const void* w3, const void* w2, void* h, void* y_perm,
                               void* hip_stream) {
  return grouped_ffn_impl(shape, x_perm, offsets, w1, w3, w2, h, y_perm, 3, hip_stream);
}

extern "C" int moe_grouped_ffn_part(const moe_shape_t* shape, const void* x_perm,
                                    const int32_t* offsets, const void* w1, const void* w3,
                                    const void* w2, void* h, void* y_perm, int part,
                                    void* hip_stream) {
  if (part != 1 && part != 2) return MOE_ERR_INVALID_ARG;
  return grouped_ffn_impl(shape, x_perm, offsets, w1, w3, w2, h, y_perm, part, hip_stream);
}
