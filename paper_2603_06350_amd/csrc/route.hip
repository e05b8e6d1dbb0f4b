// moe_route: gate product, softmax and top-k routing (Section 2.2: the gating
// network routes each token to its experts; the gate is a bias-free d x E linear
// map, Sections 5 and 6.6).
//
// One block = one 16-row MFMA tile of tokens, 8 waves.  Large batches fill all 16
// rows; small ones give a block fewer tokens (down to one, the other rows idle) so
// that the batch still spreads over the chip.  The waves split the hidden dimension;
// each runs v_mfma_f32_16x16x32_bf16 on its slice straight from global memory (x is
// read exactly once from HBM, 16 B per lane; w_gate is small and stays in L2), the
// eight partial score tiles meet in LDS and are summed in a fixed order, so the
// scores are deterministic.  Each wave then routes its tokens: k+1 rounds of "largest
// remaining score, lowest index among equals" (a DPP maximum over the wave, then a
// ballot on equality), which also yields the gap from every chosen score to its
// nearest neighbour; the softmax weights come from the same scores.
//
// The integer choice must not depend on the order of an fp32 sum.  After the fast
// pass a token is "ambiguous" if one of its k chosen scores has another score within
// 2^-14 * max|logit| (plus a few ulps of the score itself).  For such tokens (about
// 1% for 64 experts, ~0.03% for 8) the whole block re-scores the experts that could
// still be among the first k (at most 16; all E if there are more) with exact
// products and fp64 sums rounded once to fp32, which is the correctly rounded score
// up to fp64 rounding, and the token is routed again.  fp32 inputs always take the
// exact path for all experts.
#include <type_traits>

#include "moe_internal.h"

namespace moe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

constexpr int RT_TM = 16;
constexpr int RT_NW = 8;
constexpr int RT_THREADS = RT_NW * MOE_WAVE;
constexpr int RT_BATCH = 8;   // MFMA steps whose x fragments are requested together

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}

constexpr int RT_CMAX = 16;   // candidate experts re-scored exactly for an ambiguous token

// Largest value of a wave, on every lane: four DPP steps make each row of 16 lanes hold its
// maximum (lane swaps inside quads, then the half-row and row mirrors), two row broadcasts carry
// it across the four rows into lane 63.
__device__ __forceinline__ float wave_max_dpp(float v) {
  auto step = [](float x, auto ctrl, auto rows) {
    const int moved = __builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x),
                                                  decltype(ctrl)::value, decltype(rows)::value, 0xF, false);
    return fmaxf(x, __int_as_float(moved));
  };
  using std::integral_constant;
  v = step(v, integral_constant<int, 0xB1>{}, integral_constant<int, 0xF>{});    // quad_perm [1,0,3,2]
  v = step(v, integral_constant<int, 0x4E>{}, integral_constant<int, 0xF>{});    // quad_perm [2,3,0,1]
  v = step(v, integral_constant<int, 0x141>{}, integral_constant<int, 0xF>{});   // row_half_mirror
  v = step(v, integral_constant<int, 0x140>{}, integral_constant<int, 0xF>{});   // row_mirror
  v = step(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{});   // row_bcast15 -> rows 1, 3
  v = step(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{});   // row_bcast31 -> rows 2, 3
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Routes one token with a full wave.  s[q] is the score of expert lane + 64 q.
// Selection: k (+1) rounds of "largest remaining score, lowest index among equals": the value by
// a DPP maximum over the wave, the index by a ballot on equality, both wave-uniform, so every
// pick costs a few dozen instructions whatever E is.  The extra round fetches the best score
// that is NOT chosen: the picks come out in descending order, so a chosen score's nearest
// neighbour is the pick before or after it.
// With `check`: if any of the k chosen experts has another score within the fast pass's error
// margin, nothing is written; the experts that could still be among the first k are listed in
// cand[] and their number is returned (RT_CMAX + 1 if there are too many).  Otherwise returns 0.
template <int QE>
__device__ int route_token(const float (&s)[QE], float lmax, bool check, int E, int k, int renorm,
                           int64_t t, int* __restrict__ cand, int32_t* __restrict__ topk_idx,
                           float* __restrict__ topk_w, float* __restrict__ scores_out) {
  const int lane = lane_id();
  bool valid[QE], taken[QE], chosen[QE];
  int rank[QE];
#pragma unroll
  for (int q = 0; q < QE; ++q) {
    valid[q] = lane + MOE_WAVE * q < E;
    taken[q] = !valid[q];
    rank[q] = 0x7FFFFFFF;
  }
  const int picks = E > k ? k + 1 : k;
  float prev = INFINITY, gap_prev = INFINITY, top = 0.f;
  bool amb = false;
  for (int i = 0; i < picks; ++i) {
    float loc = -INFINITY;
#pragma unroll
    for (int q = 0; q < QE; ++q)
      if (!taken[q]) loc = fmaxf(loc, s[q]);
    const float v = wave_max_dpp(loc);
    int e_star = E;                            // lowest index among the remaining scores equal to v
#pragma unroll
    for (int q = 0; q < QE; ++q) {
      const unsigned long long m = __ballot(!taken[q] && s[q] == v);
      if (m != 0ull && e_star == E) e_star = __ffsll(static_cast<long long>(m)) - 1 + MOE_WAVE * q;
    }
#pragma unroll
    for (int q = 0; q < QE; ++q) {
      if (lane + MOE_WAVE * q == e_star) {
        taken[q] = true;
        if (i < k) rank[q] = i;
      }
    }
    if (i == 0) top = v;
    if (i >= 1) {
      // pick i-1 is a chosen one (i-1 <= k-1): its neighbours are picks i-2 and i
      const float gap = prev - v;
      const float tol = 6.103515625e-05f * lmax + 9.5367431640625e-07f * fabsf(prev);
      amb = amb || !(fminf(gap_prev, gap) > tol);
      gap_prev = gap;
    }
    prev = v;
  }
  if (picks == k) {                            // E == k: the last chosen score has no lower neighbour
    const float tol = 6.103515625e-05f * lmax + 9.5367431640625e-07f * fabsf(prev);
    amb = amb || !(gap_prev > tol);
  }
#pragma unroll
  for (int q = 0; q < QE; ++q) chosen[q] = valid[q] && rank[q] < k;
  if (check && amb) {                          // wave-uniform
    // candidates: every expert whose score is not clearly below the neighbourhood of the last pick
    // (the best unchosen score, or the k-th chosen one if every expert is chosen)
    const float thr = prev;
    const float margin = 2.0f * (6.103515625e-05f * lmax + 9.5367431640625e-07f * fabsf(thr));
    int n = 0;
#pragma unroll
    for (int q = 0; q < QE; ++q) {
      const bool c = valid[q] && s[q] >= thr - margin;
      const unsigned long long m = __ballot(c);
      const int pos = n + __popcll(m & ((1ull << lane) - 1ull));
      if (c && pos < RT_CMAX) cand[pos] = lane + MOE_WAVE * q;
      n += __popcll(m);
    }
    return n <= RT_CMAX ? n : RT_CMAX + 1;
  }
  const float m = top;
  float p[QE];
  float psum = 0.f;
#pragma unroll
  for (int q = 0; q < QE; ++q) {
    p[q] = valid[q] ? expf(s[q] - m) : 0.f;
    psum += p[q];
  }
  const float denom = wave_sum(psum);
  float wsel = 0.f;
#pragma unroll
  for (int q = 0; q < QE; ++q) {
    p[q] = p[q] / denom;
    wsel += chosen[q] ? p[q] : 0.f;
  }
  const float ws = renorm ? wave_sum(wsel) : 1.0f;
#pragma unroll
  for (int q = 0; q < QE; ++q) {
    if (chosen[q]) {
      topk_idx[t * k + rank[q]] = lane + MOE_WAVE * q;
      topk_w[t * k + rank[q]] = renorm ? p[q] / ws : p[q];
    }
    if (scores_out && valid[q]) scores_out[t * E + lane + MOE_WAVE * q] = s[q];
  }
  return 0;
}

// Exact gate sums (fp64) of one token for up to RT_CMAX listed experts, this wave's part of the
// hidden dimension.  Lane = (candidate slot, one of four sub-slices).
template <bool BF16>
__device__ void exact_candidates(const uint4* __restrict__ xrow, const uint4* __restrict__ wg,
                                 int row16, const int* __restrict__ cand, int n, int wave,
                                 double* __restrict__ dpart) {
  const int lane = lane_id();
  const int c = lane & (RT_CMAX - 1);
  const int sub = lane / RT_CMAX;
  constexpr int NSUB = MOE_WAVE / RT_CMAX;
  const int e = cand[c < n ? c : 0];
  const uint4* wrow = wg + static_cast<int64_t>(e) * row16;
  const int cw = (row16 + RT_NW - 1) / RT_NW;
  const int c0 = wave * cw;
  const int c1 = min(row16, c0 + cw);
  double acc = 0.0;
  constexpr int XB = 8;
  for (int cb = c0 + sub; cb < c1; cb += XB * NSUB) {
    uint4 av[XB], bv[XB];
#pragma unroll
    for (int u = 0; u < XB; ++u) {
      const int cc = min(cb + u * NSUB, row16 - 1);
      av[u] = xrow[cc];
      bv[u] = wrow[cc];
    }
#pragma unroll
    for (int u = 0; u < XB; ++u) {
      if (cb + u * NSUB < c1) {
        const uint4 a = av[u];
        const uint4 b = bv[u];
        if (BF16) {
          acc = fma(static_cast<double>(bf16lo(a.x)), static_cast<double>(bf16lo(b.x)), acc);
          acc = fma(static_cast<double>(bf16hi(a.x)), static_cast<double>(bf16hi(b.x)), acc);
          acc = fma(static_cast<double>(bf16lo(a.y)), static_cast<double>(bf16lo(b.y)), acc);
          acc = fma(static_cast<double>(bf16hi(a.y)), static_cast<double>(bf16hi(b.y)), acc);
          acc = fma(static_cast<double>(bf16lo(a.z)), static_cast<double>(bf16lo(b.z)), acc);
          acc = fma(static_cast<double>(bf16hi(a.z)), static_cast<double>(bf16hi(b.z)), acc);
          acc = fma(static_cast<double>(bf16lo(a.w)), static_cast<double>(bf16lo(b.w)), acc);
          acc = fma(static_cast<double>(bf16hi(a.w)), static_cast<double>(bf16hi(b.w)), acc);
        } else {
          acc = fma(static_cast<double>(__uint_as_float(a.x)), static_cast<double>(__uint_as_float(b.x)), acc);
          acc = fma(static_cast<double>(__uint_as_float(a.y)), static_cast<double>(__uint_as_float(b.y)), acc);
          acc = fma(static_cast<double>(__uint_as_float(a.z)), static_cast<double>(__uint_as_float(b.z)), acc);
          acc = fma(static_cast<double>(__uint_as_float(a.w)), static_cast<double>(__uint_as_float(b.w)), acc);
        }
      }
    }
  }
  acc += __shfl_xor(acc, 16);
  acc += __shfl_xor(acc, 32);
  if (sub == 0 && c < n) dpart[wave * RT_CMAX + c] = acc;
}

// Exact partial gate sums of one token over this wave's part of the hidden
// dimension: products are exact in fp64 (bf16 x bf16 and fp32 x fp32 both fit),
// sums are fp64.  Lanes are (expert, sub-slice) pairs when E < 64.
template <bool BF16, int QE>
__device__ void exact_partial(const uint4* __restrict__ xrow, const uint4* __restrict__ wg,
                              int row16, int E, int wave, double* __restrict__ dpart) {
  const int lane = lane_id();
  int ep = 1;
  while (ep < E && ep < MOE_WAVE) ep <<= 1;
  const int nsub = MOE_WAVE / ep;
  const int e_l = lane & (ep - 1);
  const int sub = lane / ep;
  const int cw = (row16 + RT_NW - 1) / RT_NW;
  const int c0 = wave * cw;
  const int c1 = min(row16, c0 + cw);
#pragma unroll
  for (int q = 0; q < QE; ++q) {
    const int e = e_l + MOE_WAVE * q;
    const int e_ld = min(e, E - 1);
    const uint4* wrow = wg + static_cast<int64_t>(e_ld) * row16;
    double acc = 0.0;
    // eight chunk pairs are requested before the first is used (the loads are L2/HBM round
    // trips; the fp64 sum order stays ascending in c)
    constexpr int XB = 8;
    for (int cb = c0 + sub; cb < c1; cb += XB * nsub) {
      uint4 av[XB], bv[XB];
#pragma unroll
      for (int u = 0; u < XB; ++u) {
        const int c = min(cb + u * nsub, row16 - 1);
        av[u] = xrow[c];
        bv[u] = wrow[c];
      }
#pragma unroll
      for (int u = 0; u < XB; ++u) {
        if (cb + u * nsub < c1) {
          const uint4 a = av[u];
          const uint4 b = bv[u];
          if (BF16) {
            acc = fma(static_cast<double>(bf16lo(a.x)), static_cast<double>(bf16lo(b.x)), acc);
            acc = fma(static_cast<double>(bf16hi(a.x)), static_cast<double>(bf16hi(b.x)), acc);
            acc = fma(static_cast<double>(bf16lo(a.y)), static_cast<double>(bf16lo(b.y)), acc);
            acc = fma(static_cast<double>(bf16hi(a.y)), static_cast<double>(bf16hi(b.y)), acc);
            acc = fma(static_cast<double>(bf16lo(a.z)), static_cast<double>(bf16lo(b.z)), acc);
            acc = fma(static_cast<double>(bf16hi(a.z)), static_cast<double>(bf16hi(b.z)), acc);
            acc = fma(static_cast<double>(bf16lo(a.w)), static_cast<double>(bf16lo(b.w)), acc);
            acc = fma(static_cast<double>(bf16hi(a.w)), static_cast<double>(bf16hi(b.w)), acc);
          } else {
            acc = fma(static_cast<double>(__uint_as_float(a.x)), static_cast<double>(__uint_as_float(b.x)), acc);
            acc = fma(static_cast<double>(__uint_as_float(a.y)), static_cast<double>(__uint_as_float(b.y)), acc);
            acc = fma(static_cast<double>(__uint_as_float(a.z)), static_cast<double>(__uint_as_float(b.z)), acc);
            acc = fma(static_cast<double>(__uint_as_float(a.w)), static_cast<double>(__uint_as_float(b.w)), acc);
          }
        }
      }
    }
    for (int off = ep; off < MOE_WAVE; off <<= 1) acc += __shfl_xor(acc, off);
    if (sub == 0 && e < E) dpart[wave * E + e] = acc;
  }
}

// Dynamic LDS: float part[RT_NW][RT_TM][E] | double dpart[RT_NW][max(E,RT_CMAX)] |
//              int cand[RT_TM][RT_CMAX] | int flag[RT_TM]
// RPW = tile rows routed per wave: 2 (a full 16-token tile; compile-time so that the two tokens'
// dependency chains interleave) or 1 (tpb <= 8 tokens per block).
template <bool BF16, int NT, int RPW>
__global__ __launch_bounds__(RT_THREADS) void route_kernel(
    const uint4* __restrict__ x, const uint4* __restrict__ wg, const float* __restrict__ bias, int T,
    int d, int E, int k, int renorm, int tpb, int32_t* __restrict__ topk_idx,
    float* __restrict__ topk_w, float* __restrict__ scores_out) {
  constexpr int QE = NT >= 4 ? NT / 4 : 1;
  extern __shared__ __align__(16) unsigned char smem[];
  float* part = reinterpret_cast<float*>(smem);
  const int dn = E > RT_CMAX ? E : RT_CMAX;
  double* dpart = reinterpret_cast<double*>(smem + static_cast<size_t>(RT_NW) * RT_TM * E * 4);
  int* cand_all = reinterpret_cast<int*>(dpart + RT_NW * dn);
  int* flag = cand_all + RT_TM * RT_CMAX;
  const int lane = lane_id();
  const int wave = threadIdx.x / MOE_WAVE;
  const int t0 = blockIdx.x * tpb;     // this block's tokens are tile rows [0, tpb)
  const int row16 = BF16 ? d / 8 : d / 4;
  // fp32 scores of tile row `row` from the eight partial tiles (fixed order) plus the bias;
  // returns the row's largest |logit| (before the bias)
  auto fast_scores = [&](int row, float (&s)[QE]) -> float {
    float la = 0.f;
#pragma unroll
    for (int q = 0; q < QE; ++q) {
      const int e = lane + MOE_WAVE * q;
      float v = 0.f;
      if (e < E) {
#pragma unroll
        for (int w = 0; w < RT_NW; ++w) v += part[(w * RT_TM + row) * E + e];
        la = fmaxf(la, fabsf(v));
        if (bias) v += bias[e];
      }
      s[q] = v;
    }
    return wave_max(la);
  };

  if (BF16) {
    // ---- fast pass: partial score tiles on the matrix cores ---------------------------------
    const int r = lane & 15;   // token row of the A fragment / expert column of the B fragment
    const int kq = lane >> 4;  // which 8-element group of the 32-wide MFMA step
    const int t_ld = min(t0 + min(r, tpb - 1), T - 1);
    const uint4* xrow = x + static_cast<int64_t>(t_ld) * row16;
    const uint4* wrow[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      wrow[nt] = wg + static_cast<int64_t>(min(nt * 16 + r, E - 1)) * row16;
    f32x4_t acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const int cw = ((row16 + RT_NW * 4 - 1) / (RT_NW * 4)) * 4;  // 16 B chunks per wave
    const int c0 = wave * cw;
    const int c1 = min(row16, c0 + cw);
    // x comes from HBM and is read exactly once: a batch of RT_BATCH MFMA steps has all of its
    // x fragments requested before the first one is used, so each wave keeps 8 KiB in flight.
    // w_gate fragments come from L2 and are fetched per step.
    for (int cb = c0; cb < c1; cb += 4 * RT_BATCH) {
      uint4 a[RT_BATCH];
#pragma unroll
      for (int u = 0; u < RT_BATCH; ++u) {
        const int cc = cb + 4 * u + kq;
        a[u] = xrow[min(cc, row16 - 1)];
      }
      // w_gate fragments: BSTEPS steps' worth (16 loads) are requested together
      constexpr int BSTEPS = NT >= 16 ? 1 : (NT <= 2 ? 8 : 16 / NT);
#pragma unroll
      for (int u0 = 0; u0 < RT_BATCH; u0 += BSTEPS) {
        uint4 b[BSTEPS][NT];
#pragma unroll
        for (int u = 0; u < BSTEPS; ++u) {
          const int cl = min(cb + 4 * (u0 + u) + kq, row16 - 1);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) b[u][nt] = wrow[nt][cl];
        }
#pragma unroll
        for (int u = 0; u < BSTEPS; ++u) {
          if (cb + 4 * (u0 + u) < c1) {                // wave-uniform
            uint4 av = a[u0 + u];
            if (cb + 4 * (u0 + u) + kq >= row16) av = make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av),
                                                                __builtin_bit_cast(bf16x8_t, b[u][nt]),
                                                                acc[nt], 0, 0, 0);
          }
        }
      }
    }
    // D layout of the 16x16 tile: lane holds expert column (lane & 15), token rows 4*(lane>>4)+v
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int e = nt * 16 + r;
      if (e < E) {
#pragma unroll
        for (int v = 0; v < 4; ++v) part[(wave * RT_TM + 4 * kq + v) * E + e] = acc[nt][v];
      }
    }
    __syncthreads();
    // ---- routing: tile rows are dealt to the waves ----------------------------------------------
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
      const int row = wave * RPW + rr;
      if (RPW == 1 && row >= tpb) break;
      const int t = t0 + row;
      int amb = 0;
      if (t < T) {
        float s[QE];
        const float lmax = fast_scores(row, s);
        amb = route_token<QE>(s, lmax, true, E, k, renorm, t, cand_all + row * RT_CMAX, topk_idx,
                              topk_w, scores_out);
      }
      if (lane == 0) flag[row] = amb;
    }
  } else {
    const int tid = static_cast<int>(threadIdx.x);
    if (tid < tpb) flag[tid] = (t0 + tid < T) ? RT_CMAX + 1 : 0;
  }
  __syncthreads();
  // ---- exact pass for the tokens that need it (block-uniform control flow) -------------------
  for (int row = 0; row < tpb; ++row) {
    const int n = flag[row];
    if (n == 0) continue;
    const int t = t0 + row;
    const uint4* xrow = x + static_cast<int64_t>(t) * row16;
    const int* cand = cand_all + row * RT_CMAX;
    if (n <= RT_CMAX)
      exact_candidates<BF16>(xrow, wg, row16, cand, n, wave, dpart);
    else
      exact_partial<BF16, QE>(xrow, wg, row16, E, wave, dpart);
    __syncthreads();
    if (wave == (row % RT_NW)) {
      float s[QE];
      if (n <= RT_CMAX) {
        // fast scores everywhere, exact (fp64 sum, one rounding) for the listed candidates
        fast_scores(row, s);
        for (int c = 0; c < n; ++c) {
          const int e = cand[c];
          double v = 0.0;
#pragma unroll
          for (int w = 0; w < RT_NW; ++w) v += dpart[w * RT_CMAX + c];
          if (bias) v += static_cast<double>(bias[e]);
#pragma unroll
          for (int q = 0; q < QE; ++q)
            if (e == lane + MOE_WAVE * q) s[q] = static_cast<float>(v);
        }
      } else {
#pragma unroll
        for (int q = 0; q < QE; ++q) {
          const int e = lane + MOE_WAVE * q;
          double v = 0.0;
          if (e < E) {
#pragma unroll
            for (int w = 0; w < RT_NW; ++w) v += dpart[w * E + e];
            if (bias) v += static_cast<double>(bias[e]);
          }
          s[q] = static_cast<float>(v);
        }
      }
      route_token<QE>(s, 0.f, false, E, k, renorm, t, nullptr, topk_idx, topk_w, scores_out);
    }
    __syncthreads();
  }
}

static size_t route_lds_bytes(int E) {
  const size_t dn = E > RT_CMAX ? E : RT_CMAX;
  return static_cast<size_t>(RT_NW) * RT_TM * E * 4 + RT_NW * dn * 8 +
         RT_TM * RT_CMAX * sizeof(int) + RT_TM * sizeof(int);
}

template <bool BF16, int NT, int RPW>
static int launch_route_rpw(const moe_shape_t* s, const void* x, const void* wg, const float* bias,
                            int32_t* idx, float* w, float* scores, int tpb, hipStream_t st) {
  static LdsOnce once;
  if (ensure_dynamic_lds(once, reinterpret_cast<const void*>(route_kernel<BF16, NT, RPW>),
                         static_cast<int>(route_lds_bytes(MOE_MAX_E))) != MOE_OK)
    return MOE_ERR_HIP;
  const int grid = (s->T + tpb - 1) / tpb;
  hipLaunchKernelGGL((route_kernel<BF16, NT, RPW>), dim3(grid), dim3(RT_THREADS),
                     route_lds_bytes(s->E), st, static_cast<const uint4*>(x),
                     static_cast<const uint4*>(wg), bias, s->T, s->d, s->E, s->k, s->renorm, tpb, idx,
                     w, scores);
  return launch_status();
}

template <bool BF16, int NT>
static int launch_route(const moe_shape_t* s, const void* x, const void* wg, const float* bias,
                        int32_t* idx, float* w, float* scores, hipStream_t st) {
  // Tokens per block: a full 16-row tile when that still gives every CU a few blocks; fewer
  // (the other tile rows idle) for small batches, where latency, not MFMA use, is what counts.
  constexpr int GRID_TARGET = 512;
  int tpb = RT_TM;
  while (tpb > 1 && (s->T + tpb - 1) / tpb < GRID_TARGET) tpb >>= 1;
  return tpb == RT_TM
             ? launch_route_rpw<BF16, NT, 2>(s, x, wg, bias, idx, w, scores, tpb, st)
             : launch_route_rpw<BF16, NT, 1>(s, x, wg, bias, idx, w, scores, tpb, st);
}

}  // namespace moe

extern "C" int moe_route(const moe_shape_t* shape, const void* x, const void* w_gate,
                         const float* gate_bias, int32_t* topk_idx, float* topk_w,
                         float* scores_out, void* hip_stream) {
  const int rc = moe::check_shape(shape);
  if (rc != MOE_OK) return rc;
  if (shape->T == 0) return MOE_OK;
  if (!x || !w_gate || !topk_idx || !topk_w) return MOE_ERR_INVALID_ARG;
  if (!moe::aligned16(x) || !moe::aligned16(w_gate)) return MOE_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int E = shape->E;
  if (shape->dtype == MOE_BF16) {
    if (E <= 16) return moe::launch_route<true, 1>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, st);
    if (E <= 32) return moe::launch_route<true, 2>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, st);
    if (E <= 64) return moe::launch_route<true, 4>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, st);
    if (E <= 128) return moe::launch_route<true, 8>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, st);
    return moe::launch_route<true, 16>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, st);
  }
  if (E <= 64) return moe::launch_route<false, 4>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, st);
  if (E <= 128) return moe::launch_route<false, 8>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, st);
  return moe::launch_route<false, 16>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, st);
}
