// moe_route: gate product, softmax and top-k routing (Section 2.2: the gating
// network routes each token to its experts; the gate is a bias-free d x E linear
// map, Sections 5 and 6.6).
//
// Three forms, chosen on the host by the shape: route_kernel (below; every batch size, every
// dtype), route_tile_kernel (large bf16 batches: several token tiles per block share one pass of
// w_gate through LDS, selection by per-lane tournaments) and gate_tile_kernel + route_kernel<PRE>
// (small batches with a workspace: the gate product spread over the chip first).
//
// route_kernel: one block = one 16-row MFMA tile of tokens, 8 waves.  Large batches fill all 16
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
// 2^-19 * |x_t| * max_e |w_e| (Euclidean norms; plus a few ulps of the score itself).  The
// rounding errors of the fast pass scale with the magnitude of the products and partial sums,
// which the product of the norms bounds, not with the magnitude of the result: a token whose
// large terms cancel has tiny logits and large errors.  Both norms come out of the same pass
// (sums of squares of the fragments it multiplies).  For inputs without cancellation
// the margin is about 2^-14 of the largest logit, some 60 times the fast pass's typical error.
// For ambiguous tokens (about
// 1% for 64 experts, ~0.03% for 8) the whole block re-scores the experts that could
// still be among the first k (at most 16; all E if there are more) with exact
// products and fp64 sums rounded once to fp32, which is the correctly rounded score
// up to fp64 rounding, and the token is routed again.  fp32 inputs always take the
// exact path for all experts.
#include <type_traits>
#include <utility>

#include "moe_internal.h"

namespace moe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

constexpr int RT_TM = 16;
constexpr int RT_NW = 8;
constexpr int RT_THREADS = RT_NW * MOE_WAVE;
constexpr int RT_BATCH = 16;  // MFMA steps whose x fragments are requested together

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

// Two fast scores closer than RT_TOL * |x_t| * max_e |w_e| are re-scored exactly.
constexpr float RT_TOL = 1.9073486328125e-06f;   // 2^-19

// acc + the sum of the squares of the eight bf16 values of a fragment (v_dot2c_f32_bf16: vector ALU
// work that issues in the shadow of the MFMAs; as separate x x^T and w w^T MFMA tiles the norms
// cost the large-batch kernel 4 % at 8 experts).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
// Four running sums, one per dword of the fragment, so that consecutive fragments do not form one
// long chain of dependent instructions; rt_sumsq_total adds them up.
struct RtSumSq {
  float a = 0.f, b = 0.f, c = 0.f, d = 0.f;
};
__device__ __forceinline__ void rt_sumsq(uint4 v, RtSumSq& s) {
  s.a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, v.x), __builtin_bit_cast(bf16x2_t, v.x), s.a, false);
  s.b = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, v.y), __builtin_bit_cast(bf16x2_t, v.y), s.b, false);
  s.c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, v.z), __builtin_bit_cast(bf16x2_t, v.z), s.c, false);
  s.d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, v.w), __builtin_bit_cast(bf16x2_t, v.w), s.d, false);
}
__device__ __forceinline__ float rt_sumsq_total(const RtSumSq& s) { return (s.a + s.b) + (s.c + s.d); }
// (The four lanes l, l + 16, l + 32, l + 48 hold the four 16-byte chunks of a row's k-step, so a
// row's sum of squares is spread over them: each writes its part to LDS and the reader adds the
// four up; exchanging them between lanes first cost a microsecond of latency per block.)
__device__ __forceinline__ f32x4_t rt_mfma(uint4 a, uint4 b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                 __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

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
// bnd: |x_t| * max_e |w_e| of the token (see RT_TOL).
// With `check`: if any of the k chosen experts has another score within the fast pass's error
// margin, nothing is written; the experts that could still be among the first k are listed in
// cand[] and their number is returned (RT_CMAX + 1 if there are too many).  Otherwise returns 0.
template <int QE>
__device__ int route_token(const float (&s)[QE], float bnd, bool check, int E, int k, int renorm,
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
      const float tol = RT_TOL * bnd + 9.5367431640625e-07f * fabsf(prev);
      amb = amb || !(fminf(gap_prev, gap) > tol);
      gap_prev = gap;
    }
    prev = v;
  }
  if (picks == k) {                            // E == k: the last chosen score has no lower neighbour
    const float tol = RT_TOL * bnd + 9.5367431640625e-07f * fabsf(prev);
    amb = amb || !(gap_prev > tol);
  }
#pragma unroll
  for (int q = 0; q < QE; ++q) chosen[q] = valid[q] && rank[q] < k;
  if (check && amb) {                          // wave-uniform
    // candidates: every expert whose score is not clearly below the neighbourhood of the last pick
    // (the best unchosen score, or the k-th chosen one if every expert is chosen)
    const float thr = prev;
    const float margin = 2.0f * (RT_TOL * bnd + 9.5367431640625e-07f * fabsf(thr));
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

// Exact gate sum (fp64) of one (token row, expert row) pair per candidate slot, this wave's part
// of the hidden dimension.  Lane = (candidate slot lane % RT_CMAX, one of four sub-slices); the
// four sub-slice sums of a slot are added by two lane exchanges; the lanes of sub-slice 0 return
// the slot's sum.
template <bool BF16>
__device__ __forceinline__ double exact_slot_sum(const uint4* __restrict__ xrow,
                                                 const uint4* __restrict__ wrow, int row16, int wave) {
  const int sub = lane_id() / RT_CMAX;
  constexpr int NSUB = MOE_WAVE / RT_CMAX;
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
  return acc;
}

// Exact gate sums of one token for up to RT_CMAX listed experts: dpart[wave * RT_CMAX + slot].
template <bool BF16>
__device__ void exact_candidates(const uint4* __restrict__ xrow, const uint4* __restrict__ wg,
                                 int row16, const int* __restrict__ cand, int n, int wave,
                                 double* __restrict__ dpart) {
  const int lane = lane_id();
  const int c = lane & (RT_CMAX - 1);
  const int e = cand[c < n ? c : 0];
  const double acc = exact_slot_sum<BF16>(xrow, wg + static_cast<int64_t>(e) * row16, row16, wave);
  if (lane < RT_CMAX && c < n) dpart[wave * RT_CMAX + c] = acc;
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
//              int cand[RT_TM][RT_CMAX] | int flag[RT_TM] | float xn[RT_NW * 4][RT_TM] |
//              float wn[RT_NW * 4][<= 16 NT]   (per wave and lane group: parts of |x_t|^2 and |w_e|^2)
// RPW = tile rows routed per wave: 2 (a full 16-token tile; compile-time so that the two tokens'
// dependency chains interleave) or 1 (tpb <= 8 tokens per block).
// PRE: the fast scores (bias included) were already written to scores_in[T][E] by
// gate_tile_kernel, and |x_t|^2, |w_e|^2 to norms[T + E]; this kernel only selects and runs the
// exact pass.  scores_in may be the same buffer as scores_out: a token's scores are read before
// they are written.
template <bool BF16, int NT, int RPW, bool PRE>
__global__ __launch_bounds__(RT_THREADS) void route_kernel(
    const uint4* __restrict__ x, const uint4* __restrict__ wg, const float* __restrict__ bias, int T,
    int d, int E, int k, int renorm, int tpb, const float* scores_in, const float* __restrict__ norms,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, float* scores_out) {
  constexpr int QE = NT >= 4 ? NT / 4 : 1;
  // |w_e|^2 sums: one per 16 experts, or, from 128 experts on, one per 64 (four experts, 16 apart,
  // added up: still an upper bound of each)
  constexpr int WG = NT >= 8 ? 4 : 1;
  constexpr int NWT = NT / WG;
  constexpr int EP = NWT * 16;
  extern __shared__ __align__(16) unsigned char smem[];
  float* part = reinterpret_cast<float*>(smem);
  const int dn = E > RT_CMAX ? E : RT_CMAX;
  double* dpart = reinterpret_cast<double*>(smem + static_cast<size_t>(RT_NW) * RT_TM * E * 4);
  int* cand_all = reinterpret_cast<int*>(dpart + RT_NW * dn);
  int* flag = cand_all + RT_TM * RT_CMAX;
  float* xn = reinterpret_cast<float*>(flag + RT_TM);
  float* wn = xn + RT_NW * 4 * RT_TM;
  const int lane = lane_id();
  const int wave = threadIdx.x / MOE_WAVE;
  const int t0 = blockIdx.x * tpb;     // this block's tokens are tile rows [0, tpb)
  const int row16 = BF16 ? d / 8 : d / 4;
  float w2max = 0.f;                   // max_e |w_e|^2 (bf16 layers; set before the routing loop)
  // fp32 scores of tile row `row` from the eight partial tiles (fixed order) plus the bias;
  // returns |x_t| * max_e |w_e| of the row's token
  auto fast_scores = [&](int row, float (&s)[QE]) -> float {
#pragma unroll
    for (int q = 0; q < QE; ++q) {
      const int e = lane + MOE_WAVE * q;
      float v = 0.f;
      if (e < E) {
        if constexpr (PRE) {
          v = scores_in[static_cast<int64_t>(t0 + row) * E + e];
        } else {
#pragma unroll
          for (int w = 0; w < RT_NW; ++w) v += part[(w * RT_TM + row) * E + e];
          if (bias) v += bias[e];
        }
      }
      s[q] = v;
    }
    float x2 = 0.f;
    if constexpr (PRE) {
      x2 = norms[min(t0 + row, T - 1)];
    } else {
#pragma unroll
      for (int w = 0; w < RT_NW * 4; ++w) x2 += xn[w * RT_TM + row];
    }
    return sqrtf(x2 * w2max);
  };

  if (BF16) {
   if constexpr (!PRE) {
    // ---- fast pass: partial score tiles on the matrix cores ---------------------------------
    const int r = lane & 15;   // token row of the A fragment / expert column of the B fragment
    const int kq = lane >> 4;  // which 8-element group of the 32-wide MFMA step
    const int t_ld = min(t0 + min(r, tpb - 1), T - 1);
    const uint4* xrow = x + static_cast<int64_t>(t_ld) * row16;
    const uint4* wrow[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      wrow[nt] = wg + static_cast<int64_t>(min(nt * 16 + r, E - 1)) * row16;
    f32x4_t acc[NT];                   // score tiles
    RtSumSq x2, w2[NWT];               // this lane's part of |x_t|^2 (token r) and |w_e|^2 (experts 16 i + r)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const int cw = ((row16 + RT_NW * 4 - 1) / (RT_NW * 4)) * 4;  // 16 B chunks per wave
    const int c0 = wave * cw;
    const int c1 = min(row16, c0 + cw);
    // x comes from HBM and is read exactly once: a batch of RT_BATCH MFMA steps has all of its
    // x fragments requested before the first one is used, so each wave keeps 16 KiB in flight.
    // w_gate fragments come from L2 and are fetched per step.
    // (128 and more experts: shorter batches, the score and norm tiles take the registers)
    constexpr int XB = NT >= 16 ? RT_BATCH / 4 : (NT >= 8 ? RT_BATCH / 2 : RT_BATCH);
    for (int cb = c0; cb < c1; cb += 4 * XB) {
      uint4 a[XB];
#pragma unroll
      for (int u = 0; u < XB; ++u) {
        const int cc = cb + 4 * u + kq;
        a[u] = xrow[min(cc, row16 - 1)];
      }
      // w_gate fragments: BSTEPS steps' worth (16 loads) are requested together
      constexpr int BSTEPS = NT >= 16 ? 1 : (NT <= 2 ? 8 : 16 / NT);
#pragma unroll
      for (int u0 = 0; u0 < XB; u0 += BSTEPS) {
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
            rt_sumsq(av, x2);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
              acc[nt] = rt_mfma(av, b[u][nt], acc[nt]);
              // (a chunk past the end of the row repeats the last one: |w_e|^2 comes out a little
              // too large, which an upper bound may)
              rt_sumsq(b[u][nt], w2[nt / WG]);
            }
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
    xn[(wave * 4 + kq) * RT_TM + r] = rt_sumsq_total(x2);
#pragma unroll
    for (int i = 0; i < NWT; ++i) wn[(wave * 4 + kq) * EP + i * 16 + r] = rt_sumsq_total(w2[i]);
    __syncthreads();
   }
    // max_e |w_e|^2 (tile rows past E repeat expert E - 1)
    {
      float m = 0.f;
      if constexpr (PRE) {
        // the same grouping as the fast pass of this kernel would use (WG experts, 16 apart, added up)
        for (int e = lane; e < EP; e += MOE_WAVE) {
          float v = 0.f;
#pragma unroll
          for (int j = 0; j < WG; ++j) v += norms[T + min(((e >> 4) * WG + j) * 16 + (e & 15), E - 1)];
          m = fmaxf(m, v);
        }
      } else {
        for (int e = lane; e < EP; e += MOE_WAVE) {
          float v = 0.f;
#pragma unroll
          for (int w = 0; w < RT_NW * 4; ++w) v += wn[w * EP + e];
          m = fmaxf(m, v);
        }
      }
      w2max = wave_max_dpp(m);
    }
    // ---- routing: tile rows are dealt to the waves ----------------------------------------------
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
      const int row = wave * RPW + rr;
      if (RPW == 1 && row >= tpb) break;
      const int t = t0 + row;
      int amb = 0;
      if (t < T) {
        float s[QE];
        const float bnd = fast_scores(row, s);
        amb = route_token<QE>(s, bnd, true, E, k, renorm, t, cand_all + row * RT_CMAX, topk_idx,
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

// ================================================================================================
// Large-batch bf16 path.  The kernel above gives every 16-token tile a block of its own and lets
// each of its waves fetch its own w_gate fragments: per token that moves E*d/16 elements of w_gate
// through the L2, four times the bytes of x itself at 64 experts, and it spends one wave per token
// on the selection.  Here a block takes TILES tiles (16*TILES tokens) and its eight waves are
// TILES x KS (tile, slice of the hidden dimension); w_gate goes through LDS once per block (a ring
// of 64-element stages filled by direct-to-LDS loads), x goes straight from HBM into MFMA
// fragments.  The partial score tiles meet in LDS and are read back in a layout made for the
// selection: every wave takes 2 TILES of the block's tokens, 64 / (2 TILES) adjacent lanes per
// token, each lane a contiguous range of experts.  A lane finds its best remaining score by a
// tournament over its registers, the lanes of a token merge by DPP butterflies, so one pick
// costs a few dozen instructions for all the wave's tokens together.  Ambiguous tokens follow the
// same protocol as above (exact re-scoring of the listed candidates by the whole block, four
// tokens per pass), after which their lanes patch the scores they hold and select once more.
constexpr int RT_KSEL = 16;      // largest k this path handles (the picks of a tile sit in LDS)

__device__ __forceinline__ int rt_swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <class F, int... I>
__device__ __forceinline__ void rt_unrolled_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void rt_unrolled(F&& f) {
  rt_unrolled_impl(f, std::make_integer_sequence<int, N>{});
}

template <int N> __device__ __forceinline__ void rt_wait_vmcnt() {
  static_assert(N >= 0 && N <= 16, "vmcnt immediate");
#define MOE_RT_VMCNT_CASE(n) \
  if constexpr (N == n) asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory");
  MOE_RT_VMCNT_CASE(0) MOE_RT_VMCNT_CASE(1) MOE_RT_VMCNT_CASE(2) MOE_RT_VMCNT_CASE(3)
  MOE_RT_VMCNT_CASE(4) MOE_RT_VMCNT_CASE(5) MOE_RT_VMCNT_CASE(6) MOE_RT_VMCNT_CASE(7)
  MOE_RT_VMCNT_CASE(8) MOE_RT_VMCNT_CASE(9) MOE_RT_VMCNT_CASE(10) MOE_RT_VMCNT_CASE(11)
  MOE_RT_VMCNT_CASE(12) MOE_RT_VMCNT_CASE(13) MOE_RT_VMCNT_CASE(14) MOE_RT_VMCNT_CASE(15)
  MOE_RT_VMCNT_CASE(16)
#undef MOE_RT_VMCNT_CASE
}

// Butterfly exchange inside groups of 4, 8 or 16 adjacent lanes by DPP (lane swaps in quads, then
// the half-row and row mirrors): after level l every lane has seen 2^(l+1) lanes of its group.
template <int CTRL> __device__ __forceinline__ float rt_dpp(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), CTRL, 0xF, 0xF, false));
}
template <int CTRL> __device__ __forceinline__ int rt_dpp(int x) {
  return __builtin_amdgcn_update_dpp(x, x, CTRL, 0xF, 0xF, false);
}
#define MOE_RT_GROUP_LEVELS(LPT, STEP)      \
  STEP(0xB1) STEP(0x4E)                     \
  if constexpr ((LPT) >= 8) { STEP(0x141) } \
  if constexpr ((LPT) >= 16) { STEP(0x140) }

template <int LPT> __device__ __forceinline__ float group_sum(float x) {
#define MOE_RT_STEP(c) x += rt_dpp<c>(x);
  MOE_RT_GROUP_LEVELS(LPT, MOE_RT_STEP)
#undef MOE_RT_STEP
  return x;
}
template <int LPT> __device__ __forceinline__ int group_sum(int x) {
#define MOE_RT_STEP(c) x += rt_dpp<c>(x);
  MOE_RT_GROUP_LEVELS(LPT, MOE_RT_STEP)
#undef MOE_RT_STEP
  return x;
}
template <int LPT> __device__ __forceinline__ float group_max(float x) {
#define MOE_RT_STEP(c) x = fmaxf(x, rt_dpp<c>(x));
  MOE_RT_GROUP_LEVELS(LPT, MOE_RT_STEP)
#undef MOE_RT_STEP
  return x;
}

// Selection for the 64 / LPT tokens of a wave.  A token belongs to LPT adjacent lanes; lane j of the
// group holds the scores s[q] of experts j S + q (anything for experts >= E: never looked at).
// picks: this wave's LDS scratch, float pw[RT_KSEL + 1][16] followed by int pe[RT_KSEL + 1][16],
// indexed by the token's number in the wave.  With `check`, a token whose choice is within the fast
// pass's error margin writes nothing; it lists its candidates in cand_row[RT_CMAX] (order
// arbitrary; *ccount_row must be zero) and appends one (row | position << 16) per candidate to
// plist, or, if there are more than RT_CMAX, its row to flist (re-score all experts).
// `commit`: this lane's token exists and writes its outputs (if it is not flagged).
// Every lane of the wave must call this (it exchanges data between lanes).
template <int S, int LPT>
__device__ void select_tile(const float (&s)[S], float bnd, bool check, bool commit, int E, int k,
                            int renorm, int64_t t, int row, float* __restrict__ picks,
                            int* __restrict__ cand_row, int* __restrict__ ccount_row,
                            int* __restrict__ plist, int* __restrict__ pcount,
                            int* __restrict__ flist, int* __restrict__ fcount,
                            int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                            float* __restrict__ scores_out) {
  const int lane = lane_id();
  const int tl = lane / LPT, j = lane % LPT;
  const int e0 = j * S;
  float* pv = picks;
  int* pe = reinterpret_cast<int*>(picks + (RT_KSEL + 1) * 16);
  unsigned taken = 0u;                         // bit q: that expert is picked or does not exist
  float wv[S];                                 // the scores still to pick from (-inf once taken)
#pragma unroll
  for (int q = 0; q < S; ++q) {
    const bool exists = e0 + q < E;
    if (!exists) taken |= 1u << q;
    wv[q] = exists ? s[q] : -INFINITY;
  }
  // softmax over all experts: partial sums per lane, the lanes of a token added as a butterfly
  // (every lane gets the same bits: each level adds the same two numbers on both sides)
  float top = -INFINITY;
#pragma unroll
  for (int q = 0; q < S; ++q) top = fmaxf(top, wv[q]);
  top = group_max<LPT>(top);
  float psum = 0.f;
#pragma unroll
  for (int q = 0; q < S; ++q)
    if (e0 + q < E) psum += expf(s[q] - top);
  const float denom = group_sum<LPT>(psum);
  float ws = 0.f;                              // sum of the chosen experts' probabilities
  const int npick = E > k ? k + 1 : k;
  float prev = INFINITY, gap_prev = INFINITY;
  bool amb = false;
  for (int i = 0; i < npick; ++i) {
    // best remaining score of this lane by a tournament: the right entry wins only if strictly
    // greater, so equal scores keep the lowest index
    float tv[S];
    int tq[S];
#pragma unroll
    for (int q = 0; q < S; ++q) {
      tv[q] = wv[q];
      tq[q] = q;
    }
#pragma unroll
    for (int w = 1; w < S; w <<= 1)
#pragma unroll
      for (int m = 0; m + w < S; m += 2 * w) {
        const bool r = tv[m + w] > tv[m];
        tv[m] = r ? tv[m + w] : tv[m];
        tq[m] = r ? tq[m + w] : tq[m];
      }
    float bv = tv[0];
    int be = e0 + tq[0];
    if ((taken >> tq[0]) & 1u) {
      // nothing is left in this lane, or only scores of -inf: the first free entry, if any
      be = 0x7FFFFFFF;
#pragma unroll
      for (int q = S - 1; q >= 0; --q)
        if (!((taken >> q) & 1u)) be = e0 + q;
    }
    // merge over the lanes of the token: larger score, then lower index ("nothing" is
    // (-inf, INT_MAX) and loses against everything)
#define MOE_RT_STEP(c)                                              \
  {                                                                 \
    const float ov = rt_dpp<c>(bv);                                 \
    const int oe = rt_dpp<c>(be);                                   \
    const bool take = ov > bv || (ov == bv && oe < be);             \
    bv = take ? ov : bv;                                            \
    be = take ? oe : be;                                            \
  }
    MOE_RT_GROUP_LEVELS(LPT, MOE_RT_STEP)
#undef MOE_RT_STEP
    {
      const int qs = be - e0;                  // in [0, S) only in the lane that holds the winner
      if (qs >= 0 && qs < S) taken |= 1u << qs;
#pragma unroll
      for (int q = 0; q < S; ++q) wv[q] = q == qs ? -INFINITY : wv[q];
    }
    const float pw = expf(bv - top) / denom;
    if (i < k) ws += pw;
    if (j == 0) {
      pv[i * 16 + tl] = pw;
      pe[i * 16 + tl] = be;
    }
    if (i >= 1) {
      // pick i-1 is a chosen one: its neighbours are picks i-2 and i
      const float gap = prev - bv;
      const float tol = RT_TOL * bnd + 9.5367431640625e-07f * fabsf(prev);
      amb = amb || !(fminf(gap_prev, gap) > tol);
      gap_prev = gap;
    }
    prev = bv;
  }
  if (npick == k) {                            // E == k: the last chosen score has no lower neighbour
    const float tol = RT_TOL * bnd + 9.5367431640625e-07f * fabsf(prev);
    amb = amb || !(gap_prev > tol);
  }
  amb = amb && check;
  // candidates of a flagged token: every expert not clearly below the last pick
  const float margin = 2.0f * (RT_TOL * bnd + 9.5367431640625e-07f * fabsf(prev));
  int n_local = 0;
  if (amb) {
#pragma unroll
    for (int q = 0; q < S; ++q)
      if (e0 + q < E && s[q] >= prev - margin) ++n_local;
  }
  const int n_all = group_sum<LPT>(n_local);
  if (amb && commit) {
    if (n_all <= RT_CMAX) {
#pragma unroll
      for (int q = 0; q < S; ++q)
        if (e0 + q < E && s[q] >= prev - margin) {
          const int pos = atomicAdd(ccount_row, 1);
          cand_row[pos] = e0 + q;
          plist[atomicAdd(pcount, 1)] = row | (pos << 16);
        }
    } else if (j == 0) {
      flist[atomicAdd(fcount, 1)] = row;
    }
  }
  if (amb || !commit) return;
  for (int i = j; i < k; i += LPT) {
    const float p = pv[i * 16 + tl];
    topk_idx[t * k + i] = pe[i * 16 + tl];
    topk_w[t * k + i] = renorm ? p / ws : p;
  }
  if (scores_out) {
#pragma unroll
    for (int q = 0; q < S; ++q)
      if (e0 + q < E) scores_out[t * E + e0 + q] = s[q];
  }
}

// Exact gate sums of up to RT_CMAX (token, candidate expert) pairs, a token of its own per slot.
// pairs[] holds (row | position in the token's candidate list << 16).
// Result: dpart[wave * RT_CMAX + pair].
__device__ void exact_pairs(const uint4* __restrict__ x, const uint4* __restrict__ wg, int row16,
                            int64_t t0, const int* __restrict__ pairs, int npairs,
                            const int* __restrict__ cand_all, int wave, double* __restrict__ dpart) {
  const int lane = lane_id();
  const int c = lane & (RT_CMAX - 1);
  const int entry = pairs[c < npairs ? c : 0];
  const int prow = entry & 0xFFFF, pos = entry >> 16;
  const int e = cand_all[prow * RT_CMAX + pos];
  const double acc = exact_slot_sum<true>(x + (t0 + prow) * row16, wg + static_cast<int64_t>(e) * row16,
                                          row16, wave);
  if (lane < RT_CMAX && c < npairs) dpart[wave * RT_CMAX + c] = acc;
}

template <int NT, int TILES>
struct RouteTileLds {
  static constexpr int KS = RT_NW / TILES;
  static constexpr int ROWS = KS * NT * 16;                 // w_gate rows (expert, slice) per stage
  static constexpr int STAGE = ROWS * 128;
  // stages in the LDS ring (one is being read, the others are in flight): small stages move few
  // bytes each, so they need a deeper ring to keep the same number of bytes on their way from HBM
  static constexpr int NS = STAGE <= 4096 ? 6 : (STAGE <= 8192 ? 4 : (STAGE <= 32768 ? 3 : 2));
  static constexpr int PART = RT_NW * NT * 4 * MOE_WAVE * 4;                // aliases the stages
  static constexpr int RING = NS * STAGE > PART ? NS * STAGE : PART;
  static constexpr int PICKS = RING;                        // float/int [RT_NW][2][RT_KSEL + 1][16]
  static constexpr int CAND = PICKS + RT_NW * 2 * (RT_KSEL + 1) * 16 * 4;   // int [16 TILES][RT_CMAX]
  static constexpr int CCOUNT = CAND + TILES * 16 * RT_CMAX * 4;            // int [16 TILES]
  static constexpr int PLIST = CCOUNT + TILES * 16 * 4;                     // int [16 TILES][RT_CMAX]
  static constexpr int FLIST = PLIST + TILES * 16 * RT_CMAX * 4;            // int [16 TILES] + two counts
  static constexpr int DPART = 0;   // double [RT_NW][max(E, RT_CMAX)]: the exact pass's partial sums also
                                    // alias the stages (nothing there is live once the scores are read back)
  static constexpr int XN = (FLIST + TILES * 16 * 4 + 16 + 15) / 16 * 16;   // float [RT_NW][4][16]: parts of |x_t|^2
  static constexpr int WN = XN + RT_NW * 4 * 16 * 4;                        // float [KS][NT][WNG][16]: parts of |w_e|^2
  static constexpr int WNG = NT >= 16 ? 1 : 4;    // lane groups kept apart (256 experts: no room, added up first)
  static constexpr int TOTAL = WN + KS * NT * WNG * 16 * 4;
  static_assert(RT_NW * (NT * 16 > RT_CMAX ? NT * 16 : RT_CMAX) * 8 <= RING, "exact-pass sums fit the ring");
  static_assert(TOTAL <= 160 * 1024, "LDS of the large-batch routing kernel");
};

// Requires d % (64 KS) == 0 and k <= RT_KSEL (the host checks).
// Four waves per SIMD (two blocks per CU, 128 registers) wherever the LDS use allows two blocks.
template <int NT, int TILES>
__global__ __launch_bounds__(RT_THREADS, (RouteTileLds<NT, TILES>::TOTAL <= 80 * 1024 ? 4 : 2)) void route_tile_kernel(
    const uint4* __restrict__ x, const uint4* __restrict__ wg, const float* __restrict__ bias, int T,
    int d, int E, int k, int renorm, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    float* __restrict__ scores_out) {
  using L = RouteTileLds<NT, TILES>;
  constexpr int KS = L::KS;
  constexpr int QE = NT >= 4 ? NT / 4 : 1;
  constexpr int NLB = (L::ROWS / 8 + RT_NW - 1) / RT_NW;    // w_gate load instructions per wave per stage
  constexpr int NL = NLB + 2;                               // ... plus the two x fragments
  extern __shared__ __align__(1024) unsigned char smem[];
  float* part = reinterpret_cast<float*>(smem);
  int* cand_all = reinterpret_cast<int*>(smem + L::CAND);
  int* ccount = reinterpret_cast<int*>(smem + L::CCOUNT);
  int* plist = reinterpret_cast<int*>(smem + L::PLIST);
  int* flist = reinterpret_cast<int*>(smem + L::FLIST);
  int* fcount = flist + TILES * 16;
  int* pcount = fcount + 1;
  double* dpart = reinterpret_cast<double*>(smem + L::DPART);
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);
  const int ks = wave / TILES, tile = wave % TILES;        // waves 0..TILES-1 (ks = 0) own the tiles
  const int t0 = blockIdx.x * (16 * TILES);
  const int row16 = d / 8;
  const int tok = lane & 15;
  const int kgrp = ((lane >> 4) & 1) * 2 + (lane >> 5);     // which 16-byte chunk of a k-step's four
  const int cs = row16 / KS;                                // chunks per slice, a multiple of 8
  const int KT = cs / 8;                                    // 64-element stages per slice
  if (threadIdx.x == 0) *fcount = *pcount = 0;

  // ---- w_gate -> LDS: instruction j of this wave fills rows 8 i .. 8 i + 7 of the stage, i = (8 j + wave)
  //      modulo the number of row groups (small stages are loaded twice with the same bytes, so
  //      that every wave issues the same number of loads and one wait count serves all).
  //      Stage row r = slice * (16 NT) + expert; experts past E re-read expert E - 1.
  const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint4*>(wg), 0, 0x7FFFFFFF, 0x00020000);
  uint32_t woff[NLB], wlds[NLB];
#pragma unroll
  for (int j = 0; j < NLB; ++j) {
    const int i = (j * RT_NW + wave) % (L::ROWS / 8);
    const int r = i * 8 + (lane >> 3);
    const int e = min(r % (NT * 16), E - 1), sl = r / (NT * 16);
    const int chunk = (lane & 7) ^ rt_swz(r);
    woff[j] = (static_cast<uint32_t>(e) * row16 + sl * cs + chunk) * 16u;
    wlds[j] = i * 1024;
  }
  // ---- x -> registers: lane (tok, kgrp) of k-step j of stage kt holds chunk 8 kt + 4 j + kgrp
  const int t_ld = min(t0 + tile * 16 + tok, T - 1);
  const uint4* xrow = x + static_cast<int64_t>(t_ld) * row16 + ks * cs + kgrp;
  constexpr int NS = L::NS, DIST = NS - 1;
  uint4 a[NS][2];
  auto issue = [&](int kt, auto slot_c) {
    constexpr int SLOT = decltype(slot_c)::value;
#pragma unroll
    for (int j = 0; j < NLB; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rs_w, (__attribute__((address_space(3))) void*)(smem + SLOT * L::STAGE + wlds[j]), 16,
          static_cast<int>(woff[j]), kt * 128, 0, 0);
    a[SLOT][0] = xrow[kt * 8];
    a[SLOT][1] = xrow[kt * 8 + 4];
  };
  // LDS read address of the w_gate fragment: row = own slice, expert 16 nt + lane % 16
  const int f = rt_swz(tok);
  const int wrd = (ks * NT * 16 + tok) * 128;
  int koff[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) koff[j] = ((j * 4 + kgrp) ^ f) << 4;

  // score tiles; this lane's part of |x_t|^2 (token tok) and of |w_e|^2 (experts 16 nt + tok): the
  // TILES waves of a slice see the same w_gate rows, so wave `tile` takes the expert tiles
  // nt = tile, tile + TILES, ...
  constexpr int NWT = (NT + TILES - 1) / TILES;
  f32x4_t acc[NT];
  RtSumSq x2p, w2p[NWT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  using std::integral_constant;
  // prologue: the first DIST stages; then stage kt waits for its own loads (up to DIST - 1 later
  // stages may still be in flight), and, after the barrier that also frees the slot of stage
  // kt - 1, sends the loads of stage kt + DIST into that slot
  rt_unrolled<DIST>([&](auto ic) {
    if (decltype(ic)::value < KT) issue(decltype(ic)::value, ic);
  });
  auto stage = [&](int kt, auto slot_c) {
    constexpr int SLOT = decltype(slot_c)::value;
    const int later = min(DIST - 1, KT - 1 - kt);          // wave-uniform
    rt_unrolled<DIST>([&](auto ic) {
      if (later == decltype(ic)::value) rt_wait_vmcnt<decltype(ic)::value * NL>();
    });
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (kt + DIST < KT) issue(kt + DIST, integral_constant<int, (SLOT + DIST) % NS>{});
    const unsigned char* sb = smem + SLOT * L::STAGE + wrd;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const bf16x8_t xf = __builtin_bit_cast(bf16x8_t, a[SLOT][j]);
      rt_sumsq(a[SLOT][j], x2p);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const bf16x8_t wf = *reinterpret_cast<const bf16x8_t*>(sb + nt * 16 * 128 + koff[j]);
        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xf, acc[nt], 0, 0, 0);
        if (nt % TILES == tile)          // wave-uniform
          rt_sumsq(__builtin_bit_cast(uint4, wf), w2p[nt / TILES]);
      }
    }
  };
  for (int kt = 0; kt < KT; kt += NS) {
    rt_unrolled<NS>([&](auto ic) {
      if (kt + decltype(ic)::value < KT) stage(kt + decltype(ic)::value, ic);
    });
  }

  // ---- the partial score tiles go through LDS and come back in the selection layout: wave
  //      (ks, tile) takes tokens ks TPW .. ks TPW + TPW - 1 of its tile, LPT adjacent lanes per token,
  //      lane j of a token the experts j S .. j S + S - 1; slices are added in slice order.
  constexpr int LPT = 4 * KS, TPW = 16 / KS, S = 4 * NT / KS;
  static_assert(S >= 1 && S * LPT == 16 * NT && TPW * LPT == MOE_WAVE, "selection layout");
  __syncthreads();                      // the ring is no longer read
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int v = 0; v < 4; ++v) part[((wave * NT + nt) * 4 + v) * MOE_WAVE + lane] = acc[nt][v];
  float* xn = reinterpret_cast<float*>(smem + L::XN);
  float* wn = reinterpret_cast<float*>(smem + L::WN);
  xn[wave * 64 + lane] = rt_sumsq_total(x2p);   // (lane = lane group * 16 + tok)
#pragma unroll
  for (int i = 0; i < NWT; ++i) {
    const int nt = i * TILES + tile;
    if constexpr (L::WNG == 4) {
      if (nt < NT) wn[(ks * NT + nt) * 64 + lane] = rt_sumsq_total(w2p[i]);
    } else {
      float v = rt_sumsq_total(w2p[i]);
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      if (nt < NT && lane < 16) wn[(ks * NT + nt) * 16 + tok] = v;
    }
  }
  for (int i = threadIdx.x; i < TILES * 16; i += RT_THREADS) ccount[i] = 0;
  __syncthreads();
  const int tl = lane / LPT, j = lane % LPT;
  const int trow = ks * TPW + tl;                           // token's row in its tile
  const int row = tile * 16 + trow;                         // ... and in the block
  const int64_t t = t0 + row;
  const bool t_ok = t < T;
  float s[S];
#pragma unroll
  for (int q = 0; q < S; ++q) {
    const int e = j * S + q;
    const int at = (((e >> 4) * 4 + (e & 3)) * MOE_WAVE) + ((e >> 2) & 3) * 16 + trow;
    float sum = 0.f;
#pragma unroll
    for (int sl = 0; sl < KS; ++sl) sum += part[(sl * TILES + tile) * NT * 4 * MOE_WAVE + at];
    if (e < E && bias) sum += bias[e];
    s[q] = sum;
  }
  // |x_t| * max_e |w_e| (stage rows past E repeat expert E - 1)
  float w2 = 0.f, x2 = 0.f;
  for (int e = lane; e < NT * 16; e += MOE_WAVE) {
    float v = 0.f;
#pragma unroll
    for (int sl = 0; sl < KS; ++sl)
#pragma unroll
      for (int g = 0; g < L::WNG; ++g) v += wn[((sl * NT + (e >> 4)) * L::WNG + g) * 16 + (e & 15)];
    w2 = fmaxf(w2, v);
  }
  w2 = wave_max_dpp(w2);
#pragma unroll
  for (int sl = 0; sl < KS; ++sl)
#pragma unroll
    for (int g = 0; g < 4; ++g) x2 += xn[((sl * TILES + tile) * 4 + g) * 16 + trow];
  const float bnd = sqrtf(x2 * w2);
  float* picks = reinterpret_cast<float*>(smem + L::PICKS) + wave * 2 * (RT_KSEL + 1) * 16;
  select_tile<S, LPT>(s, bnd, true, t_ok, E, k, renorm, t, row, picks, cand_all + row * RT_CMAX,
                      ccount + row, plist, pcount, flist, fcount, topk_idx, topk_w, scores_out);
  __syncthreads();
  // ---- exact pass for the flagged tokens (block-uniform control flow) ----------------------------
  bool redo = false;                    // this lane's token was flagged
  const int np = *pcount;
  for (int base = 0; base < np; base += RT_CMAX) {
    // up to RT_CMAX (token, candidate) pairs share one pass over the hidden dimension
    const int cnt = min(RT_CMAX, np - base);
    exact_pairs(x, wg, row16, t0, plist + base, cnt, cand_all, wave, dpart);
    __syncthreads();
    for (int c = 0; c < cnt; ++c) {
      const int prow = plist[base + c] & 0xFFFF;
      if (prow == row) {
        // the lanes of the token replace the score they hold by the exact one (fp64 sum of the
        // eight slices in wave order, rounded once)
        redo = true;
        const int e = cand_all[prow * RT_CMAX + (plist[base + c] >> 16)];
        double v64 = 0.0;
#pragma unroll
        for (int w = 0; w < RT_NW; ++w) v64 += dpart[w * RT_CMAX + c];
        if (bias) v64 += static_cast<double>(bias[e]);
#pragma unroll
        for (int q = 0; q < S; ++q)
          if (j * S + q == e) s[q] = static_cast<float>(v64);
      }
    }
    __syncthreads();
  }
  const int nf = *fcount;
  for (int fi = 0; fi < nf; ++fi) {
    // too many candidates: all experts of this one token
    const int frow = flist[fi];
    exact_partial<true, QE>(x + static_cast<int64_t>(t0 + frow) * row16, wg, row16, E, wave, dpart);
    __syncthreads();
    if (frow == row) {
      redo = true;
#pragma unroll
      for (int q = 0; q < S; ++q) {
        const int e = j * S + q;
        if (e < E) {
          double v64 = 0.0;
#pragma unroll
          for (int w = 0; w < RT_NW; ++w) v64 += dpart[w * E + e];
          if (bias) v64 += static_cast<double>(bias[e]);
          s[q] = static_cast<float>(v64);
        }
      }
    }
    __syncthreads();
  }
  if (__ballot(redo) != 0ull)
    select_tile<S, LPT>(s, 0.f, false, redo, E, k, renorm, t, row, picks, nullptr, nullptr, nullptr,
                        nullptr, nullptr, nullptr, topk_idx, topk_w, scores_out);
}

// ================================================================================================
// Small batches with a large gate matrix.  A block of route_kernel pulls the whole w_gate through
// one CU, and a CU alone gets about 35 GB/s out of a cold L2 (two microseconds of latency on every
// batch of loads): 30 us for the 1 MB gate of a 128-expert layer, however few tokens there are.
// With a score buffer from the caller the gate product is spread over the chip instead: a block of
// gate_tile_kernel computes the fast scores of one 16-token x 16-expert tile (same arithmetic and
// summation order as route_kernel's fast pass, so the same bits) and writes them to the buffer;
// route_kernel<.., PRE> then selects from the buffer and runs the exact pass.
constexpr int RT_PRE_MAX_T = MOE_ROUTE_WS_MAX_T;

// GNT: 16-expert tiles per block (1 for the smallest batches, 4 once there are enough token tiles
// to fill the chip: x is then read E / 64 times instead of E / 16 times).
constexpr int GT_BATCH = 8;   // MFMA steps whose fragments (x and up to four w_gate tiles) are requested together
template <int GNT>
__global__ __launch_bounds__(RT_THREADS) void gate_tile_kernel(
    const uint4* __restrict__ x, const uint4* __restrict__ wg, const float* __restrict__ bias, int T,
    int d, int E, float* __restrict__ scores, float* __restrict__ norms) {
  __shared__ float part[RT_NW][RT_TM][16 * GNT];
  __shared__ float xn[RT_NW * 4][RT_TM], wn[RT_NW * 4][16 * GNT];
  const int lane = lane_id();
  const int wave = threadIdx.x / MOE_WAVE;
  const int t0 = blockIdx.x * RT_TM, e0 = blockIdx.y * (16 * GNT);
  const int row16 = d / 8;
  const int r = lane & 15;   // token row of the A fragment / expert column of the B fragment
  const int kq = lane >> 4;  // which 8-element group of the 32-wide MFMA step
  const uint4* xrow = x + static_cast<int64_t>(min(t0 + r, T - 1)) * row16;
  const uint4* wrow[GNT];
  f32x4_t acc[GNT];
  RtSumSq x2, w2[GNT];
#pragma unroll
  for (int nt = 0; nt < GNT; ++nt) {
    wrow[nt] = wg + static_cast<int64_t>(min(e0 + nt * 16 + r, E - 1)) * row16;
    acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
  const int cw = ((row16 + RT_NW * 4 - 1) / (RT_NW * 4)) * 4;  // 16 B chunks per wave
  const int c0 = wave * cw;
  const int c1 = min(row16, c0 + cw);
  for (int cb = c0; cb < c1; cb += 4 * GT_BATCH) {
    uint4 a[GT_BATCH], b[GT_BATCH][GNT];
#pragma unroll
    for (int u = 0; u < GT_BATCH; ++u) {
      const int cc = min(cb + 4 * u + kq, row16 - 1);
      a[u] = xrow[cc];
#pragma unroll
      for (int nt = 0; nt < GNT; ++nt) b[u][nt] = wrow[nt][cc];
    }
#pragma unroll
    for (int u = 0; u < GT_BATCH; ++u) {
      if (cb + 4 * u < c1) {                         // wave-uniform
        uint4 av = a[u];
        if (cb + 4 * u + kq >= row16) av = make_uint4(0, 0, 0, 0);
        rt_sumsq(av, x2);
#pragma unroll
        for (int nt = 0; nt < GNT; ++nt) {
          acc[nt] = rt_mfma(av, b[u][nt], acc[nt]);
          rt_sumsq(b[u][nt], w2[nt]);                       // (past the end: see route_kernel)
        }
      }
    }
  }
  // D layout: lane holds expert column (lane & 15), token rows 4 * (lane >> 4) + v
#pragma unroll
  for (int nt = 0; nt < GNT; ++nt)
#pragma unroll
    for (int v = 0; v < 4; ++v) part[wave][4 * kq + v][nt * 16 + r] = acc[nt][v];
  xn[wave * 4 + kq][r] = rt_sumsq_total(x2);
#pragma unroll
  for (int nt = 0; nt < GNT; ++nt) wn[wave * 4 + kq][nt * 16 + r] = rt_sumsq_total(w2[nt]);
  __syncthreads();
  // |x_t|^2 from the blocks of the first expert tile, |w_e|^2 from those of the first token tile
  {
    const int i = static_cast<int>(threadIdx.x);
    if (blockIdx.y == 0 && i < RT_TM && t0 + i < T) {
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < RT_NW * 4; ++w) v += xn[w][i];
      norms[t0 + i] = v;
    }
    const int ee = i - MOE_WAVE;
    if (blockIdx.x == 0 && ee >= 0 && ee < 16 * GNT && e0 + ee < E) {
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < RT_NW * 4; ++w) v += wn[w][ee];
      norms[T + e0 + ee] = v;
    }
  }
  for (int i = static_cast<int>(threadIdx.x); i < RT_TM * 16 * GNT; i += RT_THREADS) {
    const int row = i / (16 * GNT), ee = i % (16 * GNT);
    const int64_t t = t0 + row;
    const int e = e0 + ee;
    if (t < T && e < E) {
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < RT_NW; ++w) v += part[w][row][ee];
      if (bias) v += bias[e];
      scores[t * E + e] = v;
    }
  }
}

static size_t route_lds_bytes(int E) {
  const size_t dn = E > RT_CMAX ? E : RT_CMAX;
  size_t ep = 16;                      // entries of a |w_e|^2 row in the kernel that serves E experts:
  while (ep < static_cast<size_t>(E)) ep <<= 1;   // 16 NT, or 4 NT from 128 experts on (grouped)
  if (ep >= 128) ep /= 4;
  return static_cast<size_t>(RT_NW) * RT_TM * E * 4 + RT_NW * dn * 8 +
         RT_TM * RT_CMAX * sizeof(int) + RT_TM * sizeof(int) + RT_NW * 4 * (RT_TM + ep) * sizeof(float);
}

template <bool BF16, int NT, int RPW, bool PRE>
static int launch_route_rpw(const moe_shape_t* s, const void* x, const void* wg, const float* bias,
                            int32_t* idx, float* w, const float* scores_in, const float* norms,
                            float* scores, int tpb, hipStream_t st) {
  static LdsOnce once;
  if (ensure_dynamic_lds(once, reinterpret_cast<const void*>(route_kernel<BF16, NT, RPW, PRE>),
                         static_cast<int>(route_lds_bytes(MOE_MAX_E))) != MOE_OK)
    return MOE_ERR_HIP;
  const int grid = (s->T + tpb - 1) / tpb;
  hipLaunchKernelGGL((route_kernel<BF16, NT, RPW, PRE>), dim3(grid), dim3(RT_THREADS),
                     route_lds_bytes(s->E), st, static_cast<const uint4*>(x),
                     static_cast<const uint4*>(wg), bias, s->T, s->d, s->E, s->k, s->renorm, tpb,
                     scores_in, norms, idx, w, scores);
  return launch_status();
}

// scratch: T x E floats the call may use between its kernels (the caller's score output or its
// workspace), or null; norms: T + E floats of the workspace for |x_t|^2 and |w_e|^2, or null.
template <bool BF16, int NT>
static int launch_route(const moe_shape_t* s, const void* x, const void* wg, const float* bias,
                        int32_t* idx, float* w, float* scores, float* scratch, float* norms,
                        hipStream_t st) {
  // Tokens per block: a full 16-row tile when that still gives every CU a block (every wave then
  // has its whole slice of the tile's rows, 16 KiB at d = 4096, requested at once); fewer (the other
  // tile rows idle) for smaller batches, where latency, not MFMA use, is what counts.
  // (Measured at T = 4096, d = 4096, E = 8 with x cold: 25.7 us with 8 tokens per block and
  // batches of 8 steps, 21.8 us with full tiles and the slice in one batch.)
  constexpr int GRID_TARGET = 256;
  int tpb = RT_TM;
  while (tpb > 1 && (s->T + tpb - 1) / tpb < GRID_TARGET) tpb >>= 1;
  if (tpb == RT_TM)
    return launch_route_rpw<BF16, NT, 2, false>(s, x, wg, bias, idx, w, nullptr, nullptr, scores, tpb, st);
  if constexpr (BF16) {
    // gate product spread over the chip first, if there is somewhere to put the scores and the
    // gate matrix is large enough (256 KB: 8 us through one CU) to pay for the second launch
    if (scratch && norms && s->T <= RT_PRE_MAX_T && static_cast<int64_t>(s->E) * s->d * 2 >= 256 * 1024) {
      const int t_tiles = (s->T + RT_TM - 1) / RT_TM;
      if (static_cast<int64_t>(t_tiles) * ((s->E + 63) / 64) >= 256)
        hipLaunchKernelGGL(gate_tile_kernel<4>, dim3(t_tiles, (s->E + 63) / 64), dim3(RT_THREADS), 0, st,
                           static_cast<const uint4*>(x), static_cast<const uint4*>(wg), bias, s->T,
                           s->d, s->E, scratch, norms);
      else
        hipLaunchKernelGGL(gate_tile_kernel<1>, dim3(t_tiles, (s->E + 15) / 16), dim3(RT_THREADS), 0, st,
                           static_cast<const uint4*>(x), static_cast<const uint4*>(wg), bias, s->T,
                           s->d, s->E, scratch, norms);
      if (launch_status() != MOE_OK) return MOE_ERR_HIP;
      return launch_route_rpw<BF16, NT, 1, true>(s, x, wg, bias, idx, w, scratch, norms, scores, tpb, st);
    }
  }
  return launch_route_rpw<BF16, NT, 1, false>(s, x, wg, bias, idx, w, nullptr, nullptr, scores, tpb, st);
}

template <int NT, int TILES>
static int launch_route_tile(const moe_shape_t* s, const void* x, const void* wg, const float* bias,
                             int32_t* idx, float* w, float* scores, hipStream_t st) {
  using L = RouteTileLds<NT, TILES>;
  static LdsOnce once;
  if (ensure_dynamic_lds(once, reinterpret_cast<const void*>(route_tile_kernel<NT, TILES>), L::TOTAL) != MOE_OK)
    return MOE_ERR_HIP;
  const int grid = (s->T + 16 * TILES - 1) / (16 * TILES);
  hipLaunchKernelGGL((route_tile_kernel<NT, TILES>), dim3(grid), dim3(RT_THREADS), L::TOTAL, st,
                     static_cast<const uint4*>(x), static_cast<const uint4*>(wg), bias, s->T, s->d, s->E,
                     s->k, s->renorm, idx, w, scores);
  return launch_status();
}

// The large-batch path takes over when the batch gives enough blocks of at least two tiles (the
// most tiles per block that still give that many blocks; the slices of the hidden dimension must
// be whole 64-element stages) and k and E fit its selection; returns false otherwise.
template <int NT>
static bool try_route_tile(const moe_shape_t* s, const void* x, const void* wg, const float* bias,
                           int32_t* idx, float* w, float* scores, hipStream_t st, int* rc) {
  {
    if (s->k > RT_KSEL) return false;
    // more than 64 experts: at least 4 tiles per block (a stage of 4 slices would not fit the ring);
    // more than 128: exactly 4 (with 8 tiles a lane would hold 64 experts)
    constexpr int TILES_MAX = NT > 8 ? 4 : 8, TILES_MIN = NT > 4 ? 4 : 2;
    auto blocks = [&](int tiles) { return (s->T + 16 * tiles - 1) / (16 * tiles); };
    auto fits = [&](int tiles) { return s->d % (64 * (RT_NW / tiles)) == 0; };
    int tiles = 0;
    const int64_t gate_bytes = static_cast<int64_t>(s->E) * s->d * 2;
    if (gate_bytes <= 128 * 1024) {
      // A small gate matrix costs little to stream once per block: the fewest tiles per block that
      // give every CU a block.  More, shorter blocks than the chip holds at once are in different
      // phases (loading, selecting, storing), so the loads of one overlap the selection of another;
      // with one resident wave of long blocks all load, then all select.  (Measured at d = 4096,
      // E = 8: 65536 tokens 121 us with 8 tiles per block, 112 with 4, 102 with 2; 32768 tokens
      // 70 -> 57 us; E = 16: 121 / 113 / 109 us.  At E = 16, d = 5120, where the matrix is 160 KB,
      // and at E = 64 the order is the opposite: 127 / 135 / 141 us and 92 / 91 / 149 us.)
      for (int c = TILES_MIN; c <= TILES_MAX && tiles == 0; c <<= 1)
        if (blocks(c) >= 256 && fits(c)) tiles = c;
    }
    // otherwise the most tiles per block that still give every CU a block ...
    for (int c = TILES_MAX; c >= TILES_MIN && tiles == 0; c >>= 1)
      if (blocks(c) >= 256 && fits(c)) tiles = c;
    // ... or the fewest tiles per block from 96 blocks on, from where this path measured faster than
    // the per-tile kernel (which streams the whole gate matrix for every 16 tokens, and whose blocks
    // all load, then all select): d = 4096, E = 8, 3072 / 4096 / 6144 tokens 17.6 / 14.2 / 25.1 us
    // -> 13.1 / 13.4 / 14.6 us; E = 16 at 4096 tokens 21 -> 19 us
    if (tiles == 0 && blocks(TILES_MIN) >= 96 && fits(TILES_MIN))
      tiles = TILES_MIN;
    if (tiles == 0) return false;
    if constexpr (NT <= 8) {
      if (tiles == 8) *rc = launch_route_tile<NT, 8>(s, x, wg, bias, idx, w, scores, st);
    }
    if constexpr (NT <= 4) {
      if (tiles == 2) *rc = launch_route_tile<NT, 2>(s, x, wg, bias, idx, w, scores, st);
    }
    if (tiles == 4) *rc = launch_route_tile<NT, 4>(s, x, wg, bias, idx, w, scores, st);
    return true;
  }
}

template <int NT>
static int launch_route_bf16(const moe_shape_t* s, const void* x, const void* wg, const float* bias,
                             int32_t* idx, float* w, float* scores, float* scratch, float* norms,
                             hipStream_t st) {
  int rc = MOE_OK;
  if (try_route_tile<NT>(s, x, wg, bias, idx, w, scores, st, &rc)) return rc;
  return launch_route<true, NT>(s, x, wg, bias, idx, w, scores, scratch, norms, st);
}

}  // namespace moe

static int route_impl(const moe_shape_t* shape, const void* x, const void* w_gate,
                      const float* gate_bias, int32_t* topk_idx, float* topk_w, float* scores_out,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int rc = moe::check_shape(shape);
  if (rc != MOE_OK) return rc;
  if (shape->T == 0) return MOE_OK;
  if (!x || !w_gate || !topk_idx || !topk_w) return MOE_ERR_INVALID_ARG;
  if (!moe::aligned16(x) || !moe::aligned16(w_gate)) return MOE_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int E = shape->E;
  // somewhere to keep T x E fast scores between two kernels: the caller's score output, else its
  // workspace if that is large enough; and T + E floats of the workspace for the norms
  float* scratch = scores_out;
  float* norms = nullptr;
  const size_t score_bytes = static_cast<size_t>(shape->T) * E * sizeof(float);
  const size_t norm_bytes = (static_cast<size_t>(shape->T) + E) * sizeof(float);
  if (workspace && moe::aligned16(workspace)) {
    if (scratch) {
      if (workspace_bytes >= norm_bytes) norms = static_cast<float*>(workspace);
    } else if (workspace_bytes >= score_bytes + norm_bytes) {
      scratch = static_cast<float*>(workspace);
      norms = scratch + static_cast<size_t>(shape->T) * E;
    }
  }
  if (shape->dtype == MOE_BF16) {
    if (E <= 16) return moe::launch_route_bf16<1>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, scratch, norms, st);
    if (E <= 32) return moe::launch_route_bf16<2>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, scratch, norms, st);
    if (E <= 64) return moe::launch_route_bf16<4>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, scratch, norms, st);
    if (E <= 128) return moe::launch_route_bf16<8>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, scratch, norms, st);
    return moe::launch_route_bf16<16>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, scratch, norms, st);
  }
  if (E <= 64) return moe::launch_route<false, 4>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, nullptr, nullptr, st);
  if (E <= 128) return moe::launch_route<false, 8>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, nullptr, nullptr, st);
  return moe::launch_route<false, 16>(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, nullptr, nullptr, st);
}

extern "C" int moe_route(const moe_shape_t* shape, const void* x, const void* w_gate,
                         const float* gate_bias, int32_t* topk_idx, float* topk_w,
                         float* scores_out, void* hip_stream) {
  return route_impl(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, nullptr, 0, hip_stream);
}

extern "C" int moe_route_ws(const moe_shape_t* shape, const void* x, const void* w_gate,
                            const float* gate_bias, int32_t* topk_idx, float* topk_w,
                            float* scores_out, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
  return route_impl(shape, x, w_gate, gate_bias, topk_idx, topk_w, scores_out, workspace,
                    workspace_bytes, hip_stream);
}
