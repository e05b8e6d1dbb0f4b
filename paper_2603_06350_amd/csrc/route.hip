// moe_route: gate product, softmax and top-k routing (Section 2.2: the gating
// network routes each token to its experts; the gate is a bias-free d x E linear
// map, Sections 5 and 6.6).
//
// One block = 16 tokens, 8 waves.  The waves split the hidden dimension; each
// runs v_mfma_f32_16x16x32_bf16 on its slice straight from global memory (x is
// read exactly once from HBM, 16 B per lane; w_gate is small and stays in L2), the
// eight partial score tiles meet in LDS and are summed in a fixed order, so the
// scores are deterministic.  Each wave then routes two tokens with a
// cross-lane butterfly arg-max (value descending, expert index ascending), k+1
// times, and derives the softmax weights from the same scores.
//
// The integer choice must not depend on the order of an fp32 sum.  After the fast
// pass a token is "ambiguous" if two neighbours among its leading k+1 scores are
// closer than 2^-14 * max|logit| (plus a few ulps of the scores themselves).
// Such tokens (about 1% for 64 experts, ~0.03% for 8) are re-evaluated by the
// whole block with exact products and fp64 sums, rounded once to fp32, which is the
// correctly rounded score up to fp64 rounding; fp32 inputs always take this path.
#include "moe_internal.h"

namespace moe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

constexpr int RT_TM = 16;
constexpr int RT_NW = 8;
constexpr int RT_THREADS = RT_NW * MOE_WAVE;

__device__ __forceinline__ void wave_argmax(float& v, int& i) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(v, off);
    const int oi = __shfl_xor(i, off);
    if (ov > v || (ov == v && oi < i)) {
      v = ov;
      i = oi;
    }
  }
}
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

// Routes one token with a full wave.  s[q] is the score of expert lane + 64 q.
// With `check`, returns true (and writes nothing) if the order of the leading k+1
// scores is not safely decided at the fast pass's accuracy.
template <int QE>
__device__ bool route_token(const float (&s)[QE], float lmax, bool check, int E, int k, int renorm,
                            int64_t t, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                            float* __restrict__ scores_out) {
  const int lane = lane_id();
  bool taken[QE];
#pragma unroll
  for (int q = 0; q < QE; ++q) taken[q] = false;
  float sel_v = 0.f;
  int sel_i = 0;
  float next_v = 0.f;  // the (k+1)-th largest score (only when E > k)
  const int npick = (check && E > k) ? k + 1 : k;
  for (int j = 0; j < npick; ++j) {
    float v = -INFINITY;
    int i = 0x7FFFFFFF;
#pragma unroll
    for (int q = 0; q < QE; ++q) {
      const int e = lane + MOE_WAVE * q;
      if (e < E && !taken[q] && (s[q] > v || (s[q] == v && e < i))) {
        v = s[q];
        i = e;
      }
    }
    wave_argmax(v, i);
    if (j < k) {
      if (lane == j) {
        sel_v = v;
        sel_i = i;
      }
    } else {
      next_v = v;
    }
#pragma unroll
    for (int q = 0; q < QE; ++q)
      if (i == lane + MOE_WAVE * q) taken[q] = true;
  }
  if (check) {
    float below = __shfl_down(sel_v, 1);
    if (lane == k - 1) below = next_v;
    const bool has_below = (lane < k - 1) || (lane == k - 1 && E > k);
    const float tol = 6.103515625e-05f * lmax + 4.76837158203125e-07f * fmaxf(fabsf(sel_v), fabsf(below));
    const bool amb = has_below && !(sel_v - below > tol);
    if (__ballot(amb) != 0ull) return true;
  }
  const float m = __shfl(sel_v, 0);
  float p = 0.f;
#pragma unroll
  for (int q = 0; q < QE; ++q)
    if (lane + MOE_WAVE * q < E) p += expf(s[q] - m);
  const float denom = wave_sum(p);
  float w = (lane < k) ? expf(sel_v - m) / denom : 0.f;
  if (renorm) {
    const float ws = wave_sum(w);
    w = w / ws;
  }
  if (lane < k) {
    topk_idx[t * k + lane] = (static_cast<unsigned>(sel_i) < static_cast<unsigned>(E)) ? sel_i : 0;
    topk_w[t * k + lane] = w;
  }
  if (scores_out) {
#pragma unroll
    for (int q = 0; q < QE; ++q)
      if (lane + MOE_WAVE * q < E) scores_out[t * E + lane + MOE_WAVE * q] = s[q];
  }
  return false;
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
    for (int c = c0 + sub; c < c1; c += nsub) {
      const uint4 a = xrow[c];
      const uint4 b = wrow[c];
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
    for (int off = ep; off < MOE_WAVE; off <<= 1) acc += __shfl_xor(acc, off);
    if (sub == 0 && e < E) dpart[wave * E + e] = acc;
  }
}

// Dynamic LDS: float part[RT_NW][RT_TM][E] | double dpart[RT_NW][E] | int flag[RT_TM]
template <bool BF16, int NT>
__global__ __launch_bounds__(RT_THREADS) void route_kernel(
    const uint4* __restrict__ x, const uint4* __restrict__ wg, const float* __restrict__ bias, int T,
    int d, int E, int k, int renorm, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    float* __restrict__ scores_out) {
  constexpr int QE = NT >= 4 ? NT / 4 : 1;
  extern __shared__ __align__(16) unsigned char smem[];
  float* part = reinterpret_cast<float*>(smem);
  double* dpart = reinterpret_cast<double*>(smem + static_cast<size_t>(RT_NW) * RT_TM * E * 4);
  int* flag = reinterpret_cast<int*>(dpart + RT_NW * E);
  const int lane = lane_id();
  const int wave = threadIdx.x / MOE_WAVE;
  const int t0 = blockIdx.x * RT_TM;
  const int row16 = BF16 ? d / 8 : d / 4;

  if (BF16) {
    // ---- fast pass: partial score tiles on the matrix cores ---------------------------------
    const int r = lane & 15;   // token row of the A fragment / expert column of the B fragment
    const int kq = lane >> 4;  // which 8-element group of the 32-wide MFMA step
    const int t_ld = min(t0 + r, T - 1);
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
#pragma unroll 2
    for (int c = c0; c < c1; c += 4) {
      const int cc = c + kq;
      const bool valid = cc < row16;
      const int cl = valid ? cc : row16 - 1;
      uint4 a = xrow[cl];
      if (!valid) a = make_uint4(0, 0, 0, 0);
      uint4 b[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) b[nt] = wrow[nt][cl];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                          __builtin_bit_cast(bf16x8_t, b[nt]),
                                                          acc[nt], 0, 0, 0);
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
    // ---- routing of two tokens per wave ----------------------------------------------------
    for (int rr = 0; rr < RT_TM / RT_NW; ++rr) {
      const int row = wave * (RT_TM / RT_NW) + rr;
      const int t = t0 + row;
      bool amb = false;
      if (t < T) {
        float s[QE];
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
        const float lmax = wave_max(la);
        amb = route_token<QE>(s, lmax, true, E, k, renorm, t, topk_idx, topk_w, scores_out);
      }
      if (lane == 0) flag[row] = amb ? 1 : 0;
    }
  } else {
    if (threadIdx.x < RT_TM) flag[threadIdx.x] = (t0 + threadIdx.x < T) ? 1 : 0;
  }
  __syncthreads();
  // ---- exact pass for the tokens that need it (block-uniform control flow) -------------------
  for (int row = 0; row < RT_TM; ++row) {
    if (!flag[row]) continue;
    const int t = t0 + row;
    exact_partial<BF16, QE>(x + static_cast<int64_t>(t) * row16, wg, row16, E, wave, dpart);
    __syncthreads();
    if (wave == (row % RT_NW)) {
      float s[QE];
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
      route_token<QE>(s, 0.f, false, E, k, renorm, t, topk_idx, topk_w, scores_out);
    }
    __syncthreads();
  }
}

static size_t route_lds_bytes(int E) {
  return static_cast<size_t>(RT_NW) * RT_TM * E * 4 + static_cast<size_t>(RT_NW) * E * 8 +
         RT_TM * sizeof(int);
}

template <bool BF16, int NT>
static int launch_route(const moe_shape_t* s, const void* x, const void* wg, const float* bias,
                        int32_t* idx, float* w, float* scores, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(route_kernel<BF16, NT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            static_cast<int>(route_lds_bytes(MOE_MAX_E))) != hipSuccess)
      return MOE_ERR_HIP;
    attr_set = true;
  }
  const int grid = (s->T + RT_TM - 1) / RT_TM;
  hipLaunchKernelGGL((route_kernel<BF16, NT>), dim3(grid), dim3(RT_THREADS), route_lds_bytes(s->E),
                     st, static_cast<const uint4*>(x), static_cast<const uint4*>(wg), bias, s->T,
                     s->d, s->E, s->k, s->renorm, idx, w, scores);
  return launch_status();
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
