// Consumers of the expert-load statistic (Sections 3.3 and 4.2, Algorithm 1): the coefficient of
// variation of a layer's per-replica loads, the greedy Expert Scaling heuristic, and the even cut
// of each expert's row segment into its replicas' pieces.
//
// Algorithm 1 adds one replica per step to the expert whose replicas carry the largest load, until
// the CV of the per-replica loads is at most V or no further replica fits into the layer's memory
// cap.  The steps depend on each other, E is at most 256 and the data fits in registers, so ONE
// wave runs the whole loop: a lane owns experts lane, lane+64, ...; the straggler comes from a
// wave-wide arg-max (the paper's text uses a max-heap on the host; 64 lanes comparing at once
// replace it), CV from a wave-wide fp64 sum in a fixed order.  Per-replica loads W_e / R_e are
// compared exactly, as W_a * R_b > W_b * R_a in 64-bit integers; equal loads go to the lowest expert
// index.  No host synchronisation: loads in, replica counts out, both on the device, so the counts
// that `moe_count_and_permute` (or a predictor's routing pass) has just produced can be consumed
// on the same stream.
#include "moe_internal.h"

namespace moe {

constexpr int SC_Q = MOE_MAX_E / MOE_WAVE;   // experts per lane

struct Straggler {
  long long w;   // load of the expert
  int r;         // its replica count
  int e;         // its index (E = none)
};

// a carries a strictly larger per-replica load than b, or the same load and a lower index
__device__ __forceinline__ bool heavier(const Straggler& a, const Straggler& b) {
  const long long lhs = a.w * b.r, rhs = b.w * a.r;
  return lhs > rhs || (lhs == rhs && a.e < b.e);
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

__global__ __launch_bounds__(MOE_WAVE) void scale_kernel(const int32_t* __restrict__ loads, int E,
                                                         int max_extra, double cv_threshold,
                                                         int32_t* __restrict__ replicas,
                                                         double* __restrict__ cv_out) {
  const int lane = lane_id();
  long long w[SC_Q];
  int r[SC_Q];
  long long s1_lane = 0;
#pragma unroll
  for (int q = 0; q < SC_Q; ++q) {
    const int e = lane + MOE_WAVE * q;
    w[q] = e < E ? max(loads[e], 0) : 0;
    r[q] = 1;
    s1_lane += w[q];
  }
  long long s1 = s1_lane;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s1 += __shfl_xor(s1, off);
  int n = E;                                   // replicas in the layer
  int extra = 0;
  double cv = 0.0, cv_first = 0.0;
  for (;;) {
    // CV of the multiset {W_e / R_e, R_e times}: population std / mean
    if (s1 > 0) {
      const double mean = static_cast<double>(s1) / static_cast<double>(n);
      double part = 0.0;
#pragma unroll
      for (int q = 0; q < SC_Q; ++q) {
        if (lane + MOE_WAVE * q < E) {
          const double dv = static_cast<double>(w[q]) / static_cast<double>(r[q]) - mean;
          part += static_cast<double>(r[q]) * dv * dv;
        }
      }
      cv = sqrt(wave_sum_f64(part) / static_cast<double>(n)) / mean;
    } else {
      cv = 0.0;
    }
    if (extra == 0) cv_first = cv;
    if (extra >= max_extra || !(cv > cv_threshold)) break;     // wave-uniform
    // the straggler
    Straggler best{0, 1, E};
#pragma unroll
    for (int q = 0; q < SC_Q; ++q) {
      const int e = lane + MOE_WAVE * q;
      const Straggler c{w[q], r[q], e};
      if (e < E && heavier(c, best)) best = c;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      Straggler o;
      o.w = __shfl_xor(best.w, off);
      o.r = __shfl_xor(best.r, off);
      o.e = __shfl_xor(best.e, off);
      if (heavier(o, best)) best = o;
    }
    if (best.e >= E || best.w == 0) break;     // nothing to split
#pragma unroll
    for (int q = 0; q < SC_Q; ++q)
      if (lane + MOE_WAVE * q == best.e) r[q] += 1;
    n += 1;
    extra += 1;
  }
#pragma unroll
  for (int q = 0; q < SC_Q; ++q) {
    const int e = lane + MOE_WAVE * q;
    if (e < E) replicas[e] = r[q];
  }
  if (cv_out && lane == 0) {
    cv_out[0] = cv_first;
    cv_out[1] = cv;
  }
}

// One block.  prefix[e] = number of segments before expert e; thread s-strided over the segments.
__global__ __launch_bounds__(256) void segments_kernel(const int32_t* __restrict__ offsets,
                                                       const int32_t* __restrict__ replicas, int E,
                                                       int max_segments,
                                                       int32_t* __restrict__ seg_offsets,
                                                       int32_t* __restrict__ seg_expert,
                                                       int32_t* __restrict__ n_segments) {
  __shared__ int prefix[MOE_MAX_E + 1];
  const int tid = threadIdx.x;
  if (tid == 0) {
    int run = 0;
    for (int e = 0; e < E; ++e) {
      prefix[e] = run;
      const int r = max(replicas[e], 1);
      run = (run > 0x7FFFFFFF - r) ? 0x7FFFFFFF : run + r;     // saturate, never wrap
    }
    prefix[E] = run;
    *n_segments = run;
    if (max_segments >= 0) seg_offsets[0] = offsets[0];
  }
  __syncthreads();
  const int total = min(prefix[E], max_segments);
  for (int s = tid; s < total; s += 256) {
    int lo = 0, hi = E - 1;                    // last expert whose prefix is <= s
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (prefix[mid] <= s) lo = mid; else hi = mid - 1;
    }
    const int e = lo;
    const long long R = max(replicas[e], 1);
    const long long c = max(offsets[e + 1] - offsets[e], 0);
    const long long rr = s - prefix[e];
    seg_expert[s] = e;
    seg_offsets[s + 1] = offsets[e] + static_cast<int32_t>((c * (rr + 1)) / R);
  }
}

}  // namespace moe

extern "C" int moe_scale_replicas(int32_t E, const int32_t* loads, int64_t expert_mem,
                                  int64_t mem_cap, double cv_threshold, int32_t* replicas,
                                  double* cv_out, void* hip_stream) {
  if (E < 1 || !loads || !replicas || expert_mem < 1 || mem_cap < 0) return MOE_ERR_INVALID_ARG;
  if (!(cv_threshold == cv_threshold)) return MOE_ERR_INVALID_ARG;   // NaN
  if (E > MOE_MAX_E) return MOE_ERR_UNSUPPORTED;
  const int64_t max_extra = mem_cap / expert_mem;
  if (max_extra > MOE_MAX_EXTRA_REPLICAS) return MOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(moe::scale_kernel, dim3(1), dim3(MOE_WAVE), 0,
                     static_cast<hipStream_t>(hip_stream), loads, E, static_cast<int>(max_extra),
                     cv_threshold, replicas, cv_out);
  return moe::launch_status();
}

extern "C" int moe_replica_segments(int32_t E, const int32_t* offsets, const int32_t* replicas,
                                    int32_t max_segments, int32_t* seg_offsets,
                                    int32_t* seg_expert, int32_t* n_segments, void* hip_stream) {
  if (E < 1 || !offsets || !replicas || !seg_offsets || !seg_expert || !n_segments ||
      max_segments < 0)
    return MOE_ERR_INVALID_ARG;
  if (E > MOE_MAX_E) return MOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(moe::segments_kernel, dim3(1), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), offsets, replicas, E, max_segments,
                     seg_offsets, seg_expert, n_segments);
  return moe::launch_status();
}

// ---------------------------------------------------------------------------------------------
// Expert Placement (Algorithm 2, Section 4.3): replicas from the most to the least loaded; a
// replica that is still alive where the previous round put it stays there, any other joins the
// GPU with the smallest aggregated load.  The steps depend on each other, so again ONE wave runs
// the loop: lane e (+64, ...) owns expert e, lane g owns GPU g's load, count and slots; "most
// loaded replica" is a wave arg-max over the experts that still have replicas to place (all
// replicas of an expert carry W_e / R_e, so they are placed one after the other), "shortest
// queue" a wave arg-min over the GPUs with a free slot.  GPU loads are fp64 sums in placement
// order.
// ---------------------------------------------------------------------------------------------
namespace moe {

constexpr int PL_MAX_GPUS = MOE_WAVE;

__global__ __launch_bounds__(MOE_WAVE) void place_kernel(
    const int32_t* __restrict__ loads, const int32_t* __restrict__ replicas, int E, int G,
    const int32_t* __restrict__ prev_replicas, const int32_t* __restrict__ prev_gpu,
    const int32_t* __restrict__ gpu_slots, int max_segments, int step_budget,
    int32_t* __restrict__ gpu_of, double* __restrict__ gpu_load, int32_t* __restrict__ gpu_count,
    int32_t* __restrict__ n_warm) {
  __shared__ int seg_start[MOE_MAX_E + 1];
  __shared__ int prev_start[MOE_MAX_E + 1];     // the same prefix over the previous round's counts
  const int lane = lane_id();
  long long w[SC_Q];
  int r[SC_Q];
  bool todo[SC_Q];
#pragma unroll
  for (int q = 0; q < SC_Q; ++q) {
    const int e = lane + MOE_WAVE * q;
    w[q] = e < E ? max(loads[e], 0) : 0;
    r[q] = e < E ? min(max(replicas[e], 1), MOE_MAX_EXTRA_REPLICAS + 1) : 1;
    todo[q] = e < E;
  }
  if (lane == 0) {
    int run = 0;
    for (int e = 0; e < E; ++e) {
      seg_start[e] = run;
      const int re = min(max(replicas[e], 1), MOE_MAX_EXTRA_REPLICAS + 1);
      run = (run > 0x7FFFFFFF - re) ? 0x7FFFFFFF : run + re;
    }
    seg_start[E] = run;
    run = 0;
    for (int e = 0; e < E; ++e) {
      prev_start[e] = run;
      const int pe = prev_replicas ? max(prev_replicas[e], 0) : 0;
      run = (run > 0x7FFFFFFF - pe) ? 0x7FFFFFFF : run + pe;
    }
    prev_start[E] = run;
  }
  __syncthreads();
  double gload = 0.0;                          // this lane's GPU
  int gcount = 0;
  const int gslots = (lane < G) ? (gpu_slots ? max(gpu_slots[lane], 0) : 0x7FFFFFFF) : 0;
  int warm = 0, steps = 0;
  for (int it = 0; it < E; ++it) {
    // the expert whose replicas carry the largest load among those not placed yet
    Straggler best{-1, 1, E};
#pragma unroll
    for (int q = 0; q < SC_Q; ++q) {
      const Straggler c{w[q], r[q], lane + MOE_WAVE * q};
      if (todo[q] && (best.e >= E || heavier(c, best))) best = c;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      Straggler o;
      o.w = __shfl_xor(best.w, off);
      o.r = __shfl_xor(best.r, off);
      o.e = __shfl_xor(best.e, off);
      if (o.e < E && (best.e >= E || heavier(o, best))) best = o;
    }
    if (best.e >= E) break;                    // wave-uniform
#pragma unroll
    for (int q = 0; q < SC_Q; ++q)
      if (lane + MOE_WAVE * q == best.e) todo[q] = false;
    const double wv = static_cast<double>(best.w) / static_cast<double>(best.r);
    const int prev_lo = prev_start[best.e];
    const int prev_n = prev_start[best.e + 1] - prev_lo;
    const int out0 = seg_start[best.e];
    for (int q = 0; q < best.r; ++q) {
      if (steps >= step_budget) break;         // wave-uniform
      ++steps;
      const bool has_room = lane < G && gcount < gslots;
      int g = -1;
      if (q < prev_n) {
        const int pg = prev_gpu[prev_lo + q];
        if (pg >= 0 && pg < G && __shfl(has_room ? 1 : 0, pg)) {
          g = pg;
          ++warm;
        }
      }
      if (g < 0) {
        // shortest queue among the GPUs with a free slot; equal loads go to the lowest index
        double bl = gload;
        int bg = has_room ? lane : -1;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
          const double ol = __shfl_xor(bl, off);
          const int og = __shfl_xor(bg, off);
          if (og >= 0 && (bg < 0 || ol < bl || (ol == bl && og < bg))) {
            bl = ol;
            bg = og;
          }
        }
        g = bg;
      }
      if (g >= 0 && lane == g) {
        gload += wv;
        gcount += 1;
      }
      if (lane == 0 && out0 + q < max_segments) gpu_of[out0 + q] = g;
    }
  }
  if (lane < G) {
    gpu_load[lane] = gload;
    gpu_count[lane] = gcount;
  }
  if (lane == 0) *n_warm = warm;
}

}  // namespace moe

extern "C" int moe_place_replicas(int32_t E, const int32_t* loads, const int32_t* replicas,
                                  int32_t n_gpus, const int32_t* prev_replicas,
                                  const int32_t* prev_gpu, const int32_t* gpu_slots,
                                  int32_t max_segments, int32_t* gpu_of, double* gpu_load,
                                  int32_t* gpu_count, int32_t* n_warm, void* hip_stream) {
  if (E < 1 || n_gpus < 1 || !loads || !replicas || !gpu_of || !gpu_load || !gpu_count || !n_warm ||
      max_segments < 0)
    return MOE_ERR_INVALID_ARG;
  if ((prev_replicas == nullptr) != (prev_gpu == nullptr)) return MOE_ERR_INVALID_ARG;
  if (E > MOE_MAX_E || n_gpus > moe::PL_MAX_GPUS) return MOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(moe::place_kernel, dim3(1), dim3(MOE_WAVE), 0,
                     static_cast<hipStream_t>(hip_stream), loads, replicas, E, n_gpus, prev_replicas,
                     prev_gpu, gpu_slots, max_segments, E + MOE_MAX_EXTRA_REPLICAS, gpu_of, gpu_load,
                     gpu_count, n_warm);
  return moe::launch_status();
}
