// moe_count_and_permute: per-expert token counts (the paper's expert load W_l,
// Sections 3.3 / 4.1), their prefix sum, the stable expert-contiguous permutation
// of the T*k assignments and the row gather that realises the single-GPU "scatter"
// of Section 2.2.
//
// Three launches on the caller's stream (two for batches of at most 256 assignments, where
// rank_small_kernel replaces 1 and 2), no host synchronisation:
//   1. hist_kernel   one thread per token; LDS histogram of the block's
//                    assignments -> partial[block][expert]              (integer)
//   2. rank_kernel   same token partition.  Every block sums `partial` to get
//                    counts, offsets and its own base row per expert, then ranks
//                    its assignments with a per-(expert, thread) LDS counter table
//                    and a prefix scan over threads, so the rank of an assignment
//                    is the number of earlier assignments of the same expert: a
//                    stable order, independent of scheduling, no atomics on the
//                    result.
//   3. gather_kernel one wave per token: reads the token row once (16 B per
//                    lane, coalesced), writes it to its k destination rows.
//                    HBM-bound: T*d*b bytes read, T*k*d*b written.
#include <mutex>

#include "moe_internal.h"

namespace moe {

template <int NTH>
__global__ __launch_bounds__(NTH) void hist_kernel(const int32_t* __restrict__ topk_idx, int T,
                                                   int k, int E,
                                                   int32_t* __restrict__ partial) {
  __shared__ int32_t hist[MOE_MAX_E];
  const int tid = threadIdx.x;
  for (int e = tid; e < E; e += NTH) hist[e] = 0;
  __syncthreads();
  const int t = blockIdx.x * NTH + tid;
  if (t < T) {
    const int32_t* row = topk_idx + static_cast<int64_t>(t) * k;
    for (int j = 0; j < k; ++j) {
      const int e = row[j];
      if (static_cast<unsigned>(e) < static_cast<unsigned>(E)) atomicAdd(&hist[e], 1);
    }
  }
  __syncthreads();
  for (int e = tid; e < E; e += NTH) partial[static_cast<int64_t>(blockIdx.x) * E + e] = hist[e];
}

// Dynamic LDS layout: uint16 cnt[E][NTH] | int32 tot[E] | int32 base[E]
template <int NTH>
__global__ __launch_bounds__(NTH) void rank_kernel(const int32_t* __restrict__ topk_idx, int T,
                                                   int k, int E,
                                                   const int32_t* __restrict__ partial, int NB,
                                                   int32_t* __restrict__ counts,
                                                   int32_t* __restrict__ offsets,
                                                   int32_t* __restrict__ dst_row,
                                                   int32_t* __restrict__ src_assign) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* cnt = reinterpret_cast<uint16_t*>(smem);
  int32_t* tot = reinterpret_cast<int32_t*>(smem + static_cast<size_t>(E) * NTH * 2);
  int32_t* base = tot + E;
  constexpr int NW = NTH / MOE_WAVE;
  constexpr int PER = NTH / MOE_WAVE;  // table entries of one row held by one lane
  const int tid = threadIdx.x;
  const int lane = tid & (MOE_WAVE - 1);
  const int wave = tid / MOE_WAVE;
  const int b = blockIdx.x;

  // zero the counter table (16 B per store)
  {
    uint4* z = reinterpret_cast<uint4*>(cnt);
    const int n16 = E * NTH * 2 / 16;
    for (int i = tid; i < n16; i += NTH) z[i] = make_uint4(0, 0, 0, 0);
  }
  // totals per expert and the part that belongs to earlier blocks: every thread takes a strided
  // share of partial[NB][E] (coalesced, several loads in flight) and adds it into LDS; integer
  // sums, so the order of the atomics does not matter
  for (int e = tid; e < E; e += NTH) {
    tot[e] = 0;
    base[e] = 0;
  }
  __syncthreads();
  {
    const int n = NB * E;
    constexpr int UNR = 8;
    for (int i0 = tid; i0 < n; i0 += UNR * NTH) {
      int v[UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int i = i0 + u * NTH;
        v[u] = i < n ? partial[i] : 0;
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int i = i0 + u * NTH;
        if (i < n && v[u] != 0) {
          const int e = i % E, bb = i / E;
          atomicAdd(&tot[e], v[u]);
          if (bb < b) atomicAdd(&base[e], v[u]);
        }
      }
    }
  }
  __syncthreads();
  // exclusive scan of tot over experts by wave 0 (E <= 256: at most 4 per lane)
  if (wave == 0) {
    const int per = (E + MOE_WAVE - 1) / MOE_WAVE;
    const int e0 = lane * per;
    int local = 0;
    for (int i = 0; i < per; ++i)
      if (e0 + i < E) local += tot[e0 + i];
    int incl = local;
    for (int off = 1; off < MOE_WAVE; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    int run = incl - local;
    for (int i = 0; i < per; ++i) {
      const int e = e0 + i;
      if (e < E) {
        const int c = tot[e];
        if (b == 0) {
          counts[e] = c;
          offsets[e] = run;
        }
        base[e] += run;
        run += c;
      }
    }
    if (b == 0 && lane == MOE_WAVE - 1) offsets[E] = incl;
  }
  // count this thread's assignments in its private column of the table
  const int t = b * NTH + tid;
  const int32_t* row = topk_idx + static_cast<int64_t>(t) * k;
  if (t < T) {
    for (int j = 0; j < k; ++j) {
      const int e = row[j];
      if (static_cast<unsigned>(e) < static_cast<unsigned>(E)) cnt[e * NTH + tid] += 1;
    }
  }
  __syncthreads();
  // per expert: exclusive prefix over threads (in place); rows are dealt to waves
  for (int e = wave; e < E; e += NW) {
    uint16_t* r = cnt + e * NTH + lane * PER;
    uint16_t v[PER];
    int local = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      v[i] = r[i];
      local += v[i];
    }
    int incl = local;
#pragma unroll
    for (int off = 1; off < MOE_WAVE; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    int run = incl - local;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      r[i] = static_cast<uint16_t>(run);
      run += v[i];
    }
  }
  __syncthreads();
  if (t < T) {
    for (int j = 0; j < k; ++j) {
      const int e = row[j];
      const int a = t * k + j;
      if (static_cast<unsigned>(e) < static_cast<unsigned>(E)) {
        const int r = cnt[e * NTH + tid];
        cnt[e * NTH + tid] = static_cast<uint16_t>(r + 1);
        const int dst = base[e] + r;
        dst_row[a] = dst;
        src_assign[dst] = a;
      } else {
        dst_row[a] = 0;  // invalid expert index: value unspecified, stays in bounds
      }
    }
  }
}

// Small batches (T*k <= RS_MAX_A): one block does the whole dispatch.  The rank of an assignment
// is counted directly, as the number of earlier assignments of the same expert (all assignments
// sit in LDS and are read as broadcasts), so there is no table to clear or scan and one launch
// replaces two.
// Measured: 8.5 us for 256 assignments against 10.5 - 16 us for the two launches, but 20 us for 384
// and 97 us for 1024 (the count is quadratic), where the two launches still take 11 - 17 us.
constexpr int RS_MAX_A = 256;
__global__ __launch_bounds__(256) void rank_small_kernel(const int32_t* __restrict__ topk_idx, int A,
                                                         int E, int32_t* __restrict__ counts,
                                                         int32_t* __restrict__ offsets,
                                                         int32_t* __restrict__ dst_row,
                                                         int32_t* __restrict__ src_assign) {
  __shared__ __align__(16) int32_t idx[RS_MAX_A];
  __shared__ int32_t cnt[MOE_MAX_E];
  __shared__ int32_t off[MOE_MAX_E + 1];
  const int tid = threadIdx.x;
  const int lane = tid & (MOE_WAVE - 1);
  for (int e = tid; e < E; e += 256) cnt[e] = 0;
  for (int a = tid; a < RS_MAX_A; a += 256) {
    int e = a < A ? topk_idx[a] : -1;
    if (static_cast<unsigned>(e) >= static_cast<unsigned>(E)) e = -1;   // invalid: never matches
    idx[a] = e;
  }
  __syncthreads();
  for (int a = tid; a < A; a += 256)
    if (idx[a] >= 0) atomicAdd(&cnt[idx[a]], 1);
  __syncthreads();
  if (tid < MOE_WAVE) {                         // exclusive scan over experts by wave 0
    const int per = (E + MOE_WAVE - 1) / MOE_WAVE;
    const int e0 = lane * per;
    int local = 0;
    for (int i = 0; i < per; ++i)
      if (e0 + i < E) local += cnt[e0 + i];
    int incl = local;
    for (int o = 1; o < MOE_WAVE; o <<= 1) {
      const int up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    int run = incl - local;
    for (int i = 0; i < per; ++i) {
      const int e = e0 + i;
      if (e < E) {
        off[e] = run;
        counts[e] = cnt[e];
        offsets[e] = run;
        run += cnt[e];
      }
    }
    if (lane == MOE_WAVE - 1) offsets[E] = incl;
  }
  __syncthreads();
  const int a4 = (A + 3) & ~3;
  for (int a = tid; a < A; a += 256) {
    const int e = idx[a];
    if (e < 0) {
      dst_row[a] = 0;                           // invalid expert index: value unspecified, in bounds
      continue;
    }
    int r = 0;
    for (int b0 = 0; b0 < a4; b0 += 4) {
      const int4 v = *reinterpret_cast<const int4*>(idx + b0);
      r += (v.x == e && b0 < a) + (v.y == e && b0 + 1 < a) + (v.z == e && b0 + 2 < a) +
           (v.w == e && b0 + 3 < a);
    }
    const int dst = off[e] + r;
    dst_row[a] = dst;
    src_assign[dst] = a;
  }
}

// One wave per token.  row16 = row size in 16-byte units.
__global__ __launch_bounds__(256) void gather_kernel(const uint4* __restrict__ x,
                                                     const int32_t* __restrict__ dst_row,
                                                     uint4* __restrict__ x_perm, int T, int k,
                                                     int row16, int A) {
  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int t = blockIdx.x * (256 / MOE_WAVE) + threadIdx.x / MOE_WAVE;
  if (t >= T) return;
  int my_dst = 0;
  if (lane < k) my_dst = dst_row[static_cast<int64_t>(t) * k + lane];
  if (static_cast<unsigned>(my_dst) >= static_cast<unsigned>(A)) my_dst = 0;
  const uint4* src = x + static_cast<int64_t>(t) * row16;
  constexpr int UNR = 4;   // 16-byte loads in flight per lane (4 KiB per wave)
  for (int c0 = 0; c0 < row16; c0 += UNR * MOE_WAVE) {
    uint4 v[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int c = c0 + u * MOE_WAVE + lane;
      if (c < row16) v[u] = src[c];
    }
    for (int j = 0; j < k; ++j) {
      const int dst = __shfl(my_dst, j);
      uint4* out = x_perm + static_cast<int64_t>(dst) * row16;
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int c = c0 + u * MOE_WAVE + lane;
        if (c < row16) out[c] = v[u];
      }
    }
  }
}

static int dispatch_threads(int E) { return E <= 128 ? 256 : 128; }

}  // namespace moe

extern "C" int moe_workspace_bytes(const moe_shape_t* shape, size_t* out_bytes) {
  const int rc = moe::check_shape(shape);
  if (rc != MOE_OK) return rc;
  if (!out_bytes) return MOE_ERR_INVALID_ARG;
  const int nth = moe::dispatch_threads(shape->E);
  const int64_t nb = (static_cast<int64_t>(shape->T) + nth - 1) / nth;
  size_t bytes = static_cast<size_t>(nb > 0 ? nb : 1) * shape->E * sizeof(int32_t);
  // moe_route_ws keeps T x E fp32 scores and T + E norms between its two kernels for small batches
  if (shape->T <= MOE_ROUTE_WS_MAX_T) {
    const size_t route_bytes =
        (static_cast<size_t>(shape->T) * shape->E + shape->T + shape->E) * sizeof(float);
    if (route_bytes > bytes) bytes = route_bytes;
  }
  *out_bytes = (bytes + 255) & ~static_cast<size_t>(255);
  return MOE_OK;
}

namespace moe {

// Bytes of partial[blocks][E] that the two-launch dispatch keeps between hist_kernel and rank_kernel.
static size_t dispatch_partial_bytes(const moe_shape_t* shape) {
  const int nth = dispatch_threads(shape->E);
  const int64_t nb = (static_cast<int64_t>(shape->T) + nth - 1) / nth;
  return static_cast<size_t>(nb > 0 ? nb : 1) * shape->E * sizeof(int32_t);
}

// Everything after the checks of the workspace: `partial` holds dispatch_partial_bytes() bytes.
// hist_kernel writes every entry of it that rank_kernel reads, so its old contents do not matter.
static int count_and_permute_impl(const moe_shape_t* shape, const void* x, const int32_t* topk_idx,
                                  int32_t* counts, int32_t* offsets, int32_t* dst_row,
                                  int32_t* src_assign, void* x_perm, int32_t* partial,
                                  hipStream_t st) {
  const int T = shape->T, k = shape->k, E = shape->E;
  const int nth = dispatch_threads(E);
  const int nb = (T + nth - 1) / nth;
  const size_t lds = static_cast<size_t>(E) * nth * 2 + static_cast<size_t>(E) * 8;
  // T == 0 still defines counts = 0 and offsets = 0: one block with no tokens does that.
  const int grid = nb > 0 ? nb : 1;
  if (static_cast<int64_t>(T) * k <= RS_MAX_A) {
    hipLaunchKernelGGL(rank_small_kernel, dim3(1), dim3(256), 0, st, topk_idx, T * k, E, counts,
                       offsets, dst_row, src_assign);
  } else if (nth == 256) {
    static LdsOnce once;
    if (ensure_dynamic_lds(once, reinterpret_cast<const void*>(rank_kernel<256>),
                           128 * 256 * 2 + 128 * 8) != MOE_OK)
      return MOE_ERR_HIP;
    hipLaunchKernelGGL(hist_kernel<256>, dim3(grid), dim3(256), 0, st, topk_idx, T, k, E, partial);
    hipLaunchKernelGGL(rank_kernel<256>, dim3(grid), dim3(256), lds, st, topk_idx, T, k, E, partial,
                       grid, counts, offsets, dst_row, src_assign);
  } else {
    static LdsOnce once;
    if (ensure_dynamic_lds(once, reinterpret_cast<const void*>(rank_kernel<128>),
                           256 * 128 * 2 + 256 * 8) != MOE_OK)
      return MOE_ERR_HIP;
    hipLaunchKernelGGL(hist_kernel<128>, dim3(grid), dim3(128), 0, st, topk_idx, T, k, E, partial);
    hipLaunchKernelGGL(rank_kernel<128>, dim3(grid), dim3(128), lds, st, topk_idx, T, k, E, partial,
                       grid, counts, offsets, dst_row, src_assign);
  }
  if (T > 0 && x_perm) {
    const int row16 = static_cast<int>(static_cast<int64_t>(shape->d) * elem_bytes(shape->dtype) / 16);
    hipLaunchKernelGGL(gather_kernel, dim3((T + 3) / 4), dim3(256), 0, st,
                       static_cast<const uint4*>(x), dst_row, static_cast<uint4*>(x_perm), T, k,
                       row16, T * k);
  }
  return launch_status();
}

static int check_dispatch_args(const moe_shape_t* shape, const void* x, const int32_t* topk_idx,
                               const int32_t* counts, const int32_t* offsets, const int32_t* dst_row,
                               const int32_t* src_assign, const void* x_perm) {
  const int rc = check_shape(shape);
  if (rc != MOE_OK) return rc;
  if (!counts || !offsets) return MOE_ERR_INVALID_ARG;
  if (shape->T > 0 && (!topk_idx || !dst_row || !src_assign)) return MOE_ERR_INVALID_ARG;
  if (shape->T > 0 && x_perm && (!x || !aligned16(x) || !aligned16(x_perm))) return MOE_ERR_INVALID_ARG;
  return MOE_OK;
}

// ---- the dispatch for callers that cannot allocate ------------------------------------------
// The block histograms of moe_count_and_permute_static live in this array instead of a caller's
// workspace: one copy per GPU, held for the life of the process.  In host code the array's name
// is only a handle for the runtime: the address the kernels are given is looked up once per
// device with hipGetSymbolAddress and kept.
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_SCRATCH_BYTES];
static void* g_scratch_addr[MOE_MAX_DEVICES] = {};
static std::mutex g_scratch_mutex;

static int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MOE_MAX_DEVICES) return MOE_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_addr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return MOE_ERR_HIP;
    }
    g_scratch_addr[dev] = p;
  }
  *out = g_scratch_addr[dev];
  return MOE_OK;
}

}  // namespace moe

extern "C" int moe_count_and_permute(const moe_shape_t* shape, const void* x,
                                     const int32_t* topk_idx, int32_t* counts, int32_t* offsets,
                                     int32_t* dst_row, int32_t* src_assign, void* x_perm,
                                     void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int rc = moe::check_dispatch_args(shape, x, topk_idx, counts, offsets, dst_row, src_assign, x_perm);
  if (rc != MOE_OK) return rc;
  size_t need = 0;
  moe_workspace_bytes(shape, &need);
  if (!workspace || !moe::aligned16(workspace)) return MOE_ERR_INVALID_ARG;
  if (workspace_bytes < need) return MOE_ERR_WORKSPACE;
  return moe::count_and_permute_impl(shape, x, topk_idx, counts, offsets, dst_row, src_assign, x_perm,
                                     static_cast<int32_t*>(workspace),
                                     static_cast<hipStream_t>(hip_stream));
}

extern "C" int moe_count_and_permute_static(const moe_shape_t* shape, const void* x,
                                            const int32_t* topk_idx, int32_t* counts,
                                            int32_t* offsets, int32_t* dst_row, int32_t* src_assign,
                                            void* x_perm, void* hip_stream) {
  const int rc = moe::check_dispatch_args(shape, x, topk_idx, counts, offsets, dst_row, src_assign, x_perm);
  if (rc != MOE_OK) return rc;
  // the batch must fit the fixed array: ceil(T / 256) * E * 4 bytes (blocks of 128 tokens above 128 experts)
  if (moe::dispatch_partial_bytes(shape) > MOE_STATIC_SCRATCH_BYTES) return MOE_ERR_WORKSPACE;
  void* partial = nullptr;
  if (moe::static_scratch(&partial) != MOE_OK) return MOE_ERR_HIP;
  return moe::count_and_permute_impl(shape, x, topk_idx, counts, offsets, dst_row, src_assign, x_perm,
                                     static_cast<int32_t*>(partial),
                                     static_cast<hipStream_t>(hip_stream));
}
