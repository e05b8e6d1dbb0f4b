/*
 * moe.h - C ABI of the single-GPU MoE-layer forward for AMD MI355X (gfx950).
 *
 * The layer is the one the paper serves (Section 2.2): a gating network plus E
 * expert networks; the gate routes every token to k experts, a "scatter" brings
 * tokens to their experts, the experts run, and a "gather" collects and reorders
 * their outputs:   y[t] = sum_{j<k} g_j(x[t]) * E_{idx[t,j]}(x[t]).
 * On one GPU the scatter is a permutation of token rows into expert-contiguous
 * order and the gather is its weighted inverse.  The per-expert token counts the
 * dispatch produces are the paper's expert load W_l (Sections 3.3 and 4.1), the
 * statistic its predictor, scaler and placer consume.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers into memory the caller owns; the
 *     library never allocates, frees or keeps them.  `shape` is a HOST pointer.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it; they never synchronise the host.
 *   - Tensors are dense row-major.  `dtype` selects the storage type of x, all
 *     weights, x_perm, h, y_perm and y: MOE_F32 (IEEE float) or MOE_BF16
 *     (bfloat16, round-to-nearest-even on every store).  Accumulation is fp32
 *     (fp64 where noted).  Row byte sizes d*b and F*b must be multiples of 16 and
 *     every pointer 16-byte aligned.
 *   - Return value: MOE_OK or a negative moe_status_t; nothing is thrown and
 *     nothing aborts.  Arguments are validated on the host before any launch; on
 *     error no work has been enqueued.  T == 0 is a valid no-op.
 *   - Non-finite inputs and expert indices outside [0,E) give unspecified values
 *     (never out-of-bounds accesses).
 *   - Limits: 1 <= k <= E <= 256, k <= 64, T*k < 2^31.
 */
#ifndef MOE_GFX950_H
#define MOE_GFX950_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype_t;

typedef enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = -1, /* null pointer, bad shape, misaligned pointer        */
  MOE_ERR_UNSUPPORTED = -2, /* shape outside the documented limits                */
  MOE_ERR_WORKSPACE = -3,   /* workspace smaller than moe_workspace_bytes()       */
  MOE_ERR_HIP = -4          /* a HIP runtime call failed (launch error)           */
} moe_status_t;

typedef struct {
  int32_t T;      /* tokens                                                       */
  int32_t d;      /* hidden size                                                  */
  int32_t E;      /* experts                                                      */
  int32_t k;      /* experts activated per token                                  */
  int32_t F;      /* SwiGLU width of one expert                                   */
  int32_t dtype;  /* moe_dtype_t                                                  */
  int32_t renorm; /* 1: the k routing weights of a token are rescaled to sum to 1 */
} moe_shape_t;

/* Bytes of device workspace that moe_count_and_permute needs, and moe_route_ws can
 * use, for this shape (one buffer of this size serves both calls of a layer). */
int moe_workspace_bytes(const moe_shape_t* shape, size_t* out_bytes);

/*
 * Gate + routing (Section 2.2: a gate decides, per token, which experts run it;
 * the gate is a bias-free d x E linear map, Sections 5 and 6.6).
 *   score[t,e] = sum_i x[t,i] * w_gate[e,i]  (+ gate_bias[e] if given), as fp32
 *   topk_idx[t,:] = the k experts with the largest score, descending; equal
 *                   scores go to the lowest expert index
 *   topk_w[t,j]   = softmax_E(score[t,:])[topk_idx[t,j]], divided by their sum
 *                   over j when shape->renorm != 0
 * x [T,d], w_gate [E,d] in `dtype`; gate_bias [E] fp32 or NULL; topk_idx [T,k]
 * int32; topk_w [T,k] fp32; scores_out [T,E] fp32 or NULL (the scores the
 * choice was taken on).  The choice is taken on correctly rounded scores: a token
 * whose leading k+1 scores are not clearly separated after the fast fp32 gate
 * product (closer than 2^-19 |x_t| max_e |w_e|, a margin that follows the size of
 * the terms that were added, not of their sum) is re-evaluated with fp64 sums.
 */
int moe_route(const moe_shape_t* shape, const void* x, const void* w_gate,
              const float* gate_bias, int32_t* topk_idx, float* topk_w, float* scores_out,
              void* hip_stream);

/*
 * moe_route with a device workspace (same operation: the same experts, weights
 * and scores to the same tolerance).  For small
 * batches (T < 8192) with a large gate matrix the gate product is then spread over
 * the whole chip by a kernel of its own and the selection reads its scores from the
 * workspace; without a workspace (and without scores_out) every block has to pull
 * the whole gate matrix through one compute unit.  workspace: 16-byte aligned,
 * contents ignored on entry and undefined on return; moe_workspace_bytes() is
 * always enough.  If it is NULL, misaligned or smaller than (T*E + T + E)*4 bytes
 * ((T + E)*4 when scores_out is given) the call behaves like moe_route (no error).
 */
int moe_route_ws(const moe_shape_t* shape, const void* x, const void* w_gate,
                 const float* gate_bias, int32_t* topk_idx, float* topk_w, float* scores_out,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Expert load + dispatch (Section 4.1: the load of expert e is its token count;
 * Section 2.2: the scatter that brings tokens to their designated experts).
 *   counts[e]  = number of assignments a = t*k+j with topk_idx[a] == e
 *   offsets    = exclusive prefix sum of counts, offsets[E] = T*k
 *   dst_row[a] = offsets[e] + number of assignments a' < a with the same expert
 *   src_assign[dst_row[a]] = a
 *   x_perm[dst_row[a], :] = x[a / k, :]
 * counts [E], offsets [E+1], dst_row [T*k], src_assign [T*k] int32; x_perm
 * [T*k,d] in `dtype`.  workspace: at least moe_workspace_bytes() bytes, 16-byte
 * aligned, contents ignored on entry.  x_perm may be NULL to skip the row copy.
 */
int moe_count_and_permute(const moe_shape_t* shape, const void* x, const int32_t* topk_idx,
                          int32_t* counts, int32_t* offsets, int32_t* dst_row,
                          int32_t* src_assign, void* x_perm, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/*
 * moe_count_and_permute for callers that cannot allocate device memory or bring a workspace:
 * code that runs under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same operation, same arguments (without the workspace) and the same results, bit for bit.  The
 * block histograms that the other call keeps in the caller's workspace live in a fixed array of
 * MOE_STATIC_SCRATCH_BYTES bytes inside the library's device image (one copy per GPU that the
 * library runs on, held until the process ends).  The call allocates and frees nothing; the first
 * call on a device looks up the array's address there (make that call outside a stream capture).
 * Limit: ceil(T / 256) * E * 4 bytes must fit the array (blocks of 128 tokens instead of 256 when
 * E > 128): up to 131072 tokens at E = 256, a million at E = 64; a larger batch returns
 * MOE_ERR_WORKSPACE and enqueues nothing.  Nothing in the array has to start at zero (every entry is
 * written before it is read), but all calls on one GPU share it: calls that overlap in time on
 * one GPU (two streams, or two host threads) race; order them on one stream.
 */
#define MOE_STATIC_SCRATCH_BYTES (1u << 20)
int moe_count_and_permute_static(const moe_shape_t* shape, const void* x, const int32_t* topk_idx,
                                 int32_t* counts, int32_t* offsets, int32_t* dst_row,
                                 int32_t* src_assign, void* x_perm, void* hip_stream);

/*
 * Grouped expert FFN (Section 3.2: expert computation dominates the layer).
 * For every expert e and every row r in [offsets[e], offsets[e+1]):
 *   h[r,:]      = silu(w1[e] x_perm[r]) * (w3[e] x_perm[r])     silu(z) = z / (1 + exp(-z))
 *   y_perm[r,:] = w2[e] h[r]
 * x_perm [T*k,d]; w1, w3 [E,F,d]; w2 [E,d,F]; h [T*k,F] (caller-provided scratch,
 * holds the activations on return); y_perm [T*k,d]; all in `dtype`; offsets [E+1]
 * int32 on the device (read by the kernels; no host round trip).
 * A GEMM's tiles run in rounds of the chip's compute units; when the last round is at most half
 * full, the bf16 MFMA kernels cut each of its tiles along the rows into 2 to 4 pieces (of 64 rows
 * or more) for the otherwise idle units.  A row's sums do not depend on the rows it shares a tile
 * with, so the outputs are the same bits whether tiles are cut or not.
 * Two launches (one per GEMM) on `hip_stream`; the library keeps no stream, event or other state
 * of its own, so calls from several host threads or on several streams are independent, and a
 * stream capture records exactly these launches.
 */
int moe_grouped_ffn(const moe_shape_t* shape, const void* x_perm, const int32_t* offsets,
                    const void* w1, const void* w3, const void* w2, void* h, void* y_perm,
                    void* hip_stream);

/*
 * One half of moe_grouped_ffn (same operation, Section 3.2; same arguments and
 * rules).  part 1: h = silu(W1 x_perm) * (W3 x_perm); part 2: y_perm = W2 h (reads
 * the h that part 1 left).  moe_grouped_ffn is part 1 followed by part 2; the
 * split lets a caller time the two GEMMs apart or put other work between them.
 * Any other `part` is MOE_ERR_INVALID_ARG.
 */
int moe_grouped_ffn_part(const moe_shape_t* shape, const void* x_perm, const int32_t* offsets,
                         const void* w1, const void* w3, const void* w2, void* h, void* y_perm,
                         int part, void* hip_stream);

/*
 * moe_grouped_ffn without the permuted copy of the activations: the up-projection reads the
 * rows of x [T,d] directly, row r of the permuted order being x[src_assign[r] / k] (the
 * `src_assign` map of moe_count_and_permute, which may then be called with x_perm = NULL).
 * Same h and y_perm, bit for bit, as moe_grouped_ffn on the x_perm that call would have
 * written; the T*k*d*b bytes of x_perm are neither written nor read.  Entries of
 * src_assign outside [0, T*k) give unspecified values in their rows (never out-of-bounds
 * accesses).  T*d*b must be below 2^31 (else MOE_ERR_UNSUPPORTED).
 */
int moe_grouped_ffn_gather(const moe_shape_t* shape, const void* x, const int32_t* src_assign,
                           const int32_t* offsets, const void* w1, const void* w3, const void* w2,
                           void* h, void* y_perm, void* hip_stream);

/* One half of moe_grouped_ffn_gather, as moe_grouped_ffn_part is of moe_grouped_ffn
 * (part 1 reads x through src_assign and writes h; part 2 reads h and writes y_perm). */
int moe_grouped_ffn_gather_part(const moe_shape_t* shape, const void* x, const int32_t* src_assign,
                                const int32_t* offsets, const void* w1, const void* w3,
                                const void* w2, void* h, void* y_perm, int part, void* hip_stream);

/*
 * Grouped FFN and combine in one call for layers that activate ONE expert per token (k = 1:
 * Llama-4-Scout in Table 1).  With k = 1 the gather that collects and reorders the expert outputs
 * (Section 2.2) has nothing to add up: y[t] = topk_w[t] * E_idx[t](x[t]), so the down-projection
 * stores row r of its result, scaled, straight to y[src_assign[r]] (fp32 product, one rounding),
 * and neither x_perm nor y_perm exists; moe_combine is not called.  x [T,d] and src_assign as for
 * moe_grouped_ffn_gather; topk_w [T] fp32 (the routing weights of moe_route); h [T,F] scratch;
 * y [T,d].  y differs from moe_grouped_ffn_gather + moe_combine by at most one rounding of the
 * storage type (those round y_perm first).  src_assign must be a permutation of 0..T-1 for every
 * row of y to be written; entries outside give unspecified rows (never out-of-bounds accesses).
 * MOE_ERR_UNSUPPORTED if shape->k != 1.  Layers with k >= 2 keep the two calls: the k
 * contributions to a token come from different experts' tiles, and adding them in the stores would
 * need atomics whose order (and with it the rounding of y) depends on scheduling.
 */
int moe_grouped_ffn_combine_k1(const moe_shape_t* shape, const void* x, const int32_t* src_assign,
                               const int32_t* offsets, const void* w1, const void* w3, const void* w2,
                               const float* topk_w, void* h, void* y, void* hip_stream);

/*
 * moe_grouped_ffn / moe_grouped_ffn_gather (Section 3.2) with a workspace that lets the bf16 MFMA
 * kernels cut tiles along the reduction dimension.  A GEMM's tiles run in rounds of the chip's
 * compute units; when the last round is at most half full, each of its tiles is computed as 2 to
 * 4 parts on otherwise idle units, the parts leave their fp32 accumulators in the workspace, and
 * a small launch right after the GEMM adds them in part order (deterministic), rounds and stores
 * once.  For such tiles the fp32 sum is grouped differently than in the calls without a
 * workspace, so h and y_perm may differ from theirs in the last bit; all other rows are
 * bit-identical.  Each GEMM costs one more (mostly empty) launch.  GEMMs whose reduction is too
 * short to be worth cutting (fewer than 96 steps of 64) keep the cut along the rows of the calls
 * without a workspace.
 *   x, src_assign   src_assign == NULL: x is x_perm [T*k, d] as for moe_grouped_ffn;
 *                   otherwise x [T, d] and the map, as for moe_grouped_ffn_gather
 *   parts           1 = up-projection only, 2 = down-projection only, 3 = both; plus 4: tiles
 *                   of an under-filled last round are not cut along their rows either (every
 *                   tile whole, as for a batch that fills its rounds: for measurements and for
 *                   tests of the whole-tile code on small inputs; same output bits)
 *   workspace       device memory, 16-byte aligned, at least moe_ffn_workspace_bytes() bytes
 *                   (80 MiB on a 256-CU device), contents irrelevant; or NULL (then exactly
 *                   moe_grouped_ffn / moe_grouped_ffn_gather).  Calls that share a workspace
 *                   must not overlap in time.
 * Errors as moe_grouped_ffn; MOE_ERR_WORKSPACE if workspace_bytes is too small.
 */
int moe_ffn_workspace_bytes(const moe_shape_t* shape, size_t* out_bytes);
int moe_grouped_ffn_ws(const moe_shape_t* shape, const void* x, const int32_t* src_assign,
                       const int32_t* offsets, const void* w1, const void* w3, const void* w2,
                       void* h, void* y_perm, int parts, void* workspace, size_t workspace_bytes,
                       void* hip_stream);

/*
 * Weighted combine (Section 2.2: the gather that collects and reorders expert
 * outputs):   y[t,:] = sum_{j<k} topk_w[t,j] * y_perm[dst_row[t*k+j], :]
 * summed in fp32 in ascending j, stored once in `dtype`.  y [T,d].
 */
int moe_combine(const moe_shape_t* shape, const void* y_perm, const int32_t* dst_row,
                const float* topk_w, void* y, void* hip_stream);

/*
 * Expert Scaling (Algorithm 1, Section 4.2): how many replicas each expert of a layer gets.
 * `loads` [E] are the layer's (predicted or measured) per-expert token counts, e.g. the
 * `counts` of moe_count_and_permute; negative entries count as 0.  Every expert starts with
 * one replica and no extra memory allocated.  While one more replica still fits
 * (allocated + expert_mem <= mem_cap; expert_mem = M_e > 0 and mem_cap = M_cap >= 0 in the same
 * unit) and the coefficient of variation of the per-replica loads exceeds `cv_threshold`
 * (V), the expert whose replicas carry the largest load W_e / R_e gets one more replica
 * (equal loads: the lowest index; an expert with no load is never split).  CV is the
 * population standard deviation over the mean of the multiset that holds W_e / R_e once per
 * replica, computed in fp64; 0 for an all-zero layer.
 *   replicas [E] int32   R_e >= 1
 *   cv_out   [2] double  optional (may be NULL): CV before the first step (= CV of `loads`
 *                        themselves) and CV of the returned replica counts
 * E <= 256; mem_cap / expert_mem <= MOE_MAX_EXTRA_REPLICAS (else MOE_ERR_UNSUPPORTED).
 * One small launch on `hip_stream`; nothing is read back to the host.
 */
#define MOE_MAX_EXTRA_REPLICAS 65536
int moe_scale_replicas(int32_t E, const int32_t* loads, int64_t expert_mem, int64_t mem_cap,
                       double cv_threshold, int32_t* replicas, double* cv_out, void* hip_stream);

/*
 * Even split of every expert's rows over its replicas (Section 3.3: an expert's load is
 * divided evenly among its replicas).  Expert e owns rows [offsets[e], offsets[e+1]) of the
 * permuted order; replica r of its R_e = replicas[e] gets the rows
 *   [offsets[e] + floor(c*r/R_e), offsets[e] + floor(c*(r+1)/R_e)),   c = offsets[e+1]-offsets[e],
 * so piece sizes differ by at most one row.  Segments are listed expert-major.
 *   n_segments  [1] int32            S = sum_e R_e
 *   seg_offsets [max_segments+1]     seg_offsets[0] = offsets[0]; segment s covers rows
 *                                    [seg_offsets[s], seg_offsets[s+1])
 *   seg_expert  [max_segments]       the expert of segment s
 * Only the first min(S, max_segments) segments are written; a caller that cannot bound S
 * checks n_segments afterwards.  E <= 256.  One small launch; no host synchronisation.
 */
int moe_replica_segments(int32_t E, const int32_t* offsets, const int32_t* replicas,
                         int32_t max_segments, int32_t* seg_offsets, int32_t* seg_expert,
                         int32_t* n_segments, void* hip_stream);

/*
 * Expert Placement (Algorithm 2, Section 4.3): the GPU of every expert replica of a layer.
 * Replicas are taken from the most to the least loaded (a replica of expert e carries
 * loads[e] / replicas[e]; equal loads in ascending (expert, replica) order).  A replica that
 * the previous round placed and that is still alive keeps its GPU (warm start); any other
 * joins the GPU with the smallest aggregated load so far (equal loads: the lowest index);
 * the GPU's load then grows by the replica's load (fp64, in placement order).
 *   loads, replicas [E]      as for moe_scale_replicas / its output
 *   n_gpus                   1 .. 64
 *   prev_replicas [E], prev_gpu [sum of prev_replicas]
 *                            optional (both NULL = no previous round): the previous round's
 *                            replica counts and its gpu_of output (expert-major: replica r of
 *                            expert e at index prev_replicas[0] + .. + prev_replicas[e-1] + r);
 *                            -1 = that replica is no longer alive.  Replica indices at or above
 *                            the previous count are new (cold)
 *   gpu_slots [n_gpus]       optional (NULL = unlimited): replicas each GPU can hold; a GPU
 *                            without a free slot takes no replica, warm or not; a replica that
 *                            finds no free slot anywhere gets -1
 *   gpu_of [max_segments]    GPU per replica, in the segment order of moe_replica_segments; only
 *                            the first min(S, max_segments) entries are written
 *   gpu_load [n_gpus] double, gpu_count [n_gpus] int32, n_warm [1] int32
 * E <= 256; at most E + MOE_MAX_EXTRA_REPLICAS replicas are placed (later ones are skipped and
 * their entries not written).  One small launch; no host synchronisation.
 */
int moe_place_replicas(int32_t E, const int32_t* loads, const int32_t* replicas, int32_t n_gpus,
                       const int32_t* prev_replicas, const int32_t* prev_gpu,
                       const int32_t* gpu_slots, int32_t max_segments, int32_t* gpu_of,
                       double* gpu_load, int32_t* gpu_count, int32_t* n_warm, void* hip_stream);

/* Static, human-readable text for a status code. */
const char* moe_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* MOE_GFX950_H */
