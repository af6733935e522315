/*
 * vp.h - C ABI of the clustered vocabulary projection library for MI355X
 * (gfx950), after "Fast Vocabulary Projection Method via Clustering for
 * Multilingual Machine Translation on GPU" (arxiv 2208.06874).
 *
 * At each decode step a hidden row h picks its nearest k-means centroid
 * (section 2.3, Eq. 2), is projected only onto that cluster's active-token
 * columns of the output embedding (Eq. 1 of section 2.1 restricted as in step
 * 3 of the inference list of section 2.3), and a log-softmax over those
 * candidates (steps 4-5: excluded tokens are at -infinity) plus a descending
 * top-k (section 2.1) are returned.  Unlike the paper's own GPU design, which
 * unions the active sets of a batch and runs one gathered GEMM, rows are
 * bucketed by cluster and each bucket streams its cluster's pre-packed slab;
 * batches that occupy so many clusters that their slabs outweigh the whole of W
 * run the full projection with every row masked to its own active set instead
 * (same results; the planner chooses per call).
 *
 * Conventions
 *  - "device" pointers are HIP device memory of the current device, "host"
 *    pointers ordinary memory.  The caller owns every device byte: the arena
 *    that holds the packed index and the per-call workspace.  The library
 *    allocates no device memory.
 *  - hip_stream is a hipStream_t passed as void* (NULL = the null stream).
 *  - vp_project* only enqueue kernels: no host synchronisation, no device to
 *    host copy, no allocation.  Argument errors are found on the host before
 *    anything is launched and leave the outputs untouched.
 *  - All calls return a vp_status; vp_last_error() gives the message of the
 *    calling thread's last failure.
 *  - Results are deterministic: equal inputs give bit-identical outputs.
 *  - fp16 inputs, fp32 accumulation; logits are never rounded to fp16.
 */
#ifndef VP_H
#define VP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vp_index vp_index; /* opaque host-side handle */

typedef enum {
    VP_OK = 0,
    VP_ERR_INVALID_ARG = 1, /* null/misaligned pointer, bad id list, size out of range */
    VP_ERR_UNSUPPORTED = 2, /* a shape the kernels do not handle (see limits below)    */
    VP_ERR_WORKSPACE = 3,   /* arena / workspace / output capacity too small           */
    VP_ERR_HIP = 4          /* a HIP runtime call or kernel launch failed               */
} vp_status;

/* Limits: d % 8 == 0, 8 <= d <= 4096; 1 <= K <= 4096; 1 <= V < 2^31 - 16;
 * 1 <= k <= k_max <= 32; N <= 65536 per call.  An active set may be empty (a cluster
 * that lost its members in training): rows that fall into it get ids -1 and log-probs
 * -inf; at least one set must hold a token. */
#define VP_MAX_TOPK 32
#define VP_MAX_CLUSTERS 4096
#define VP_MAX_ROWS 65536
#define VP_MAX_DIM 4096
#define VP_WS_OVERFLOW_WORD 2 /* index of the overflow flag among the workspace's 32-bit words */

/* vp_build_desc.flags: leave out the copy of W with one contiguous row per token (V * d_pad * 2
 * bytes, as much again as the packed W) that only vp_project_union reads; that call then returns
 * VP_ERR_UNSUPPORTED for the index. */
#define VP_BUILD_NO_UNION 1u

typedef struct {
    int32_t d;             /* embedding dimension                                        */
    int32_t V;             /* vocabulary size                                            */
    int32_t K;             /* number of clusters (the paper's r)                         */
    const void *W;         /* device, fp16, W[d, V] row-major as in section 2.1          */
    const void *bias;      /* device, fp16, b[V]                                         */
    const void *centroids; /* device, fp16, C[K, d] row-major                            */
    const int64_t *cand_offsets; /* host, [K+1], cand_offsets[0] = 0, increasing         */
    const int32_t *cand_ids;     /* host, active sets A_j (section 2.2) back to back;
                                    each strictly ascending, ids in [0, V)               */
    void *arena;           /* device, 256-byte aligned, >= vp_build_bytes()              */
    size_t arena_bytes;
    int32_t k_max;         /* largest top-k that will be requested                       */
    uint32_t flags;        /* 0, or VP_BUILD_NO_UNION                                    */
} vp_build_desc;

typedef struct {
    int32_t d, V, K, k_max;
    int32_t d_pad;            /* d rounded up to the packed k-extent                    */
    int32_t n_min, n_max;     /* smallest / largest active set                          */
    int64_t n_total;          /* sum of active-set sizes                                */
    int64_t slab_bytes;       /* packed per-cluster slabs                               */
    int64_t full_bytes;       /* packed copy of the whole W                             */
    int64_t arena_bytes_used;
} vp_index_info;

/* Bytes of arena vp_build needs for this description (device pointers are not
 * read).  Returns 0 and sets the error message if the description is invalid. */
size_t vp_build_bytes(const vp_build_desc *desc);

/* Packs the index into the arena: ||C_j||^2 per centroid (the precomputed term
 * of Eq. 2), centroids and W re-tiled for the matrix cores, W once more with one
 * contiguous row per token (for vp_project_union; not with VP_BUILD_NO_UNION), a
 * membership bit list per cluster, and per cluster a slab with its active
 * tokens' columns, their bias and their ids.  W, bias and
 * centroids are only read during this call (the index keeps its own copies);
 * the arena must outlive the index.  Synchronises the stream before returning.
 * Unsorted, duplicate or out-of-range ids: VP_ERR_INVALID_ARG.  All active sets
 * empty, d % 8 != 0, limits exceeded: VP_ERR_UNSUPPORTED. */
vp_status vp_build(const vp_build_desc *desc, void *hip_stream, vp_index **out);

vp_status vp_get_info(const vp_index *idx, vp_index_info *info);

/* Tuning knobs (host side, take effect on the next call):
 *   "target_items"  work items the projection is split into (default 8192)
 *   "rstar"         buckets with at most this many rows use the dot-product
 *                   GEMV loop, larger ones the MFMA loop (default 0, max 4)
 *   "full_target_items"  same as target_items for vp_project_full
 *   "dispatch"      1 (default): vp_project runs the full projection with every row masked
 *                   to its own cluster's active set instead of streaming the occupied
 *                   slabs, when the planner's cost model says that is cheaper (many
 *                   occupied clusters whose slabs outweigh one pass over W); same token ids,
 *                   log-probs equal up to the order of the fp32 sums.  0: always the slabs.
 *   "cost_bw_slab_gbs", "cost_bw_full_gbs", "cost_bw_l2_gbs", "cost_bw_gemm_gbs",
 *   "cost_bw_gemm_split_gbs", "cost_bw_gather_gbs"   GB/s of the cost model
 *   "cost_row_slab_ns"   its time per row of the slab form beyond the bytes (default 60)
 *   "union_dispatch" 1 (default): vp_project_union may skip the gather of U's columns and run
 *                   the full projection with the batch's boolean list as every row's mask
 *                   when the cost model says that is cheaper (large unions); same results
 *   "gemm_min_rows" projections that keep all rows in one bucket (full, masked, union)
 *                   use the kernel with 64 rows per work item from this many rows on
 *                   (default 17; 0: never); d_pad must be 256, 512, 1024, 1536 or 2048
 *   "gemm_target_items"  work items of that kernel (default 512)
 *   "gemm_lds"      1 (default): up to d_pad = 1536 those items run on the kernel that keeps
 *                   their rows in LDS (64 rows, 48 at d_pad = 1536; no split of the k-extent;
 *                   one lock-free top-k list per row and workgroup); 0: the split-k kernel
 *                   everywhere
 *   "gemm_lds_items"  work items of that kernel per round (default: one per compute unit)
 *   "wide_items"    1 (default): below gemm_min_rows, vp_project_full / vp_project_union
 *                   of more than 16 rows with k <= 2 put 32 rows in an item; 0: always 16
 *   "small_path"    1 (default): batches of at most 16 rows run without a planning kernel;
 *                   every workgroup of the projection finds its own share of the work
 *                   from the per-part minima of Eq. 2 (two dependent kernels fewer in
 *                   front of the first slab byte); 0: always the planning kernel.
 *                   Same plan, same results, bit for bit.
 *   "small_pf"      1 KiB loads a wavefront of that path keeps in flight: 8, 16 or 32
 *                   (0, the default: chosen from the batch size)
 *   "raw_logits"    1 (default): calls with k >= 4 whose rows can meet at most 8,192
 *                   candidate groups of 16 in all (a few rows, short lists) keep the raw
 *                   logits of every short work item and select its k best at the end;
 *                   0: top-k lists are built while streaming, as everywhere else.
 *                   Same results.
 *   "profile"       1: time the projection kernel with HIP events (vp_get_profile)
 * Unknown name or out-of-range value: VP_ERR_INVALID_ARG. */
vp_status vp_set_option(vp_index *idx, const char *name, int64_t value);

/* Workspace bytes vp_project / vp_project_full / vp_project_debug_logits need
 * for up to N_max rows with the current options.  0 on error. */
size_t vp_workspace_bytes(const vp_index *idx, int32_t N_max);

/* Clustered projection of N hidden rows.
 *   hidden       device, fp16 [N, d] row-major, 16-byte aligned
 *   out_ids      device, int32 [N, k]: token ids by (logit descending, token id
 *                ascending); -1 where the row's active set has fewer than k tokens
 *   out_logp     device, fp32 [N, k]: logit minus log-sum-exp over the row's
 *                active set; -inf in padded slots
 *   out_cluster  device, int32 [N] or NULL: Eq. 2 cluster of each row (ties to
 *                the lowest index)
 *   workspace    device, 256-byte aligned, >= vp_workspace_bytes(idx, N)
 * Status word: the plan header at the start of the workspace holds, as its third
 * 32-bit word (VP_WS_OVERFLOW_WORD), a flag that is non-zero after a call whose
 * work list did not fit the room the host side reserved for it.  That is never
 * expected (the room is an upper bound); if it happens, every output of the call
 * is id -1 / log-prob NaN rather than a result that silently lost candidates,
 * and the flag can be read once the stream has finished the call.
 * N == 0 is a no-op returning VP_OK.  Calls that share a workspace must be
 * ordered on one stream: a call that overlaps another on the same workspace
 * reads half-written plans and may access memory out of bounds.  Calls with
 * workspaces and outputs of their own may overlap on different streams. */
vp_status vp_project(const vp_index *idx, const void *hidden, int32_t N, int32_t k,
                     int32_t *out_ids, float *out_logp, int32_t *out_cluster,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/* vp_project for callers that cannot allocate device memory and so have no
 * workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments, outputs and results as
 * vp_project, minus the workspace: the call's scratch (plan, per-part minima of
 * Eq. 2, partial results) lives in an array of VP_STATIC_SCRATCH_BYTES bytes that
 * is part of the library's device code (every GPU the library runs on holds its
 * own copy until the process ends).  Nothing is allocated or freed here, on the
 * device or by any library this calls.
 *   - N and k must be such that vp_workspace_bytes(idx, N) fits the array
 *     (about 10 MB at k_max = 8 for small batches); otherwise VP_ERR_WORKSPACE
 *     and nothing is launched.
 *   - All calls on one GPU share that GPU's array: calls that overlap on one
 *     GPU (different streams, or different indexes) race on it and may read
 *     half-written plans.  Order them on one stream.  The array keeps the last
 *     call's contents; every call rewrites what it reads. */
#define VP_STATIC_SCRATCH_BYTES (16u << 20)
vp_status vp_project_static(const vp_index *idx, const void *hidden, int32_t N, int32_t k,
                            int32_t *out_ids, float *out_logp, int32_t *out_cluster, void *hip_stream);

/* The default projection of section 2.1 over all V tokens (log-softmax over V,
 * top-k), same output contract; the baseline the speed-up is quoted against. */
vp_status vp_project_full(const vp_index *idx, const void *hidden, int32_t N, int32_t k,
                          int32_t *out_ids, float *out_logp,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* The paper's own batched form of the inference list (section 2.3): the active
 * sets of the predicted clusters of all N rows are united (boolean list over
 * the vocabulary -> reduced column set U, ascending), every row is projected
 * onto U and its log-softmax is normalised over U (tokens outside U are at
 * -infinity).  Same output contract as vp_project, with logp relative to U;
 * the two agree when all rows of the batch fall into one cluster.
 *   out_union_size  device, int32 [1] or NULL: receives |U|
 *   workspace       device, 256-byte aligned, >= vp_union_workspace_bytes(idx, N)
 *                   (it also holds the columns of U gathered for this call) */
size_t vp_union_workspace_bytes(const vp_index *idx, int32_t N_max);
vp_status vp_project_union(const vp_index *idx, const void *hidden, int32_t N, int32_t k,
                           int32_t *out_ids, float *out_logp, int32_t *out_cluster,
                           int32_t *out_union_size, void *workspace, size_t workspace_bytes,
                           void *hip_stream);

/* Parity/debug entry, not part of the timed path: every candidate logit.
 *   full == 0: row r's logits over its cluster's active set, in list order, at
 *              out_logits[out_row_offsets[r] .. out_row_offsets[r+1]);
 *              out_cluster (required) receives the clusters.
 *   full != 0: all V logits of row r at out_logits[r * V ..]; out_cluster may be
 *              NULL; out_row_offsets[r] = r * V.
 *   out_row_offsets  device, int64 [N+1]
 *   out_logits       device, fp32, capacity in elements must be >= N * n_max
 *                    (full == 0) or N * V (full != 0), else VP_ERR_WORKSPACE. */
vp_status vp_project_debug_logits(const vp_index *idx, const void *hidden, int32_t N, int32_t full,
                                  int32_t *out_cluster, int64_t *out_row_offsets,
                                  float *out_logits, size_t out_logits_capacity,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

/* Benchmark aid: after vp_set_option(idx, "profile", 1) every vp_project and
 * vp_project_full brackets its projection kernel (the kernel that streams the
 * slabs) with a pair of HIP events on the call's stream.  vp_get_profile waits
 * for the recorded events, returns the summed kernel time in milliseconds and
 * the number of launches, and forgets them.  At most 16384 launches are kept
 * between two calls.  Not meant for use under graph capture. */
vp_status vp_get_profile(vp_index *idx, double *kernel_ms_total, int64_t *launches);

/* Benchmark aid: what this GPU actually sustains, to stand beside the published peaks in a
 * roofline.  Streams buf once per repeat with a kernel that only reads (1 KiB non-temporal
 * loads per wavefront, 8 in flight, as the slab kernel issues them) and runs a loop of
 * v_mfma_f32_16x16x32_f16 on register operands; both timed with HIP events on the stream.
 *   buf          device, 256-byte aligned, only read; bytes >= 64 MiB
 *   read_gbs     host, receives the best GB/s over the repeats
 *   mfma_tflops  host, receives the best dense fp16 TFLOP/s over the repeats
 * Synchronises the stream.  repeats in [1, 100]. */
vp_status vp_measure_ceilings(const void *buf, size_t bytes, int32_t repeats, double *read_gbs,
                              double *mfma_tflops, void *hip_stream);

/* ---- Offline training of the clusters (section 2.2 "Offline Training of Clusters";
 * training settings of section 3.1: k-means, 20 iterations) ----
 *
 * vp_kmeans: `iters` Lloyd iterations over n recorded hidden vectors, then the
 * membership of every vector against the final centroids.  An iteration assigns
 * every vector to its nearest centroid (Eq. 2 as at decode time: fp16 inputs, fp32
 * accumulation, ties to the lowest index) and replaces every centroid by the mean
 * of its members; a cluster without members keeps its centroid.  The sums are
 * exact (every fp16 value is a multiple of 2^-24; see the bound on x below) and each
 * mean is rounded once to fp16 (nearest, ties to even), so equal inputs give
 * bit-identical centroids and, given the memberships, the centroids equal the
 * correctly rounded means.
 *   x          device, fp16 [n, d] row-major, 16-byte aligned, finite values;
 *              per cluster and coordinate the sum of |x| must stay below 2^29
 *   centroids  device, fp16 [K, d]: starting centroids in, trained centroids out
 *   assign     device, int32 [n]: cluster of every vector under the final centroids
 *   counts     device, int32 [K]: members per cluster under the final centroids
 *   workspace  device, 256-byte aligned, >= vp_kmeans_workspace_bytes(n, d, K)
 *   flags      0, or VP_KMEANS_SPLIT_EMPTY: after every iteration the clusters without
 *              members, in ascending order, each take the cluster with the most members
 *              at that moment (ties: lowest index; at least two members), whose centroid
 *              c becomes c (1 - 2^-10) while c (1 + 2^-10), both rounded to fp16, goes to
 *              the empty cluster, and half of whose member count moves with it (the paper
 *              names no remedy for such clusters; this is the usual one made deterministic)
 * Only enqueues kernels.  Limits: d % 8 == 0, 8 <= d <= 4096, 1 <= K <= 4096,
 * 1 <= n < 2^31, 0 <= iters <= 1000. */
#define VP_KMEANS_SPLIT_EMPTY 1u
size_t vp_kmeans_workspace_bytes(int64_t n, int32_t d, int32_t K);
vp_status vp_kmeans(const void *x, int64_t n, int32_t d, int32_t K, int32_t iters, uint32_t flags, void *centroids,
                    int32_t *assign, int32_t *counts, void *workspace, size_t workspace_bytes,
                    void *hip_stream);

/* vp_active_sets: the active set of cluster j is the ascending union of the T
 * recorded likely tokens of all of its members (section 2.2; the worked example
 * there: members with tokens {2,4,6} and {2,8,9} give {2,4,6,8,9}).
 *   top_ids       device, int32 [n, T]: recorded tokens (for instance out_ids of
 *                 vp_project_full with k = T); entries outside [0, V) are skipped
 *   assign        device, int32 [n]: cluster of every vector (vp_kmeans); vectors
 *                 with a cluster outside [0, K) are skipped
 *   cand_offsets  device, int64 [K + 1]: receives the offsets (always written)
 *   cand_ids      device, int32 [capacity]: receives the sets back to back, the
 *                 layout vp_build_desc takes (after a copy to the host)
 *   total         host, receives the number of entries; when it exceeds capacity
 *                 nothing is written to cand_ids and VP_ERR_WORKSPACE is returned
 *   workspace     device, 256-byte aligned, >= vp_active_sets_workspace_bytes(K, V)
 * Synchronises the stream once (to learn the total).  A cluster without members
 * gets an empty set (which vp_build accepts). */
size_t vp_active_sets_workspace_bytes(int32_t K, int32_t V);
vp_status vp_active_sets(const int32_t *top_ids, const int32_t *assign, int64_t n, int32_t T, int32_t K,
                         int32_t V, int64_t *cand_offsets, int32_t *cand_ids, int64_t capacity,
                         int64_t *total, void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---- Toy search consumer (section 2.1: the sorted probabilities feed beam search,
 * greedy search or sampling) ----
 * One beam-search step for S sentences of B hypotheses each.  Row s * B + b of the
 * inputs belongs to hypothesis b of sentence s.
 *   cand_ids    device, int32 [S * B, k]: the projection's out_ids (entries < 0: none)
 *   cand_logp   device, fp32 [S * B, k]: the projection's out_logp
 *   scores      device, fp32 [S * B]: accumulated log-probability of every hypothesis
 *               (-inf: dead; a search starts with 0 for hypothesis 0 and -inf elsewhere)
 *   out_scores  device, fp32 [S * B]: the B largest sums scores[b] + cand_logp[b][j] of
 *               each sentence, descending; equal sums in order of b, then j
 *   out_parent  device, int32 [S * B]: the hypothesis b each one continues
 *   out_token   device, int32 [S * B]: the token that continues it
 * Missing hypotheses (fewer than B finite sums): -inf, -1, -1.  B = 1 is greedy search.
 * Limits: B * k <= 2048, k <= 32.  Only enqueues one kernel. */
vp_status vp_beam_step(const int32_t *cand_ids, const float *cand_logp, const float *scores, int32_t S,
                       int32_t B, int32_t k, float *out_scores, int32_t *out_parent, int32_t *out_token,
                       void *hip_stream);

/* Host utility: v rounded to fp16 bits exactly as vp_kmeans rounds a mean. */
uint16_t vp_round_to_half(double v);

/* Frees the host handle only; the arena stays the caller's. */
void vp_destroy(vp_index *idx);

/* Message of the calling thread's last non-OK status ("" if none). */
const char *vp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* VP_H */
