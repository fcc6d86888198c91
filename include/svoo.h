/*
 * svoo.h -- C boundary of the MI355X (gfx950) implementation of the ONLINE stage of SVOO:
 * per-head block-sparse self-attention of a video Diffusion Transformer layer
 * (paper Sec. 4.2 "Online Bidirectional Co-Clustering", Algorithm 1, paragraph
 * "Top Block-Pair Selection"; attention itself as defined in Sec. 4.1).
 *
 * One layer is five calls on one HIP stream:
 *
 *   svoo_cocluster          Q,K            -> labels, centroids, cluster sizes        (Algorithm 1)
 *   svoo_permute            labels, X      -> perm, offsets, X in cluster order       (implied layout)
 *   svoo_block_mask         centroids      -> kept key blocks per query block         (Top Block-Pair Selection)
 *   svoo_block_sparse_attn  sorted Q,K,V   -> sorted O over kept blocks only          (same paragraph, last sentence)
 *   svoo_unpermute          sorted O, perm -> O in token order
 *
 * plus svoo_attn, the dense softmax(Q K^T / sqrt(d)) V used for warm-up layers/steps
 * (Sec. 5.1 "Implementations") and as the speed-up denominator; svoo_kmeans, the independent
 * partitioner of the ablation; and svoo_attention_density, the measurement of the offline
 * profiling module that produces the per-layer budgets the online stage consumes.
 *
 * Conventions that hold for every entry point
 * -------------------------------------------
 *  - Every pointer except `const svoo_shape*` is a DEVICE pointer owned by the caller.  The library
 *    never allocates, frees or keeps a pointer after the call returns.  Scratch memory comes from
 *    the caller through (ws, ws_bytes); svoo_workspace_bytes() gives a size sufficient for every
 *    call with that shape.  `ws` must be 256-byte aligned; tensors must be 16-byte aligned.
 *  - Tensors are dense row-major.  Q, K, V, O are [bh, n, d]: batch and heads are folded into `bh`
 *    and every slice is an independent problem (the paper clusters per layer and per head).
 *    dtype SVOO_BF16 = 16-bit brain float bit patterns, SVOO_F32 = IEEE binary32.
 *  - Calls only enqueue work on `hip_stream` (a hipStream_t cast to void*; NULL = the null stream)
 *    and return without synchronising.  Two calls that share a workspace must be ordered on one
 *    stream.
 *  - Return value: SVOO_OK, or an error code.  Argument errors are detected on the host before
 *    anything is launched and leave all outputs untouched.  Nothing is printed, nothing aborts.
 *  - Limits: d in {64, 128}; 1 <= kq, kk <= 1024; kq, kk <= n; n <= 2^24; bh >= 1.
 *  - Cluster labels are int32 in [0, K).  An EMPTY cluster is legal everywhere: it owns zero rows
 *    after the permute (offsets[j] == offsets[j+1]), keeps its previous centroid in
 *    svoo_cocluster, and is never selected by svoo_block_mask.
 *  - Outputs are fully overwritten.  Results are deterministic: the same inputs give the same
 *    bits on every run (no floating-point atomics anywhere).
 *  - Index arrays (labels, anchor indices, permutations, offsets, block counts and lists, row lists)
 *    live in device memory, so the host cannot validate them.  An entry outside its range is clamped
 *    into it before it addresses anything: the result of such a call is meaningless, but no memory
 *    outside the tensors of the call is read or written and every kernel ends.
 */
#ifndef SVOO_H
#define SVOO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SVOO_OK = 0,
    SVOO_ERR_INVALID_ARG = 1,         /* null required pointer, size out of range, bad alignment */
    SVOO_ERR_UNSUPPORTED = 2,         /* d or dtype the kernels do not cover */
    SVOO_ERR_WORKSPACE_TOO_SMALL = 3, /* ws_bytes below what this call needs */
    SVOO_ERR_HIP = 4,                 /* a HIP launch reported an error */
    SVOO_ERR_STATIC_LIMIT = 5         /* shape beyond the fixed scratch of svoo_block_sparse_attn_static */
} svoo_status;

typedef enum { SVOO_BF16 = 0, SVOO_F32 = 1 } svoo_dtype;

typedef struct {
    int32_t bh;     /* batch * heads: number of independent slices            */
    int32_t n;      /* tokens per slice (flattened t*h*w latent grid)          */
    int32_t d;      /* head dimension d' of Sec. 4.1: 64 or 128                */
    int32_t dtype;  /* svoo_dtype of Q, K, V, O                                */
    int32_t kq;     /* number of query blocks K_q (Algorithm 1 input)          */
    int32_t kk;     /* number of key blocks K_k                                */
} svoo_shape;

/* Static string for a status code. */
const char* svoo_status_string(int status);

/* Library version, major*10000 + minor*100 + patch. */
int32_t svoo_version(void);

/* Bytes of workspace sufficient for any call below with this shape (0 if the shape is invalid). */
size_t svoo_workspace_bytes(const svoo_shape* shape);

/* Bytes of workspace svoo_permute needs for labels with n_clusters bins (they may exceed shape->kq / kk; 0 if
 * invalid).  svoo_workspace_bytes() covers n_clusters <= max(kq, kk). */
size_t svoo_permute_workspace_bytes(const svoo_shape* shape, int32_t n_clusters);

/*
 * Algorithm 1, bidirectional co-clustering.  For it = 1..iters:
 *   Step A  P = K C_q^T, Pbar = C_k C_q^T, both row-normalised (L2, floor 1e-12);
 *           labels_k[i] = argmin_j ||P^_i - Pbar^_j||_2 (lowest j on ties); C_k[j] = mean of its keys.
 *   Step B  the same for queries against the NEW C_k, with the OLD C_q as own-side centroids.
 * Sample(.) of the algorithm's first line is an input: initial centroids are the rows
 * q[init_q_idx[c]] / k[init_k_idx[c]] (indices in [0, n)), or, when init_cq / init_ck are given,
 * those float32 centroids (warm start, e.g. from the clustering of an earlier diffusion step;
 * paragraph "Clustering Reuse").  Exactly one of (init_*_idx, init_c*) is needed per side; the
 * centroid arrays win if both are given.
 *
 * Outputs: labels_q/labels_k [bh, n]; cq [bh, kq, d], ck [bh, kk, d] float32 = exact means of the
 * returned labels (previous value for empty clusters); counts_q [bh, kq], counts_k [bh, kk].
 * objective (nullable) [bh, iters, 2] float64 (sums of N float64 terms; float32 would lose the
 * differences between iterations): sum_i ||P^_i - Pbar^_{L_i}||^2 at assignment time of Step A
 * (index 0) and Step B (index 1) -- a diagnostic, costs one extra pass per half-step.
 * Arithmetic: assignment decisions are taken in float64 (a bf16 matrix-core pass only pre-filters
 * tokens whose best and second-best scores are far apart); centroid means are float64 sums in a
 * fixed order, carried in float64 between iterations and rounded to float32 on output.
 */
int svoo_cocluster(const svoo_shape* shape, const void* q, const void* k,
                   const int32_t* init_q_idx, const int32_t* init_k_idx,
                   const float* init_cq, const float* init_ck, int32_t iters,
                   int32_t* labels_q, int32_t* labels_k, float* cq, float* ck,
                   int32_t* counts_q, int32_t* counts_k, double* objective,
                   void* ws, size_t ws_bytes, void* hip_stream);

/*
 * svoo_cocluster that also hands out the cluster-order layout of the labels it returns: perm_q [bh, n],
 * q_offsets [bh, kq+1], perm_k [bh, n], k_offsets [bh, kk+1], exactly what svoo_permute would compute
 * from labels_q / labels_k (the last iteration's centroid updates sort the labels anyway).  The
 * caller then moves Q, K, V with svoo_gather and skips the two sorts of svoo_permute.  All four
 * outputs are required.
 */
int svoo_cocluster_sorted(const svoo_shape* shape, const void* q, const void* k,
                          const int32_t* init_q_idx, const int32_t* init_k_idx,
                          const float* init_cq, const float* init_ck, int32_t iters,
                          int32_t* labels_q, int32_t* labels_k, float* cq, float* ck,
                          int32_t* counts_q, int32_t* counts_k, double* objective,
                          int32_t* perm_q, int32_t* q_offsets, int32_t* perm_k, int32_t* k_offsets,
                          void* ws, size_t ws_bytes, void* hip_stream);

/*
 * One assignment of Algorithm 1 on its own (the "Assign ... to blocks" line of Step A or B):
 * x [bh, n, d] rows against own-side centroids c_own [bh, k_own, d] through the affinity to
 * c_opp [bh, k_opp, d] (float32 both).  labels [bh, n].  k_own, k_opp <= 1024.
 */
int svoo_assign(const svoo_shape* shape, const void* x, const float* c_own, int32_t k_own,
                const float* c_opp, int32_t k_opp, int32_t* labels,
                void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Independent partitioner: Lloyd's K-means on the raw rows of ONE tensor x [bh, n, d], with no
 * coupling to the other side.  This is the block partitioning of the ablation variant "w/o On"
 * (Sec. "Ablation Study") and of the K-means based prior work the paper contrasts its co-clustering
 * with (paragraph "Difference from SVG2"; attention-recall comparison of the clustering-strategy
 * section).  Call it once for Q and once for K; everything after the partition (svoo_permute ...
 * svoo_unpermute) is unchanged.  For it = 1..iters:
 *   labels[i] = argmin_j ||x_i - c_j||_2^2 (lowest j on ties);  c_j = mean of its rows (an empty
 *   cluster keeps its centroid).
 * Start: rows x[init_idx[j]] (init_idx [bh, k]) or float32 centroids init_c [bh, k, d] (wins if
 * both are given).  1 <= k <= 1024, k <= n; shape->kq / kk are ignored.
 * Outputs: labels [bh, n]; c [bh, k, d] float32 = means of the returned labels; counts [bh, k];
 * inertia (nullable) [bh, iters] float64 = sum_i ||x_i - c_{labels[i]}||^2 at assignment time.
 * Decisions in float64 behind a bf16 matrix-core pre-filter, as in svoo_cocluster.
 * Workspace: svoo_workspace_bytes() of a shape whose kq or kk is >= k suffices.
 */
int svoo_kmeans(const svoo_shape* shape, const void* x, int32_t k, const int32_t* init_idx,
                const float* init_c, int32_t iters, int32_t* labels, float* c, int32_t* counts,
                double* inertia, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Cluster-contiguous layout (the contiguous block layout block-sparse kernels need; the paper
 * inherits it from the k-means based prior work it builds on, Sec. 2.2 / "Kernel Customization").
 * Stable counting sort of labels [bh, n] with n_clusters bins:
 *   perm[bh, n]               perm[p] = token stored at sorted position p (clusters ascending,
 *                             token index ascending inside a cluster -- the order is unique)
 *   offsets[bh, n_clusters+1] first sorted position of each cluster; offsets[n_clusters] = n
 * then, for t < n_tensors (0..4): dst[t][b, p, :] = src[t][b, perm[b, p], :].  src/dst are HOST
 * arrays of device pointers, each tensor [bh, n, d] of shape->dtype; dst must not alias src.
 * Labels outside [0, n_clusters) are clamped into range.
 */
int svoo_permute(const svoo_shape* shape, const int32_t* labels, int32_t n_clusters,
                 int32_t n_tensors, const void* const* src, void* const* dst,
                 int32_t* perm, int32_t* offsets, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * The row gather of svoo_permute alone, with a permutation computed earlier:
 * dst[t][b, p, :] = src[t][b, perm[b, p], :] for t < n_tensors (1..4).  This is what a diffusion
 * step between two re-clusterings needs (paragraph "Clustering Reuse": block partitions are stable
 * across steps, so labels, permutations and block lists are kept and only the new Q, K, V move).
 * perm values must lie in [0, n).
 */
int svoo_gather(const svoo_shape* shape, const int32_t* perm, int32_t n_tensors,
                const void* const* src, void* const* dst, void* hip_stream);

/* dst[b, perm[b, p], :] = src_sorted[b, p, :]  (inverse of the row gather above). */
int svoo_unpermute(const svoo_shape* shape, const void* src_sorted, const int32_t* perm, void* dst,
                   void* hip_stream);

/*
 * Top Block-Pair Selection.  Per slice b and query block r (skipped, count 0, if counts_q[r]==0):
 *   a_j   = scale * <cq[r], ck[j]>                      coarse estimate A_bar = C_q C_k^T
 *   w_j   = counts_k[j] * exp(a_j - max) / Z            size-weighted softmax over non-empty key blocks
 *   order = key blocks by w descending, equal weights by lower j
 *   m     = shortest prefix of `order` whose cumulative w >= tau  (all non-empty blocks if tau >= 1)
 *   b     = ceil(keep[b] * kk)                          keep = fraction of key blocks kept (budget s); a product
 *                                                       within 1e-6 kk of an integer counts as that integer
 *                                                       (keep is a float32: 0.3f * 20 must give 6, not 7)
 *   kept  = first (keep[b] > theta ? min(m, b) : max(m, b)) of `order`, clamped to [1, #non-empty]
 * (the threshold-dependent rule of the selection paragraph; Recall(A_bar, tau) is read as m / kk).
 * All of it in float64 (A_bar is written to the workspace first, bh*kq*kk doubles).  keep [bh] float32
 * in [0, 1] on the device; tau in (0, 1], theta any.
 *
 * Outputs: block_count [bh, kq]; block_list [bh, kq, kk] kept key-block ids ascending in the first
 * block_count entries (the rest is set to -1); bitmap (nullable) [bh, kq, kk] 0/1 bytes.
 */
int svoo_block_mask(const svoo_shape* shape, const float* cq, const float* ck,
                    const int32_t* counts_q, const int32_t* counts_k, const float* keep,
                    float tau, float theta, float scale,
                    int32_t* block_count, int32_t* block_list, uint8_t* bitmap,
                    void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Attention over kept block pairs only: for sorted query row p in query block r,
 *   out[p] = sum_t softmax_t(scale * <q[p], k[t]>) v[t],  t over the rows of all kept key blocks of r,
 * the softmax normalised over those keys.  q_sorted / k_sorted / v_sorted / out_sorted [bh, n, d]
 * in cluster order; q_offsets [bh, kq+1], k_offsets [bh, kk+1] from svoo_permute; block_count /
 * block_list from svoo_block_mask.  lse (nullable) [bh, n] float32: log-sum-exp of the scaled
 * logits over the kept keys (natural log).  A query block with no kept key writes zeros.
 * scale must be finite and > 0.
 * bf16: both contractions on bf16 matrix cores with float32 accumulation, probabilities rounded to
 * bf16 before the second one; f32: float32 arithmetic throughout.
 */
int svoo_block_sparse_attn(const svoo_shape* shape, const void* q_sorted, const void* k_sorted,
                           const void* v_sorted, const int32_t* q_offsets, const int32_t* k_offsets,
                           const int32_t* block_count, const int32_t* block_list, float scale,
                           void* out_sorted, float* lse, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * The same attention with the query-side row moves folded in: q, out (and lse) are in TOKEN order
 * and q_perm [bh, n] is the query permutation of svoo_permute (sorted row p is token q_perm[p],
 * every value in [0, n), each once).  The kernel reads its query rows through q_perm and writes
 * each output row straight to its token, so the caller needs neither the gather of Q (call
 * svoo_permute on the query labels with n_tensors = 0) nor svoo_unpermute.  Same arithmetic, same
 * results bit for bit as svoo_block_sparse_attn followed by svoo_unpermute.
 */
int svoo_block_sparse_attn_tokens(const svoo_shape* shape, const void* q, const int32_t* q_perm,
                                  const void* k_sorted, const void* v_sorted, const int32_t* q_offsets,
                                  const int32_t* k_offsets, const int32_t* block_count,
                                  const int32_t* block_list, float scale, void* out, float* lse,
                                  void* ws, size_t ws_bytes, void* hip_stream);

/*
 * svoo_block_sparse_attn for callers that cannot allocate device memory or carry a workspace: code
 * recorded into a HIP graph, tight serving loops between two re-clusterings, harnesses that forbid
 * hipMalloc.  Same arguments without (ws, ws_bytes), same kernels, same results bit for bit.  The one
 * piece of scratch the attention needs (the query-tile schedule, bh * (kq + 1) int32) lives in a
 * 1 MiB device array inside the library, which every GPU the library runs on holds until the process
 * ends; the call allocates nothing and frees nothing.  Limit: bh * (kq + 1) <= 262,144, otherwise
 * SVOO_ERR_STATIC_LIMIT and nothing is launched (split the slices over several calls).  All calls on
 * one GPU share that array: two calls that overlap in time on one GPU (different streams, or
 * different host threads) race on it and must be ordered by the caller; calls on one stream are safe.
 * Nothing in the array has to survive between calls and nothing needs clearing.
 */
int svoo_block_sparse_attn_static(const svoo_shape* shape, const void* q_sorted, const void* k_sorted,
                                  const void* v_sorted, const int32_t* q_offsets, const int32_t* k_offsets,
                                  const int32_t* block_count, const int32_t* block_list, float scale,
                                  void* out_sorted, float* lse, void* hip_stream);

/* Dense attention out = softmax(scale * Q K^T) V in token order; kq, kk of the shape are ignored. */
int svoo_attn(const svoo_shape* shape, const void* q, const void* k, const void* v, float scale,
              void* out, float* lse, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Attention recall of a block partition and mask (the measure of the paper's comparison of clustering
 * strategies, read as the share of each query's dense softmax mass that falls on its kept keys):
 *   recall[b, q_perm[b, p]] = exp(lse_kept_sorted[b, p] - lse_all[b, q_perm[b, p]])
 * lse_kept_sorted [bh, n]: the lse output of svoo_block_sparse_attn (cluster order); lse_all [bh, n]:
 * the lse output of svoo_attn (token order); q_perm [bh, n] the query permutation; recall [bh, n]
 * float32 in token order.  A diagnostic, not a step of the layer.  shape->kq / kk are ignored.
 */
int svoo_row_recall(const svoo_shape* shape, const float* lse_kept_sorted, const float* lse_all,
                    const int32_t* q_perm, float* recall, void* hip_stream);

/*
 * Offline profiling: attention density (Sec. 4.1, offline profiling module, the equation defining
 * d_{l,h}).  For slice b and query row i (all rows, or the n_rows rows listed in `rows`, one list
 * shared by all slices, indices in [0, n)):
 *   p_t  = softmax_t(scale * <q_i, k_t>) over all n keys of the slice,
 *   prefix_len[b, i] = size of the shortest descending-sorted prefix of p whose sum reaches tau
 *                      (reaching it exactly is enough; equal entries are taken as needed),
 *   density[b] = mean_i prefix_len[b, i] / n.
 * q, k [bh, n, d]; rows (nullable, then n_rows must equal n) [n_rows] int32; tau in (0, 1] (the
 * paper uses 0.95); prefix_len [bh, n_rows] int32; density [bh] float64; passes (nullable) [bh]
 * int32 = number of passes over the keys the slowest row group of the slice needed (what the
 * call cost: passes x n_rows x n x d multiply-adds).  shape->kq / kk are ignored.  No workspace.
 * Logits in float32 (bf16 inputs: matrix cores, float32 accumulation), masses added in float32
 * within 64 keys and in float64 across them, in a fixed order that depends only on the shape of
 * the call (small row samples split the keys between the waves of a workgroup), so a result is
 * reproducible and two shapes can differ only where a cumulative sum meets tau to rounding.  No
 * sort: the cut is found by bisection on the logit value, one pass over the keys per step (about
 * 30 passes at 75,600 keys), so a call costs that many score-matrix computations for the listed rows.
 */
int svoo_attention_density(const svoo_shape* shape, const void* q, const void* k, const int32_t* rows,
                           int32_t n_rows, float tau, float scale, int32_t* prefix_len, double* density,
                           int32_t* passes, void* hip_stream);

/*
 * Measurement aids (not part of the method; for callers that quote a kernel's rate against what
 * this GPU sustains rather than against the data-sheet figure).
 *
 * svoo_microbench_mfma_bf16: `workgroups` groups of 4 waves each run `iters` x 16 bf16 matrix-core
 * instructions (32x32x16, float32 accumulation) on register operands -- random ones if
 * random_operands != 0, else one constant (the sustained clock depends on the data).  sink
 * (device) [workgroups * 256] float receives values that only keep the work alive; *flops (host,
 * nullable) receives the launch's flop count.  The caller times the launch on its stream.
 *
 * svoo_microbench_copy: dst[0..bytes) = src[0..bytes) (device, 16-byte aligned, bytes a multiple
 * of 16, no overlap) with plain 16-byte loads and stores; moves 2 x bytes.
 *
 * svoo_microbench_attn_tile: what one 64-key tile step of the bf16 attention kernel (d = 128, 4 waves x 32
 * query rows, two workgroups per CU, 512 workgroups in all) moves through the LDS, without the softmax:
 * per wave 16 K fragment reads, 32 transposing V fragment reads, 8 direct global->LDS loads of 1 KB out of
 * L2 and the 32 matrix instructions they feed -- the subset in `parts` (bit 0 K reads, 1 V reads, 2 direct
 * loads, 3 matrix instructions; instantiated: 1, 2, 3, 4, 7, 8, 11, 15), `iters` steps with one barrier
 * each.  src (device, 16-byte aligned, at least 4 MiB + 64 KiB readable): tile data, e.g. a K tensor;
 * sink (device) [512 * 256] float.  Launch time / iters = time of one tile round of a CU (256 query rows
 * x 64 keys = 256 matrix instructions = 8.39 MFLOP).
 */
int svoo_microbench_attn_tile(int32_t parts, int32_t iters, const void* src, float* sink, void* hip_stream);
int svoo_microbench_mfma_bf16(int32_t workgroups, int32_t iters, int32_t random_operands, float* sink,
                              double* flops, void* hip_stream);
int svoo_microbench_copy(const void* src, void* dst, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SVOO_H */
