/*
 * stream.h - C ABI of the MI355X (gfx950) Stream library.
 *
 * The two operations of the paper's method on the hot path, each a sequence of HIP kernels:
 *
 *   stream_prune        Algorithm 2 ("Stream", Appendix C; prose in Section 3):
 *                       hierarchical, binary-search-style estimation of a
 *                       per-head block-sparse attention mask that keeps the
 *                       top-k key blocks of every query block under the
 *                       attention mask C, in O(T log T) time and O(T) memory.
 *   stream_sparse_attn  Eq. (2): softmax attention restricted to the retained
 *                       blocks (mask M, C inside blocks), plus the column
 *                       sums of the probabilities (the "vertical attention
 *                       scores" of Section 4.1 = attention mass received by
 *                       every key).
 *
 * and what the paper builds around them: stream_prune_multi (the sweep over k of the tracing
 * driver), stream_prune_variable (a sparsity constant per row), stream_select_update (the
 * selection step alone), stream_mask_diff (difference of two estimated masks),
 * stream_receiver_stats (block means of the dense pattern and their vertical kurtosis), and
 * stream_prune_static (stream_prune with the scratch in a device array of the library, for
 * callers that cannot allocate).
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller unless it is
 *     marked HOST.  The library allocates nothing, frees nothing and never
 *     synchronises: all work is enqueued on `hip_stream` (a hipStream_t passed
 *     as void*; NULL = the default stream).  Scratch memory comes from the
 *     caller as `workspace` (256-byte aligned, size from the *_workspace_bytes
 *     query); its contents are undefined afterwards.  (stream_prune_static is
 *     the one exception: its scratch is a device array of the library.)
 *   - Layouts: Q and O are [heads, T, head_dim], K and V are
 *     [kv_heads, T, head_dim], last dimension contiguous; the head and token
 *     strides (in elements) are given in stream_shape, 0 meaning the contiguous
 *     default.  Query head h reads key/value head h / (heads / kv_heads).
 *   - A ragged batch is packed along the token axis; cu_seqlens (HOST,
 *     int32[batch+1], cu[0] = 0, cu[batch] = T) gives the boundaries.  Blocks
 *     never straddle sequences.  As in the preamble of Algorithm 2 a sequence of
 *     L_s tokens is padded (virtually) to T_p = L_s rounded up to a multiple of
 *     lcm(b_q, b_k) and has N_s = T_p / b_q query blocks and T_p / b_k key blocks;
 *     NB = sum_s N_s counts query blocks.  With b_q = b_k = b that is
 *     N_s = ceil(L_s / b) of each.  A query block that holds padding only (possible
 *     when b_q < b_k) gets an empty list.  Key-block ids in `idx` are local to
 *     their sequence.
 *   - b_q = shape.block, b_k = shape.block_k (0 = b_q); the mask C is one of the rules of
 *     stream_mask or an explicit T x T bit array (a zero-initialised shape means causal,
 *     b_k = b_q).  A key block is valid for
 *     a query block when at least one of its real keys is visible to one of the block's real
 *     queries.
 *   - Every entry point validates its arguments on the host before any launch
 *     and returns a stream_status; nothing is thrown or logged.  Outputs are
 *     fully overwritten on STREAM_OK and untouched on an argument error.
 */
#ifndef STREAM_H_
#define STREAM_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    STREAM_OK = 0,
    STREAM_EINVAL = 1,       /* null pointer, non-positive size, inconsistent shape          */
    STREAM_EUNSUPPORTED = 2, /* valid but outside what the kernels are built for             */
    STREAM_EWORKSPACE = 3,   /* workspace missing, misaligned or smaller than the query says */
    STREAM_EDEVICE = 4       /* a HIP call (launch, copy) reported an error                  */
} stream_status;

typedef enum { STREAM_F32 = 0, STREAM_BF16 = 1 } stream_dtype;

/* The attention mask C (an input of Algorithm 2; the models of the paper use causal layers
   and, for Gemma 3, sliding-window layers; without a mask Algorithm 2 is Algorithm 1):
   key u of a sequence is visible to query t of the same sequence iff                       */
typedef enum {
    STREAM_MASK_CAUSAL = 0,  /* u <= t                                                       */
    STREAM_MASK_FULL = 1,    /* always (no mask)                                             */
    STREAM_MASK_SLIDING = 2, /* u <= t and t - u < window                                    */
    STREAM_MASK_ARRAY = 3    /* bit u of row t of the T x T bit array mask_bits is set        */
} stream_mask;

typedef struct {
    int heads;       /* query heads H                                                  */
    int kv_heads;    /* key/value heads, divides H                                     */
    int head_dim;    /* 64 or 128                                                      */
    int block;       /* b_q (and b_k unless block_k is set): 32, 64 or 128             */
    int dtype;       /* stream_dtype of Q, K, V, O                                     */
    int batch;       /* sequences in the packed batch, 1 .. 64                         */
    long long T;     /* total tokens                                                   */
    const int *cu_seqlens; /* HOST int32[batch+1]; may be NULL when batch == 1         */
    long long q_stride_h, q_stride_t; /* element strides; 0 = contiguous default       */
    long long k_stride_h, k_stride_t;
    long long v_stride_h, v_stride_t; /* stream_sparse_attn only                        */
    long long o_stride_h, o_stride_t; /* stream_sparse_attn only                        */
    int mask;        /* stream_mask: the attention mask C of Algorithm 2 and Eq. (2)   */
    long long window;/* STREAM_MASK_SLIDING: window length W in tokens, >= 1           */
    int block_k;     /* b_k: 32, 64 or 128; 0 = the same as block (b_q = b_k)          */
    /* STREAM_MASK_ARRAY: the mask C of Algorithm 2 as an explicit array, shared by all heads.
       DEVICE pointer to T rows of mask_pitch 32-bit words; C[t][u] is bit (u % 32) of word
       t * mask_pitch + u / 32; mask_pitch >= ceil(T / 32); bits at u >= T are ignored.  Single
       sequence only (batch = 1).  The array must stay unchanged until the call's work is done. */
    const unsigned int *mask_bits;
    long long mask_pitch;
} stream_shape;

/* Optional diagnostics of stream_prune (each member may be NULL). */
typedef struct {
    /* (f, l) of the nodes kept after every level, int32 [levels, heads, NB, topk_max, 2],
       -1 where a slot holds no live node; `levels` = stream_prune_levels().  Lets a checker
       replay a row level by level (the final list alone does not show which branches were
       kept at one level and dropped at the next).                                           */
    int *trace;
    /* unsigned 64-bit counter, incremented by the number of block scores (b x b x d tile
       products) the kernels computed; the caller zeroes it.                                 */
    unsigned long long *tiles_scored;
    /* HOST array of 2 * stream_prune_levels() hipEvent_t handles created by the caller, or NULL:
       event 2j is recorded on hip_stream right before the j-th launch of the refinement kernel
       and event 2j+1 right after it (there are ceil(levels / levels_per_launch) launches), so
       the caller can read each launch's duration after its own synchronisation.  Nothing is
       waited on.                                                                               */
    void *const *level_events;
    /* Refinement levels every row runs back to back inside one kernel launch: 0 = the
       library's default (all of them in one launch), 1 = one launch per level, n = at most n. */
    int levels_per_launch;
} stream_prune_diag;

/* NB = total number of query blocks of the (packed) shape, or -1 on a bad shape. */
long long stream_num_blocks(const stream_shape *shape);

/* NBk = total number of key blocks (sum over sequences of T_p / b_k; = NB when b_q = b_k), or -1. */
long long stream_num_key_blocks(const stream_shape *shape);

/* Number of refinement levels stream_prune runs for these arguments (max over sequences):
   max(1, ceil(log2(ceil(N_s / k_s)))).  The listing's n_it = ceil(log2 N) iterations give the
   same result: once every node is a single block a level maps the node set to itself.
   Returns -1 on bad arguments. */
int stream_prune_levels(const stream_shape *shape, int topk, const int *topk_per_seq);

size_t stream_prune_workspace_bytes(const stream_shape *shape, int topk_max);

/*
 * Algorithm 2 for every (query head, query block).
 *
 *   Q, K          inputs (device), layouts above
 *   topk          k, the number of key blocks kept per query block (>= 1); k > N_s keeps every
 *                 causal block
 *   topk_per_seq  HOST int[batch] overriding topk per sequence, or NULL
 *   topk_max      row length of idx/score (>= every k in use, <= 512; beyond 64 a second kernel
 *                 keeps the row's node list in on-chip memory instead of registers: no
 *                 levels_per_launch split there, and no F32 with head_dim 128 in 128 x 128 blocks)
 *   idx           int32 [heads, NB, topk_max]: retained key-block ids, ascending, padded with -1
 *   cnt           int32 [heads, NB]: number of retained blocks = min(k, valid key blocks of the
 *                 row) (causal: min(k, q+1))
 *   score         float [heads, NB, topk_max] or NULL: block score (max masked dot product,
 *                 Eq. (4), unscaled) of each retained block, padded with -inf
 *   diag          optional diagnostics or NULL
 *
 * Levels after the first reuse the parent's score for the child that contains the parent's
 * representative (same block, same score) and compute one new block score per kept node.
 * Ties in "top-k" go to the lower branch position.
 */
stream_status stream_prune(const void *Q, const void *K, const stream_shape *shape,
                           int topk, const int *topk_per_seq, int topk_max,
                           int *idx, int *cnt, float *score, const stream_prune_diag *diag,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * stream_prune for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, outputs and errors as stream_prune without `workspace`; the scratch (packed K
 * tiles, node lists, block summaries of a mask array) is a device array of
 * STREAM_STATIC_SCRATCH_BYTES that belongs to the library: every GPU the library is used on holds
 * it from the moment the library is loaded there until the process ends.  The call allocates and
 * frees nothing (no hipMalloc / hipFree, no allocating library routine) and never synchronises.
 *
 *   - Problems whose stream_prune_workspace_bytes(shape, topk_max) exceeds
 *     STREAM_STATIC_SCRATCH_BYTES return STREAM_EWORKSPACE before anything is launched (80 MiB
 *     covers e.g. 32,768 tokens x 8 KV heads x head_dim 128 in bf16 with k = 16, or 10 sequences
 *     of 8 K tokens at 28/4 heads).
 *   - The first call on a device looks up the array's address there (one hipGetSymbolAddress, no
 *     allocation); make that call outside a graph capture.
 *   - All calls on one GPU share that GPU's array, which keeps whatever the last call left in it
 *     (nothing in it has to start at zero).  Calls that overlap in time on one GPU - different
 *     streams, or different host threads - race on it: serialise them.
 */
#define STREAM_STATIC_SCRATCH_BYTES (80 * 1024 * 1024)

stream_status stream_prune_static(const void *Q, const void *K, const stream_shape *shape,
                                  int topk, const int *topk_per_seq, int topk_max,
                                  int *idx, int *cnt, float *score, const stream_prune_diag *diag,
                                  void *hip_stream);

size_t stream_sparse_attn_workspace_bytes(const stream_shape *shape, int topk_max);

/*
 * Eq. (2) on the retained blocks:  for every real query token t of query block q,
 *     S~[t,u] = scale * <Q_t, K_u>  for keys u of the blocks idx[h, q, 0..cnt-1] that the mask C
 *                                   of `shape` shows to t (causal: u <= t),
 *     P~ = softmax(S~),  O_t = sum_u P~[t,u] V_u.
 * A query that sees none of its row's retained keys (possible under a window or a mask array)
 * gets O_t = 0 and lse = -inf.
 *
 *   idx, cnt      as written by stream_prune: strictly ascending ids of key blocks of the
 *                 sequence (any such lists work); topk_max <= 512.  Other lists are handled safely
 *                 rather than fast: a row whose list is not strictly ascending or holds an id
 *                 outside [0, key blocks of the sequence) takes the token-level mask on every
 *                 tile, so a key after its query or outside the sequence never counts; ids outside
 *                 the range contribute nothing, an id listed twice counts twice
 *   scale         multiplies the dot products (the paper's Eq. (2) has scale = 1; models use
 *                 1/sqrt(head_dim))
 *   O             [heads, T, head_dim] in the input dtype
 *   lse           float [heads, T] or NULL: log-sum-exp of each row of S~
 *   mass          float [heads, T] or NULL: mass[h,u] = sum_t P~[t,u]; zeroed by the library,
 *                 accumulated with floating-point atomics (summation order not fixed)
 */
stream_status stream_sparse_attn(const void *Q, const void *K, const void *V,
                                 const stream_shape *shape,
                                 const int *idx, const int *cnt, int topk_max, float scale,
                                 void *O, float *lse, float *mass,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Algorithm 2 for several values of k over the same Q and K in one call: the tracing driver of
 * Section 3 estimates the mask again and again while it searches for the smallest k that
 * preserves the model's output.  K is packed once; a (head, query block) row runs Algorithm 2
 * for every k of the list in turn inside one kernel, keeping its Q tile on chip and reusing every
 * block score it has already computed (a block's score does not depend on k), so the values
 * after the first mostly cost a few selections.
 *
 * Result i (i < n_k) is exactly what stream_prune returns for topk = topk_list[i] (every
 * sequence of a ragged batch uses that same k):
 *   topk_list  HOST int[n_k], each in [1, topk_max]; n_k <= 32; any order (largest first reuses
 *              the most).  topk_max <= 512; beyond 64 every value runs as a launch of its own
 *              of the wide kernel (K still packed once, no reuse of scores between values)
 *   idx        int32 [heads, n_k, NB, topk_max]
 *   cnt        int32 [heads, n_k, NB]
 *   score      float [heads, n_k, NB, topk_max] or NULL
 *   diag       as for stream_prune; the trace is [levels, heads, n_k, NB, topk_max, 2] with
 *              `levels` = stream_prune_levels() of the smallest k; tiles_scored counts the
 *              block scores actually computed; levels_per_launch is ignored
 *   workspace  stream_prune_multi_workspace_bytes(shape, n_k, topk_max) bytes, 256-byte aligned
 * Errors: as stream_prune; STREAM_EUNSUPPORTED when n_k > 32.
 */
size_t stream_prune_multi_workspace_bytes(const stream_shape *shape, int n_k, int topk_max);

stream_status stream_prune_multi(const void *Q, const void *K, const stream_shape *shape,
                                 const int *topk_list, int n_k, int topk_max,
                                 int *idx, int *cnt, float *score, const stream_prune_diag *diag,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Algorithm 2 with a sparsity constant that varies per query block.  Section 4.2.1 (Discussion)
 * and Section 6 (4) observe that under a causal mask a constant k prunes the rows at the bottom
 * of the pattern harder than those at the top, and name a variable k as the remedy without
 * defining one; this entry point keeps a fixed share of each row's valid key blocks:
 *
 *     k(row) = min(topk_max, max(topk_min, ceil(valid(row) * keep_num / keep_den)))
 *
 * where valid(row) is the number of key blocks the mask C leaves to the row (q + 1 for the
 * causal mask).  Every row then runs Algorithm 2 as printed with its own k (and its own number
 * of levels).  Outputs as stream_prune: idx/score rows have topk_max entries, cnt = min(k(row),
 * valid(row)).  1 <= keep_num <= keep_den, 1 <= topk_min <= topk_max <= 512.  Workspace:
 * stream_prune_workspace_bytes(shape, topk_max).  diag->trace has stream_prune_levels(shape,
 * topk_min, NULL) levels.
 */
stream_status stream_prune_variable(const void *Q, const void *K, const stream_shape *shape,
                                    int keep_num, int keep_den, int topk_min, int topk_max,
                                    int *idx, int *cnt, float *score, const stream_prune_diag *diag,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The "top-k indices" and "update" lines of Algorithm 2 (Appendix C) as a pass of their own.
 * stream_prune performs this step inside its scoring kernels; this entry point applies it to
 * branch scores that already sit in memory.
 *
 * For each of `rows` independent rows: the row's first node_count[row] nodes
 * [node_first[row][j], node_last[row][j]] (key-block ranges, inclusive) are split at
 * m = floor((first + last + 1) / 2) into a left branch [first, m-1] (position 2j) and a right
 * branch [m, last] (position 2j+1) whose scores are branch_score[row][2j] and [2j+1].  An empty
 * branch and a branch whose score is -inf (no valid block under the mask C) are dropped; of the
 * others the `topk` with the largest scores are kept, equal scores going to the lower position.
 * The kept branches, in position order, overwrite the head of the row's node list and
 * node_count[row] becomes their number; list slots after it are left as they were.
 *
 *   branch_score  float [rows, 2 * topk_max], 8-byte aligned; must hold no NaN
 *   node_first    int32 [rows, topk_max], in/out
 *   node_last     int32 [rows, topk_max], in/out
 *   node_count    int32 [rows], in/out; values outside [0, topk_max] are clamped
 *   1 <= topk <= topk_max <= 512; rows >= 0 (0 is a no-op: the pointers are not looked at).
 * Errors: STREAM_EINVAL (null pointer, misaligned scores, bad sizes), STREAM_EUNSUPPORTED
 * (topk_max > 512, too many rows for one launch), STREAM_EDEVICE.  No workspace, no synchronisation.
 */
stream_status stream_select_update(const float *branch_score, int *node_first, int *node_last,
                                   int *node_count, long long rows, int topk, int topk_max,
                                   void *hip_stream);

/*
 * Difference of two estimated masks (Section 4.2.2, "Exploring Information Flow": the masks
 * obtained with k_fail are subtracted from those obtained with k_success to isolate the
 * connections that enable a behaviour, each weighted by its block score in the k_success run).
 *
 * For each of `rows` independent (head, query block) rows: the entries of list a (k_success)
 * that do not occur in list b (k_fail), in ascending order.
 *
 *   idx_a, cnt_a   int32 [rows, kmax_a], [rows]: ascending key-block ids, as written by
 *                  stream_prune / stream_prune_multi (entries at and after cnt are ignored)
 *   score_a        float [rows, kmax_a] or NULL: block scores of list a
 *   idx_b, cnt_b   int32 [rows, kmax_b], [rows]
 *   idx_out        int32 [rows, kmax_a]: the difference, padded with -1; must not alias an input
 *   cnt_out        int32 [rows]
 *   weight_out     float [rows, kmax_a] or NULL: score_a of the kept entries, padded with -inf
 *                  (needs score_a)
 *   1 <= kmax_a, kmax_b <= 512; counts outside [0, kmax] are clamped; rows >= 0 (0 is a no-op:
 *   the pointers are not looked at).
 * Errors: STREAM_EINVAL, STREAM_EUNSUPPORTED (kmax > 512), STREAM_EDEVICE.  No workspace.
 */
stream_status stream_mask_diff(const int *idx_a, const int *cnt_a, const float *score_a, int kmax_a,
                               const int *idx_b, const int *cnt_b, int kmax_b, long long rows,
                               int *idx_out, int *cnt_out, float *weight_out, void *hip_stream);

/*
 * Receiver-head statistics (Section 4.1, "Thought Anchors"): the section looks for heads whose
 * attention concentrates on a few parts of the context by averaging the head's DENSE attention
 * probabilities over b_q x b_k spans (the "block mean" pattern of its attention-patterns figure)
 * and measuring the maximum vertical kurtosis of these block means.  The dense pattern is never
 * stored: O(T^2 d) time, O(T) memory besides the optional block_mean output.
 *
 *   P = softmax over the visible keys of scale * Q K^T (mask C of `shape`), per head/sequence
 *   M[i, j] = sum of P over (queries of block i) x (keys of block j) / (real queries of i *
 *             real keys of j), where key block j is valid for query block i, else 0
 *   column j = the values M[i, j] over the query blocks i that j is valid for ("vertical"):
 *             col_mean[j] their mean, col_kurt[j] their excess kurtosis m4 / m2^2 - 3 (biased
 *             central moments; 0 with fewer than 4 values or no spread)
 *
 *   scale       as stream_sparse_attn (> 0, finite)
 *   block_mean  float [heads, NB, NBk] (query block, key block; global block ids; NBk =
 *               stream_num_key_blocks(), = NB when b_q = b_k) or NULL; zero outside the valid
 *               blocks and across sequences of a packed batch
 *   col_mean    float [heads, NBk]
 *   col_kurt    float [heads, NBk]
 *   head_stats  float [heads, batch, 2]: [0] the maximum of col_kurt over the sequence's columns
 *               with at least 4 values (0 if there is none), [1] the excess kurtosis of
 *               col_mean over the sequence's columns that hold a real key (0 for fewer than 4)
 *   workspace   stream_receiver_stats_workspace_bytes(shape) bytes (packed Q and K, one float
 *               per padded token and head), 256-byte aligned
 * The moments are accumulated in fp64 from the fp32 block means.  Errors: as stream_prune;
 * STREAM_EUNSUPPORTED also for dtype F32 with head_dim 128 and b_k = 128.  With STREAM_MASK_ARRAY a
 * query that sees no key has a zero row of probabilities, and a key block no query block sees is
 * no column (col_mean = col_kurt = 0, left out of head_stats).
 */
size_t stream_receiver_stats_workspace_bytes(const stream_shape *shape);

stream_status stream_receiver_stats(const void *Q, const void *K, const stream_shape *shape, float scale,
                                    float *block_mean, float *col_mean, float *col_kurt,
                                    float *head_stats, void *workspace, size_t workspace_bytes,
                                    void *hip_stream);

const char *stream_status_str(stream_status s);

#ifdef __cplusplus
}
#endif
#endif /* STREAM_H_ */
