/*
 * scfa.h -- C ABI of the Sparse Causal Flash Attention library for MI355X (gfx950).
 *
 * The library computes exact causal softmax attention restricted to a dynamic
 * sparsity pattern (paper Sec. 3), in two variants:
 *   - hash-sparse (Sec. 3.2): query i may attend key j iff j <= i and
 *     bucket_q[i] == bucket_k[j];
 *   - QK-sparse / QK-dropping (Sec. 3.1): iff j <= i and both are kept.
 * A query with no allowed key outputs a zero vector (Sec. 3.1, "Edge cases");
 * its logsumexp is -inf.
 *
 * Pipeline (one (batch, head) pair is a "segment"; S = B*H segments):
 *   scfa_lsh_buckets                          (optional) bucket ids from the rows, Sec. 4.2
 *   scfa_sort_by_bucket[_pair] / scfa_compact_keep[_pair]
 *                                             stable permutation: original-index vectors, sort keys
 *   scfa_gather_qkv / scfa_gather_rows        permuted / compacted Q, K, V
 *   scfa_block_ranges                         tile-skip schedule (work lists)
 *   scfa_hash_attn_fwd / scfa_qkdrop_attn_fwd O and logsumexp, written in ORIGINAL order
 *   scfa_hash_attn_bwd / scfa_qkdrop_attn_bwd dQ, dK, dV, written in ORIGINAL order
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless it is marked "host".
 *   - Tensors are contiguous: Q/K/V/O/dO [B,H,T,d] (= [S,T,d]); per-token
 *     vectors [B,H,T] (= [S,T]).  T_Q == T_KV == T.
 *   - The caller owns every buffer.  The library never allocates or frees
 *     device memory and never synchronises: all work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL is the default stream).
 *   - Outputs are fully written (zeros for dropped / stranded rows); callers
 *     need not clear them.
 *   - Every function returns SCFA_OK or a negative error code; nothing is
 *     launched when an argument check fails.  No function throws or aborts.
 *   - `flags`: 0, or SCFA_FLAG_STRICT_CAUSAL: a query attends keys at STRICTLY earlier
 *     positions only (App. B.1: ">=" replaced by ">", the form used with shared
 *     query / key projections).  The same flag must be given to scfa_block_ranges and to
 *     the attention calls that consume its work lists.  The first token of every bucket
 *     (or the first kept token) then has no allowed key: zero output row, LSE = -inf.
 */
#ifndef SCFA_H
#define SCFA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SCFA_OK            0
#define SCFA_EINVAL       (-1)  /* null pointer, non-positive size, bad alignment, bad value */
#define SCFA_EUNSUPPORTED (-2)  /* dtype / head dim / nb / tile size outside the built set */
#define SCFA_EWORKSPACE   (-3)  /* workspace too small */
#define SCFA_EHIP         (-4)  /* a HIP runtime call failed; see scfa_last_hip_error() */

#define SCFA_BF16 0             /* 16-bit brain float, fp32 accumulation */
#define SCFA_F32  1             /* fp32 (forward only) */
#define SCFA_F16  2             /* compute format of the permuted copies of bf16 tensors */

#define SCFA_HASH   0
#define SCFA_QKDROP 1

#define SCFA_FLAG_STRICT_CAUSAL 1   /* allowed keys are at strictly earlier positions */

#define SCFA_MAX_BUCKETS 256
#define SCFA_MAX_T 16777200     /* positions take the low 24 bits of a sort key.  Effective limits are lower:
                                 * scfa_block_ranges needs ceil(T / 128) + nb <= 8192 (T of about one million:
                                 * its ranking scratch lives in LDS), and the attention entry points need
                                 * T * d * sizeof(element) < 2^31 (byte offsets inside a segment are 32-bit);
                                 * both return SCFA_EUNSUPPORTED beyond that. */
#define SCFA_WORK_STRIDE 8      /* int32 words per work item */

/* Library version (major*10000 + minor*100 + patch). */
int scfa_version(void);

/* hipError_t value of the last failed HIP call made by this library on the
 * calling thread (0 if none). */
int scfa_last_hip_error(void);

/* Human-readable name of an SCFA_* error code (static string, host). */
const char *scfa_error_string(int code);

/* ------------------------------------------------------------------------
 * a1. Stable sort of token positions by bucket id, per segment (Sec. 3.2:
 * the rows of Q, K and V are brought into bucket order along the sequence dimension; the
 * sort must be stable so that original positions stay increasing inside a
 * bucket).
 *
 *   bucket             [S,T] int32, 0 <= bucket < nb (ids outside the range are
 *                      clamped into it so the call stays memory-safe)
 *   idx_out            [S,T] int32: idx_out[s,r] = original position of sorted row r;
 *                      (bucket[idx[r]], idx[r]) is lexicographically increasing
 *   bucket_sorted_out  [S,T] int32 (nullable): bucket id of sorted row r
 *   bucket_off_out     [S,nb+1] int32: off[s,b] = number of tokens with id < b
 *   sort_key_out       [S,T] uint32 (nullable; needs T <= SCFA_MAX_T): the pair the rows
 *                      are ordered by, packed as bucket << 24 | position; increasing
 *                      along r.  The hash-sparse attention entry points take these: "same
 *                      bucket and position <= p" is one range test on them.
 *   ws, ws_bytes       (nullable) device scratch of scfa_sort_workspace_bytes(S, T, nb)
 *                      bytes, 4-byte aligned, contents undefined afterwards.  Long
 *                      sequences (T >= 8192) in few segments are cut into chunks that
 *                      several workgroups sort.  Up to T = 16384 every workgroup counts
 *                      the keys of the other chunks itself and the scratch is not touched;
 *                      beyond that a counting kernel runs first and writes its counters
 *                      here, and without the scratch, or when it is too small, one
 *                      workgroup sorts a segment.  The outputs are the same bits either way.
 * Limits: 1 <= nb <= SCFA_MAX_BUCKETS, 1 <= T, 1 <= S.
 */
size_t scfa_sort_workspace_bytes(int S, int T, int nb);   /* also for the compaction (any nb) */

int scfa_sort_by_bucket(const int32_t *bucket, int S, int T, int nb,
                        int32_t *idx_out, int32_t *bucket_sorted_out,
                        int32_t *bucket_off_out, uint32_t *sort_key_out,
                        void *ws, size_t ws_bytes, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): scfa_sort_by_bucket with the chunk
 * counters of the multi-workgroup sort in a device array the library itself owns, instead
 * of a caller workspace.  Arguments and outputs as scfa_sort_by_bucket (same bits).  The
 * call allocates and frees nothing and creates no events (the scfa_prof_* timers skip it);
 * its first call on a device looks the array's address up once, with that device current.
 * `stream` must belong to the current device (SCFA_EINVAL otherwise).
 * Limit: scfa_sort_workspace_bytes-worth of counters, 4 * S * chunks * nb bytes (chunks =
 * min(ceil(256 / S), T / 4096, 64) for T >= 8192, else none), must not exceed
 * SCFA_STATIC_SCRATCH_BYTES; larger problems return SCFA_EWORKSPACE and launch nothing.
 * Every device the library runs on holds the array until the process ends.  All calls on
 * one device share it: calls that may overlap on one device (different streams, or threads)
 * race on the counters and must be serialised by the caller. */
#define SCFA_STATIC_SCRATCH_BYTES (256 * 1024)
int scfa_sort_by_bucket_static(const int32_t *bucket, int S, int T, int nb,
                               int32_t *idx_out, int32_t *bucket_sorted_out,
                               int32_t *bucket_off_out, uint32_t *sort_key_out,
                               void *stream);

/* Validating mode for the bucket ids (Sec. 3.2 takes ids in [0, nb) for granted; the sort
 * clamps what lies outside so that it stays memory-safe, which hides a caller's mistake):
 * counts the entries of `bucket` outside [0, nb).
 *
 *   bucket         [n] int32 (device), any shape flattened
 *   n_invalid_out  [1] int32 (device): overwritten with the count (0 = every id is valid);
 *                  the caller reads it when it wants to, the call does not synchronise
 * Errors: SCFA_EINVAL for null pointers or n < 0; nb as for the sort.
 */
int scfa_count_invalid_buckets(const int32_t *bucket, long long n, int nb,
                               int32_t *n_invalid_out, void *stream);

/* The same sort for the query and the key bucket ids of one attention call in ONE
 * launch (Sec. 3.2 sorts both); outputs as above, one set per side.  The *_sorted_out
 * and *_sort_key_out pointers are nullable. */
int scfa_sort_by_bucket_pair(const int32_t *bucket_q, const int32_t *bucket_k,
                             int S, int T, int nb,
                             int32_t *q_idx_out, int32_t *q_sorted_out, int32_t *q_off_out,
                             uint32_t *q_sort_key_out,
                             int32_t *k_idx_out, int32_t *k_sorted_out, int32_t *k_off_out,
                             uint32_t *k_sort_key_out,
                             void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------
 * a0. LSH bucketing, the step in front of the hash-sparse path (Sec. 4.2 "Hashing
 * mechanism": the cross-polytope scheme of Andoni et al. with a chosen number of hash
 * codes).  For every row x[s,t,:] and the projection R[h] of its head h = s % H:
 *     bucket[s,t] = argmax over the 2r values [x R[h], -x R[h]],  r = nb / 2,
 * the lowest index winning a tie, i.e. a value in [0, nb).
 *
 *   x_q, x_k    [S,T,d] SCFA_BF16 or SCFA_F32; x_k (and bucket_k_out) may be NULL: one tensor
 *   R           [H,d,r] float32, row-major (d rows of r columns per head)
 *   bucket_*_out [S,T] int32
 * The projections are formed in fp32; a row whose two largest candidates differ by less
 * than fp32 rounding of the dot products may land on either of them.
 * Limits: nb even, 2 <= nb <= SCFA_MAX_BUCKETS, d in {64, 128}, S % H == 0, d * r * 4 <= 64 KiB.
 */
int scfa_lsh_buckets(const void *x_q, const void *x_k, const float *R,
                     int S, int H, int T, int d, int nb, int dtype,
                     int32_t *bucket_q_out, int32_t *bucket_k_out, void *stream);

/* ------------------------------------------------------------------------
 * a2. Compaction for QK-dropping (Sec. 3.1, "Shrinking the attention matrix").
 *
 *   keep       [S,T] uint8, non-zero = kept
 *   idx_out    [S,T] int32: first count[s] entries = kept positions, increasing;
 *              the remaining entries = dropped positions, increasing (the order a
 *              stable descending sort of the keep flag gives)
 *   count_out  [S] int32: number of kept tokens
 *   ws, ws_bytes  (nullable) scratch as for scfa_sort_by_bucket
 */
int scfa_compact_keep(const uint8_t *keep, int S, int T,
                      int32_t *idx_out, int32_t *count_out,
                      void *ws, size_t ws_bytes, void *stream);

/* Query and key keep flags of one attention call compacted in ONE launch. */
int scfa_compact_keep_pair(const uint8_t *keep_q, const uint8_t *keep_k, int S, int T,
                           int32_t *q_idx_out, int32_t *n_q_out,
                           int32_t *k_idx_out, int32_t *n_k_out,
                           void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------
 * a3. Row gather: out[s,r,:] = x[s, idx[s,r], :] for r < n[s], where n[s] =
 * count[s] if `count` is non-null, else T.  Rows r >= n[s] of `out` are not
 * touched.  `out` has the same [S,T,d] capacity as `x` (Sec. 3: the permuted /
 * compacted Q, K, V the kernels consume).  x and out must be 16-byte aligned
 * and must not overlap.  dtype: SCFA_BF16 or SCFA_F32; d*sizeof(elem) must be a
 * multiple of 16.
 * out_dtype: equal to dtype, or SCFA_F16 for SCFA_BF16 input: the compute format of
 * the attention kernels.  bf16 -> fp16 rounds to nearest even (IEEE): exact for
 * magnitudes in [2^-17, 65504], smaller ones lose low bits (absolute error < 2^-25),
 * larger ones become +-inf and NaN stays NaN -- an input outside the compute format then
 * shows as non-finite attention outputs instead of being replaced by a finite value.
 * scale: every element is multiplied by `scale` in fp32 and the product is then
 * converted to out_dtype.  scale == 1 with out_dtype == dtype is a bit-exact copy; bf16 -> bf16
 * with another scale is SCFA_EUNSUPPORTED.  The attention entry points expect
 * queries, keys and values gathered with scale 1 (the inputs' own values).
 */
int scfa_gather_rows(const void *x, const int32_t *idx, const int32_t *count,
                     int S, int T, int d, int dtype, int out_dtype, float scale,
                     void *out, void *stream);

/* Q, K and V of one attention call gathered in ONE launch: q_out = q_scale * q[q_idx]
 * (rows < n_q[s]), k_out = k[k_idx], v_out = v[k_idx] (rows < n_k[s]); n_q / n_k
 * nullable (= T).  Same dtype rules as scfa_gather_rows; pass q_scale = 1 for the
 * attention entry points. */
int scfa_gather_qkv(const void *q, const void *k, const void *v,
                    const int32_t *q_idx, const int32_t *k_idx,
                    const int32_t *n_q, const int32_t *n_k,
                    int S, int T, int d, int dtype, int out_dtype, float q_scale,
                    void *q_out, void *k_out, void *v_out, void *stream);

/* ------------------------------------------------------------------------
 * a4. Tile-skip schedule.  The paper finds, per block of queries, the range of
 * key blocks that can hold an allowed pair (Sec. 3.1 j_stop; Sec. 3.2 j_start,
 * j_stop and its causal refinement).  This library owns its tiling, so it
 * anchors tiles at bucket boundaries: a work item covers query rows of ONE
 * bucket and the keys of that same bucket, so the bucket test is structural
 * and only the causal test on original positions remains inside a tile.
 * Buckets with fewer rows than a tile are the exception: consecutive ones are
 * put together into one item (as many whole buckets as fit a tile of the
 * tiled side) that spans all their queries and all their keys; inside such an
 * item every tile takes the bucket and the causal test.
 *
 * Tile sizes must be the ones scfa_tile_config() reports for (d, dtype).
 *
 *   variant     SCFA_HASH: q_off/k_off are the [S,nb+1] offsets of
 *               scfa_sort_by_bucket.  SCFA_QKDROP: nb must be 1 and q_off/k_off
 *               are the [S] kept counts of scfa_compact_keep.
 *   q_idx,k_idx [S,T] original positions of the permuted rows
 *
 *   fwd_work_out [S, n_fwd, 8] int32, n_fwd = scfa_num_work_items(T, nb, fwd_tile_m).
 *     Item = { q_begin, q_count, k_begin, k_count, k_nomask, bucket, n_buckets, 0 }:
 *     permuted query rows [q_begin, q_begin+q_count) attend permuted key rows
 *     [k_begin, k_begin+k_count): the keys of the same bucket whose position is
 *     <= the LARGEST query position of the item.  The first k_nomask of these
 *     keys have a position <= the SMALLEST query position: no mask needed.
 *     n_buckets > 1: all rows of buckets [bucket, bucket + n_buckets) on both
 *     sides, k_nomask = 0.
 *     Items of a segment are ordered by bucket pair (bucket / 2) and, inside a pair,
 *     by decreasing k_count; unused trailing items have q_count == 0.
 *   bwd_work_out [S, n_bwd, 8] int32 (nullable), n_bwd = scfa_num_work_items(T, nb, bwd_tile_n).
 *     Item = { k_begin, k_count, q_begin, q_count, q_masked, bucket, n_buckets, 0 }:
 *     permuted key rows [k_begin, k_begin+k_count) are attended by permuted
 *     query rows [q_begin, q_begin+q_count): the queries of the same bucket
 *     whose position is >= the SMALLEST key position of the item.  Only the
 *     first q_masked of them (position < the LARGEST key position) need a mask.
 *     n_buckets > 1: all rows of those buckets on both sides, q_masked = q_count.
 *     Ordered by bucket pair and, inside a pair, by decreasing q_count.
 *   counters_out [S,4] int64 (nullable): { forward tiles of fwd_tile_m x fwd_tile_n,
 *     sum of q_count*k_count, backward tiles of bwd_tile_m x bwd_tile_n, sum of
 *     k_count*q_count } -- the "computed tile" counts throughput is quoted on.
 */
int scfa_block_ranges(int variant, const int32_t *q_idx, const int32_t *k_idx,
                      const int32_t *q_off, const int32_t *k_off,
                      int S, int T, int nb,
                      int fwd_tile_m, int fwd_tile_n, int bwd_tile_n, int bwd_tile_m,
                      int flags,
                      int32_t *fwd_work_out, int32_t *bwd_work_out,
                      int64_t *counters_out, void *stream);

/* Number of work items per segment for a tiling of `tile` rows: ceil(T/tile) + nb
 * (an upper bound of sum_b ceil(n_b/tile)).  Host arithmetic only. */
int scfa_num_work_items(int T, int nb, int tile);

/* Tile sizes the attention kernels are built for (host out-pointers).
 * Returns SCFA_EUNSUPPORTED for an unsupported (d, dtype). */
int scfa_tile_config(int d, int dtype, int *fwd_tile_m, int *fwd_tile_n,
                     int *bwd_tile_n, int *bwd_tile_m);

/* ------------------------------------------------------------------------
 * a5 (+a8). Forward attention over the scheduled tiles (Sec. 3.1 / 3.2; the
 * per-tile work of Alg. 1 / Alg. 2: scores, bucket and causal mask, online softmax
 * with the NaN-safe handling of fully masked rows, P.V).
 *
 *   q_perm,k_perm,v_perm  [S,T,d] rows in sorted (hash) or compacted (qkdrop) order, as
 *                         scfa_gather_rows writes them: fp32 for SCFA_F32, fp16
 *                         (out_dtype = SCFA_F16) for SCFA_BF16, all gathered with scale 1
 *   q_sort_key,k_sort_key [S,T] sort keys of those rows (scfa_sort_by_bucket's sort_key_out);
 *                         the QK-dropping entry points take the compacted index vectors
 *                         q_idx, k_idx themselves (one bucket, id 0: position = sort key)
 *   T                     at most SCFA_MAX_T
 *   fwd_work, n_fwd       work list of scfa_block_ranges
 *   sm_scale              tau > 0 (the paper's default is 1/sqrt(d))
 *   o_out                 [B,H,T,d] in ORIGINAL order, dtype of the inputs
 *   lse_out               [B,H,T] float, ORIGINAL order: natural-log logsumexp of the
 *                         scaled scores over allowed keys; -inf for a row with none
 *   o_f16_out             [B,H,T,d] fp16 (nullable, SCFA_BF16 only): the same O rounded to fp16
 *                         (11 significant bits instead of bf16's 8), for the backward's
 *                         D = <dO, O>; pass it to the backward as o_f16.  Rows of dropped
 *                         queries are not written.
 * d: 64 or 128.  SCFA_BF16: the permuted copies are fp16 (the bf16 values themselves for
 * magnitudes in [2^-17, 65504]); scores are fp16 x fp16 products on the matrix cores,
 * exact, accumulated in fp32; the softmax runs in fp32; P is rounded to fp16 for P.V, which
 * accumulates in fp32.  Finite inputs of any scale inside that range are handled (the
 * logsumexp is exact to fp32 rounding whatever the size of the logits).
 *
 * scfa_qkdrop_attn_fwd additionally takes the kept-query counts n_q [S] and
 * writes zeros / -inf for the dropped query rows idx[n_q[s] .. T).
 */
int scfa_hash_attn_fwd(const void *q_perm, const void *k_perm, const void *v_perm,
                       const uint32_t *q_sort_key, const uint32_t *k_sort_key,
                       const int32_t *fwd_work, int n_fwd,
                       int B, int H, int T, int d, int dtype, float sm_scale, int flags,
                       void *o_out, float *lse_out, void *o_f16_out, void *stream);

int scfa_qkdrop_attn_fwd(const void *q_c, const void *k_c, const void *v_c,
                         const int32_t *q_idx, const int32_t *k_idx, const int32_t *n_q,
                         const int32_t *fwd_work, int n_fwd,
                         int B, int H, int T, int d, int dtype, float sm_scale, int flags,
                         void *o_out, float *lse_out, void *o_f16_out, void *stream);

/* ------------------------------------------------------------------------
 * a6 + a7 (+a8). Backward.  The paper states the backward is adapted like the
 * forward (Sec. 3.1, 3.2: iterate over query blocks per key block); the
 * gradients are those of the masked softmax attention:
 *   D_i = <dO_i, O_i>, P_ij = exp(tau s_ij - LSE_i), dS_ij = P_ij (<dO_i,V_j> - D_i),
 *   dQ_i = tau sum_j dS_ij K_j,  dK_j = tau sum_i dS_ij Q_i,  dV_j = sum_i P_ij dO_i.
 *
 *   o, lse        outputs of the forward (ORIGINAL order)
 *   o_f16         (nullable) the forward's o_f16_out; when given, D is computed from it
 *                 instead of the bf16-rounded o (tighter gradients), and o may be NULL
 *   d_o           [B,H,T,d] upstream gradient, ORIGINAL order, dtype of the inputs
 *   dq_out, dk_out, dv_out   [B,H,T,d] FLOAT32, ORIGINAL order; rows of dropped or
 *                 stranded queries (dQ) and of dropped or never-attended keys
 *                 (dK, dV) are written as zeros
 *   ws, ws_bytes  scratch of at least scfa_attn_bwd_workspace_bytes(S,T,d,dtype),
 *                 256-byte aligned; contents are undefined afterwards
 * q_perm, k_perm, v_perm, sm_scale as in the forward: the scores are recomputed from the same
 * exact products and scaled per element in fp32.  dtype: SCFA_BF16 only.
 * Range of the backward (beyond it the gradients of the rows concerned are NON-FINITE, not
 * finite and wrong): per query the kernels hold LSE / tau and D * (power-of-two dO scale, largest
 * |dO| of the segment in [1, 2)) as sums of three fp16 numbers, which reach |LSE| / tau < 2.09e6
 * (logits of +-2.6e5 at tau = 1/8) and |D| < 65504 (|D| <= 2 d max|O|: |O| in the hundreds);
 * dS = P (dP - D) is formed in fp16: |<dO_i, V_j> - D_i| must stay below 65504, i.e. |V| in the
 * hundreds at the least.  A softmax that is one-hot to fp32 precision (logits in the tens of
 * thousands) has dS = P (dP - D) with dP = D up to rounding: its gradients are cancellation
 * noise of relative size 2^-11 against |dO| |V| |K| tau, not against their own (vanishing) size.
 *
 * scfa_qkdrop_attn_bwd additionally takes n_q, n_k [S] (kept counts).
 */
size_t scfa_attn_bwd_workspace_bytes(int S, int T, int d, int dtype);

int scfa_hash_attn_bwd(const void *q_perm, const void *k_perm, const void *v_perm,
                       const uint32_t *q_sort_key, const uint32_t *k_sort_key,
                       const int32_t *fwd_work, int n_fwd,
                       const int32_t *bwd_work, int n_bwd,
                       const void *o, const void *o_f16, const float *lse, const void *d_o,
                       int B, int H, int T, int d, int dtype, float sm_scale, int flags,
                       float *dq_out, float *dk_out, float *dv_out,
                       void *ws, size_t ws_bytes, void *stream);

int scfa_qkdrop_attn_bwd(const void *q_c, const void *k_c, const void *v_c,
                         const int32_t *q_idx, const int32_t *k_idx,
                         const int32_t *n_q, const int32_t *n_k,
                         const int32_t *fwd_work, int n_fwd,
                         const int32_t *bwd_work, int n_bwd,
                         const void *o, const void *o_f16, const float *lse, const void *d_o,
                         int B, int H, int T, int d, int dtype, float sm_scale, int flags,
                         float *dq_out, float *dk_out, float *dv_out,
                         void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------
 * Per-kernel timing with HIP events on the caller's stream (measurement aid).
 * While enabled, every kernel launch of the library is bracketed by two
 * events.  scfa_prof_read synchronises on the recorded events.
 *   kernel ids: see SCFA_K_* below.
 */
#define SCFA_K_SORT        0
#define SCFA_K_COMPACT     1
#define SCFA_K_GATHER      2
#define SCFA_K_RANGES      3
#define SCFA_K_FWD         4
#define SCFA_K_BWD_PREP    5
#define SCFA_K_BWD_DKDV    6
#define SCFA_K_BWD_DQ      7
#define SCFA_K_FILL        8
#define SCFA_K_LSH         9
#define SCFA_K_COUNT       10

int scfa_prof_enable(int on);      /* returns the previous state */
int scfa_prof_reset(void);
/* total_ms / launches (host out-pointers) accumulated since the last reset */
int scfa_prof_read(int kernel_id, double *total_ms, int *launches);
/* Workgroups of an attention kernel (SCFA_K_FWD, SCFA_K_BWD_DKDV, SCFA_K_BWD_DQ; bf16 path,
 * head dimension d) that one compute unit of the current device holds at once, as the HIP
 * runtime computes it from the kernel's registers and LDS (host out-pointer). */
int scfa_prof_occupancy(int kernel_id, int d, int *workgroups_per_cu);

#ifdef __cplusplus
}
#endif
#endif /* SCFA_H */
