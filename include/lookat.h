/*
 * lookat.h -- C ABI of the MI355X (gfx950) LOOKAT library.
 *
 * LOOKAT stores every cached attention key as m uint8 codes (product
 * quantisation: the head dimension d_k is cut into m subspaces of d_sub = d_k/m
 * coordinates, each with a codebook of K = 256 centroids) and scores a query
 * against the cache by summing m entries of a per-query lookup table instead of
 * reconstructing keys (asymmetric distance computation).
 *
 * General rules for every call
 *   - All array arguments are DEVICE pointers (HBM of the current HIP device)
 *     unless marked "host".  The caller owns every buffer; the library neither
 *     allocates nor frees device memory and keeps no state between calls except
 *     a thread-local error string.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls validate their arguments on the host, enqueue kernels on `stream`
 *     and return without waiting.  Buffers must stay valid until the stream has
 *     run the work.
 *   - Return value: a lookat_status.  LOOKAT_OK means "enqueued".  On any other
 *     value nothing was enqueued and lookat_last_error() describes the reason.
 *     The library never aborts, prints or throws.
 *   - Arrays are dense row-major with the last index fastest, except where a
 *     stride argument says otherwise.  Strides are in ELEMENTS of the array.
 *   - Inputs are expected to be finite.  In the encoder a NaN distance never
 *     compares below the running minimum (so it never wins unless it is
 *     centroid 0's).
 *   - Supported shapes: K == 256; d_k a multiple of 8 with 8 <= d_k <= 256;
 *     m divides d_k, 1 <= m <= 32.  Anything else: LOOKAT_ERR_UNSUPPORTED or
 *     LOOKAT_ERR_SHAPE.
 */
#ifndef LOOKAT_H
#define LOOKAT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LOOKAT_F16 = 1, /* IEEE binary16 */
    LOOKAT_F32 = 2, /* IEEE binary32 */
    /* Not dtypes.  They give the type the whole range of int, so that the library (built as C++, where an
     * enumeration only holds values up to its largest enumerator's bit width) can test and reject any
     * value a C caller passes: an unknown value returns LOOKAT_ERR_DTYPE. */
    LOOKAT_DTYPE_RANGE_LOW_ = -0x7fffffff - 1,
    LOOKAT_DTYPE_RANGE_HIGH_ = 0x7fffffff
} lookat_dtype;

typedef enum {
    LOOKAT_OK = 0,
    LOOKAT_ERR_NULL = -1,        /* a required pointer is NULL */
    LOOKAT_ERR_SHAPE = -2,       /* non-positive size, m does not divide d_k, stride too small ... */
    LOOKAT_ERR_DTYPE = -3,       /* dtype tag is not LOOKAT_F16 / LOOKAT_F32 */
    LOOKAT_ERR_ALIGN = -4,       /* a pointer or stride breaks the alignment stated below */
    LOOKAT_ERR_WORKSPACE = -5,   /* workspace missing or smaller than *_workspace_bytes() */
    LOOKAT_ERR_UNSUPPORTED = -6, /* valid problem, but outside the shapes this build handles */
    LOOKAT_ERR_HIP = -7          /* the HIP runtime refused a launch; text in lookat_last_error() */
} lookat_status;

/* Problem shape shared by all calls: B batch entries, H heads, head dimension
 * d_k split into m subspaces, K centroids per subspace (must be 256, the
 * codebook size the paper fixes in Sec. 3.4 so that a code is one byte). */
typedef struct {
    int32_t B, H, d_k, m, K;
} lookat_shape;

/*
 * Key encoding (paper Sec. 3.4, "Encoding"):
 *     codes[b,h,n,i] = argmin_c || keys[b,h,n, i*d_sub:(i+1)*d_sub] - codebooks[h,i,c,:] ||^2
 * The squared distance is evaluated in fp64, coordinates in ascending order,
 * with a separately rounded subtract, multiply and add per coordinate (no fused
 * multiply-add); among equal distances the lowest index c wins.  The result is
 * therefore unique and reproducible bit for bit.  (The kernels may rank the centroids
 * with a cheaper product first and evaluate this rule only where the ranking cannot
 * decide; the codes are those of the rule in every case.  Setting the environment
 * variable LOOKAT_ENCODE_EXACT=1 makes every call evaluate the rule for all centroids.)
 *
 *   keys       [B,H,N,d_k]  key_dtype (fp16 or fp32), 16-byte aligned, dense
 *   codebooks  [H,m,K,d_sub] fp32, 16-byte aligned (one set per head)
 *   codes      out; element (b,h,n,i) is written at
 *              codes[(b*H+h)*code_stride_bh + n*m + i]; code_stride_bh >= N*m.
 *              A caller appending to a cache [B,H,Lmax,m] at position p passes
 *              codes = cache + p*m and code_stride_bh = Lmax*m.
 *   N          keys per (b,h), >= 0 (N == 0 is a no-op that returns LOOKAT_OK)
 */
int lookat_encode_keys(const lookat_shape *shape, int64_t N,
                       const void *keys, lookat_dtype key_dtype,
                       const float *codebooks,
                       uint8_t *codes, int64_t code_stride_bh,
                       void *stream);

/*
 * Lookup-table construction (paper Sec. 3.5, "Precomputation Lookup Tables";
 * Algorithm 1, first loop), for T queries per (b,h):
 *     lut[b,h,t,i,c] = sum_j q[b,h,t, i*d_sub + j] * codebooks[h,i,c,j]
 * accumulated in fp32.
 *
 *   q          [B,H,T,d_k]  q_dtype (fp16 or fp32), 16-byte aligned, dense
 *   codebooks  [H,m,K,d_sub] fp32, 16-byte aligned
 *   lut        out [B,H,T,m,K] fp32, 16-byte aligned
 *   T          queries per (b,h), >= 1 (decode: T = 1)
 */
int lookat_build_lut(const lookat_shape *shape, int32_t T,
                     const void *q, lookat_dtype q_dtype,
                     const float *codebooks,
                     float *lut,
                     void *stream);

/*
 * Attention decode over the coded cache (paper Algorithm 1 after the table
 * build: lookup-and-sum scores, softmax, weighted value sum), one query per (b,h):
 *     s[b,h,l]   = sum_i lut[b,h,i, codes[b,h,l,i]]
 *     out[b,h,:] = sum_l softmax_l(scale * s[b,h,:]) * values[b,h,l,:]
 * The sequence is cut into num_splits contiguous ranges per (b,h); each range
 * keeps a running maximum and running sum (online softmax) and the ranges are
 * merged exactly afterwards, so the result does not depend on num_splits beyond
 * fp32 rounding.
 *
 *   L               cached keys per (b,h), >= 1
 *   lut             [B,H,m,K] fp32, 16-byte aligned
 *   codes           element (b,h,l,i) at codes[(b*H+h)*code_stride_bh + l*m + i];
 *                   base pointer and code_stride_bh multiples of m bytes when m is
 *                   2, 4, 8 or 16 (a key's codes are fetched with one load)
 *   values          fp16; element (b,h,l,j) at values[(b*H+h)*value_stride_bh + l*d_k + j];
 *                   base pointer 16-byte aligned, value_stride_bh >= L*d_k
 *   scale           softmax scale (Algorithm 1 uses 1/sqrt(d_k))
 *   num_splits      >= 1, or 0 to let the library choose from the shape
 *   workspace       device scratch of at least
 *                   lookat_attend_decode_workspace_bytes(shape, L, num_splits)
 *                   bytes, 16-byte aligned; may be NULL when that size is 0.
 *                   Contents before and after the call are unspecified.  Two calls
 *                   in flight at once must not share a workspace.
 *   out             [B,H,d_k] fp32, 16-byte aligned
 *   scores_out      optional [B,H,L] fp32: the unscaled scores s (NULL = not stored)
 */
size_t lookat_attend_decode_workspace_bytes(const lookat_shape *shape, int64_t L, int32_t num_splits);

int lookat_attend_decode(const lookat_shape *shape, int64_t L,
                         const float *lut,
                         const uint8_t *codes, int64_t code_stride_bh,
                         const void *values, int64_t value_stride_bh,
                         float scale, int32_t num_splits,
                         void *workspace, size_t workspace_bytes,
                         float *out, float *scores_out,
                         void *stream);

/*
 * lookat_attend_decode for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and error behaviour as lookat_attend_decode, without `workspace`: the
 * per-range partial results live in LOOKAT_NOALLOC_SCRATCH_BYTES of device memory that is part of
 * the library's own image (every GPU the library runs on holds one copy until the process ends;
 * its address is looked up on the first call on a device).  The call allocates and frees nothing.
 *   - Problems that need more than that (B*H*ranges*(d_k+2) floats, see
 *     lookat_attend_decode_workspace_bytes): LOOKAT_ERR_WORKSPACE, nothing enqueued.
 *   - All calls on one GPU share the memory: two calls whose kernels may overlap on one GPU
 *     (different streams, no ordering between them) race.  Calls on one stream do not.
 *   - Nothing in it needs a defined value before a call: every partial result that is read was
 *     written by the same call.
 */
#define LOOKAT_NOALLOC_SCRATCH_BYTES (4 * 1024 * 1024)

int lookat_attend_decode_noalloc(const lookat_shape *shape, int64_t L,
                                 const float *lut,
                                 const uint8_t *codes, int64_t code_stride_bh,
                                 const void *values, int64_t value_stride_bh,
                                 float scale, int32_t num_splits,
                                 float *out, float *scores_out,
                                 void *stream);

/*
 * Attention decode with grouped queries (the combination with grouped-query attention that the
 * paper names as future work, Sec. "Future Work"; sharing of key/value heads: Sec. "Structural
 * Approaches"): `group` consecutive query heads share one key/value head.  Per query head the
 * computation is Algorithm 1 unchanged,
 *     s[b,hq,l]   = sum_i lut[b,hq,i, codes[b, hq/group, l, i]]
 *     out[b,hq,:] = sum_l softmax_l(scale * s[b,hq,:]) * values[b, hq/group, l, :]
 * but the codes and values of a key/value head are streamed once for its `group` query heads.
 * With d_k = 128 and group 4 or 8 the weighted value sum runs on the matrix cores: each softmax
 * weight enters as two fp16 terms (22 bits), the fp16 values exactly, accumulation in fp32; the
 * sum of weights stays an fp32 sum of the unsplit weights.  Other shapes accumulate with fp32
 * multiply-adds as lookat_attend_decode does.
 *
 *   shape           B, H = number of KEY/VALUE heads, d_k, m, K; query heads = H * group
 *   group           1, 2, 4 or 8 (1 forwards to lookat_attend_decode)
 *   lut             [B, H*group, m, K] fp32, 16-byte aligned (tables of query head hq built against
 *                   the codebooks of key/value head hq/group)
 *   codes, values   as in lookat_attend_decode, indexed by key/value head
 *   out             [B, H*group, d_k] fp32;  scores_out: [B, H*group, L] fp32 or NULL
 *   workspace       lookat_attend_decode_gqa_workspace_bytes(shape, group, L, num_splits) bytes
 * Supported: d_k in {64, 128}, m in {2, 4, 8, 16}, group*m tables within the 160 KB of LDS;
 * otherwise LOOKAT_ERR_UNSUPPORTED.  Other rules (ownership, stream, errors) as lookat_attend_decode.
 */
size_t lookat_attend_decode_gqa_workspace_bytes(const lookat_shape *shape, int32_t group, int64_t L, int32_t num_splits);

int lookat_attend_decode_gqa(const lookat_shape *shape, int32_t group, int64_t L,
                             const float *lut,
                             const uint8_t *codes, int64_t code_stride_bh,
                             const void *values, int64_t value_stride_bh,
                             float scale, int32_t num_splits,
                             void *workspace, size_t workspace_bytes,
                             float *out, float *scores_out,
                             void *stream);

/*
 * Fused decode step: the three calls a decode step makes per layer, in one kernel.
 * For every (b,h):
 *   1. the new token's key k_new[b,h,:] is encoded by the rule of lookat_encode_keys and its m
 *      codes are written to row L-1 of the code cache (paper Sec. 3.4 "Encoding");
 *   2. the query's lookup tables are built as in lookat_build_lut (Sec. 3.5), kept on chip;
 *   3. the query attends over the L cached keys as in lookat_attend_decode (Algorithm 1).
 * Results equal those of the three separate calls (codes bit for bit; out within fp32
 * rounding).  Each workgroup re-reads its head's codebook from L2 (where the library pairs two batch
 * entries of a head in one workgroup, see lookat_decode_step_entries_per_workgroup, once for both); with
 * few (b,h) pairs and a long context lookat_decode_step_split, which cuts the sequence into ranges, is faster.
 *
 *   L          cached keys per (b,h) INCLUDING the new one, >= 1
 *   q, k_new   [B,H,d_k], both of type qk_dtype (fp16 or fp32), 16-byte aligned, dense
 *   codes      code cache, element (b,h,l,i) at codes[(b*H+h)*code_stride_bh + l*m + i];
 *              rows 0..L-2 are read, row L-1 is written (its previous content is ignored)
 *   values     value cache as in lookat_attend_decode; row L-1 must already hold the new
 *              token's value
 *   out        [B,H,d_k] fp32
 * Supported shapes: d_k in {64, 128}, m in {2, 4, 8, 16}; others: LOOKAT_ERR_UNSUPPORTED.
 */
int lookat_decode_step(const lookat_shape *shape, int64_t L,
                       const void *q, const void *k_new, lookat_dtype qk_dtype,
                       const float *codebooks,
                       uint8_t *codes, int64_t code_stride_bh,
                       const void *values, int64_t value_stride_bh,
                       float scale,
                       float *out,
                       void *stream);

/* Batch entries one workgroup of lookat_decode_step serves for this problem (host only, no HIP call):
 * 1, or 2 where the library pairs the entries (b, h) and (b + 1, h) so that their head's codebook is
 * fetched once for both (even B, 257..512 (b,h) pairs, and d_k = 64 with m in {2, 4} and L >= 768, or
 * d_k = 128 with m = 4 and L >= 512 or m = 8 and L >= 2048; results do not depend on it, bit for bit).  0 if the shape is invalid or the step has no kernel for it.  Exists so
 * that tests and measurements can state which kernel instance a shape exercises. */
int32_t lookat_decode_step_entries_per_workgroup(const lookat_shape *shape, int64_t L);

/*
 * The fused decode step with the sequence of every (b,h) cut into num_splits ranges, for few
 * (b,h) pairs and long contexts (single-user decode), where one workgroup per (b,h) would leave
 * most of the chip idle.  Same results as lookat_decode_step (Algorithm 1 with the split-K merge
 * of lookat_attend_decode; paper Sec. 3.4 "Encoding", Sec. 3.5): every range's workgroup builds
 * the query's tables, the one that holds position L-1 also encodes and appends the new key, and
 * a second kernel merges the ranges.
 *   num_splits                 ranges per (b,h); 0 = the library's choice (as lookat_attend_decode)
 *   workspace, workspace_bytes device scratch of at least
 *                              lookat_decode_step_split_workspace_bytes(shape, L, num_splits) bytes,
 *                              16-byte aligned, caller-owned; may be NULL when that is 0
 * All other arguments, supported shapes and error behaviour as lookat_decode_step.
 */
size_t lookat_decode_step_split_workspace_bytes(const lookat_shape *shape, int64_t L, int32_t num_splits);

int lookat_decode_step_split(const lookat_shape *shape, int64_t L,
                             const void *q, const void *k_new, lookat_dtype qk_dtype,
                             const float *codebooks,
                             uint8_t *codes, int64_t code_stride_bh,
                             const void *values, int64_t value_stride_bh,
                             float scale, int32_t num_splits,
                             void *workspace, size_t workspace_bytes,
                             float *out,
                             void *stream);

/*
 * The fused decode step for grouped-query attention (paper, "Future Work": grouped-query and
 * multi-query attention; Algorithm 1 per query head, encoding rule of Sec. 3.4 per key/value head):
 * shape->H counts KEY/VALUE heads, query head hq reads the cache of key/value head hq / group.
 * For every (b, key/value head): k_new is encoded and appended at row L-1, the tables of the head's
 * `group` query heads are built from one pass over its codebook and kept on chip, and those query
 * heads attend over the L cached keys; codes and values are read once per group.  Results equal
 * lookat_encode_keys + lookat_build_lut (each query head against its key/value head's codebooks)
 * + lookat_attend_decode_gqa.
 *   q          [B, H*group, d_k]   k_new  [B, H, d_k]   (both of type qk_dtype, 16-byte aligned)
 *   codebooks  [H, m, K, d_sub] fp32;  codes, values: the key/value caches as in lookat_decode_step
 *   out        [B, H*group, d_k] fp32
 *   num_splits, workspace, workspace_bytes: ranges per (b,h) as in lookat_attend_decode_gqa; the
 *              workspace size comes from lookat_decode_step_gqa_workspace_bytes
 * Supported: group in {1, 2, 4, 8}, d_k in {64, 128}, m in {2, 4, 8, 16}, group*m tables plus the
 * reduction buffer within the 160 KB of LDS; otherwise LOOKAT_ERR_UNSUPPORTED.
 */
size_t lookat_decode_step_gqa_workspace_bytes(const lookat_shape *shape, int32_t group, int64_t L, int32_t num_splits);

int lookat_decode_step_gqa(const lookat_shape *shape, int32_t group, int64_t L,
                           const void *q, const void *k_new, lookat_dtype qk_dtype,
                           const float *codebooks,
                           uint8_t *codes, int64_t code_stride_bh,
                           const void *values, int64_t value_stride_bh,
                           float scale, int32_t num_splits,
                           void *workspace, size_t workspace_bytes,
                           float *out,
                           void *stream);

/* The split count lookat_attend_decode uses when num_splits == 0 (host only,
 * no HIP call); 0 if the shape is invalid. */
int32_t lookat_attend_decode_auto_splits(const lookat_shape *shape, int64_t L);

/* The launch shape lookat_attend_decode takes for this problem (host only, no HIP call):
 * *ranges = ranges per (b,h) (num_splits, or the library's choice when it is 0), *wavefronts =
 * wavefronts per workgroup of the kernel instance that streams a range (4 for ranges under
 * 2048 keys and for shapes without a large-workgroup instance, 16 otherwise).  Either pointer
 * may be NULL.  Exists so that tests can state which instance a shape exercises.  Returns a
 * lookat_status. */
int lookat_attend_decode_launch_shape(const lookat_shape *shape, int64_t L, int32_t num_splits,
                                      int32_t *ranges, int32_t *wavefronts);

/*
 * Causal lookup-and-sum scoring of a block of T queries against L >= T coded keys
 * (prefill; paper Sec. 3.5 applied to every query position, as the paper's evaluation does
 * with its T x T attention maps).  The T queries are the last T positions of the cache:
 * query t sits at position t + (L - T) and sees the keys l <= t + (L - T).
 *     scores[b,h,t,l] = sum_i ( sum_j q[b,h,t, i*d_sub + j] * codebooks[h,i, codes[b,h,l,i], j] )
 * for visible l, and -inf elsewhere.  Nothing but `scores` is written: no table and no decoded key
 * leaves the chip.  Two kernels compute it, chosen by shape:
 *   - T >= 24: the double sum is taken as one dense product of the queries with the keys' centroids
 *     (fetched from the codebook by code) on the matrix cores; centroids, and fp32 queries, are scaled
 *     by a power of two and split into two fp16 terms (products exact; the product of two small terms,
 *     2^-22 of a product, is dropped), accumulation in fp32 over all d_k coordinates in the matrix
 *     unit's order;
 *   - T < 24: per-query tables built in LDS and summed by look-up (table entries accumulated in
 *     fp32, the coordinates j in ascending groups of four whose inner order depends on the
 *     centroid; entries then summed in ascending i).
 * Either way |error| stays within 1e-4 of sum_i sum_j |q_j| |c_j|.
 *
 *   q          [B,H,T,d_k] q_dtype (fp16 or fp32), 16-byte aligned, dense
 *   codebooks  [H,m,K,d_sub] fp32, 16-byte aligned
 *   codes      element (b,h,l,i) at codes[(b*H+h)*code_stride_bh + l*m + i], alignment as in
 *              lookat_attend_decode
 *   scores     out [B,H,T,L] fp32 (unscaled), 4-byte aligned
 * Supported shapes: d_k in {64, 128}, m in {2, 4, 8, 16}, L <= 2^30; others:
 * LOOKAT_ERR_UNSUPPORTED.
 */
int lookat_score_prefill(const lookat_shape *shape, int32_t T, int64_t L,
                         const void *q, lookat_dtype q_dtype,
                         const float *codebooks,
                         const uint8_t *codes, int64_t code_stride_bh,
                         float *scores,
                         void *stream);

/*
 * One Lloyd iteration of codebook learning (paper Sec. 3.4, "Prototype Learning":
 * k-means with K = 256 per subspace on a set of calibration keys).  Every calibration
 * sub-vector is assigned to its nearest centroid by the rule of lookat_encode_keys;
 * each centroid then moves to the mean of its members, computed as an fp64 sum in
 * ascending key order, divided by the count and rounded to fp32.  A centroid without
 * members keeps its value.  The result is reproducible bit for bit.
 *
 *   shape          B must be 1 (one calibration set per head)
 *   Nc             calibration keys per head, >= 1
 *   calib          [H,Nc,d_k] fp32, 16-byte aligned
 *   codebooks_in   [H,m,K,d_sub] fp32, 16-byte aligned
 *   codebooks_out  same shape; must not alias codebooks_in
 *   assign         out [H,Nc,m] uint8: the assignment made against codebooks_in
 */
int lookat_kmeans_step(const lookat_shape *shape, int64_t Nc,
                       const float *calib,
                       const float *codebooks_in, float *codebooks_out,
                       uint8_t *assign,
                       void *stream);

/* Host pointer to a thread-local, NUL-terminated description of the last
 * failure on this thread; valid until the next library call on this thread. */
const char *lookat_last_error(void);

/* Library version: major*10000 + minor*100 + patch. */
int lookat_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LOOKAT_H */
