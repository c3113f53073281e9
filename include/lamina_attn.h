/*
 * lamina_attn.h -- C ABI of the MI355X (gfx950) decode attention operator.
 *
 * The operator is the attention step that model-attention disaggregation places on the
 * memory-optimised device that owns the KV cache (paper Sec. 3.1, Sec. 2.2.2): per
 * decode iteration and layer it receives one query vector per in-flight request and
 * query head, and returns one output vector per request and query head,
 *
 *     out[r][h] = sum_j softmax_j( scale * <q[r][h], K[r][g][j]> ) * V[r][g][j],
 *     j = 0 .. seq_lens[r]-1,   g = h div G,   G = num_q_heads / num_kv_heads
 *
 * (Sec. 2.1, the starred equation; grouped-query attention as in Sec. 2.2.2: the G query
 * heads of a group read the same K/V and their outputs are concatenated), together with
 * lse[r][h] = ln sum_j exp(scale * <q, K_j>), the natural logarithm of the softmax
 * denominator S_q(I) of Sec. 4.2.2, so that results over disjoint token sets can be
 * combined by the divide-and-conquer identity of that section.
 *
 * All tensor pointers are DEVICE pointers owned by the caller; the library never frees
 * or reallocates them and never copies them to the host.  Calls only enqueue kernels on
 * the given HIP stream and return; they do not synchronise.  Functions return LAMINA_OK
 * (0) or a negative error code; nothing aborts and no C++ exception crosses the ABI.
 */
#ifndef LAMINA_ATTN_H
#define LAMINA_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lamina_attn *lamina_attn_t;            /* opaque handle */

enum {
    LAMINA_OK              =  0,
    LAMINA_ERR_INVALID_ARG = -1,   /* NULL/ill-formed argument; nothing was launched      */
    LAMINA_ERR_UNSUPPORTED = -2,   /* well-formed but outside what the kernels cover      */
    LAMINA_ERR_HIP         = -3,   /* a HIP runtime call failed; see lamina_attn_last_error */
    LAMINA_ERR_WORKSPACE   = -4    /* the split-KV workspace could not be allocated       */
};

enum { LAMINA_BF16 = 0, LAMINA_FP8_E4M3 = 1, LAMINA_F32 = 2 };

/*
 * Fixed properties of one attention layer-share, given at creation.
 * head_dim must be 128.  num_q_heads must be a multiple of num_kv_heads and the group
 * size G = num_q_heads / num_kv_heads must be one of 1, 2, 4, 8, 16.
 */
typedef struct {
    int32_t num_q_heads;
    int32_t num_kv_heads;
    int32_t head_dim;
    int32_t kv_dtype;       /* LAMINA_BF16, or LAMINA_FP8_E4M3 (OCP e4m3fn bytes + fp32 scales) */
    int32_t out_dtype;      /* LAMINA_BF16 or LAMINA_F32                                        */
    int32_t block_size;     /* 0: contiguous strided cache; 16: paged cache with a block table  */
    int32_t max_batch;      /* upper bound on `batch` of any call; sizes grid and workspace     */
    int32_t max_seq_len;    /* upper bound on any seq_lens[r] (larger values are clamped to it) */
    int32_t num_splits;     /* how the KV range of a (request, kv head) row is cut (split-KV):
                               1: never; N>1: into N partitions of ceil(max_seq_len / N) tokens
                               (rounded up to a multiple of 256), each processed on its own;
                               0: the library decides, normally "balanced": per call, from seq_lens,
                               every work-group (one per compute unit) gets a fixed share of the
                               call's work (tokens in blocks of 128, or 256 for fp8, plus one
                               block per row for its fixed cost; shares are equal, except that
                               from 12 blocks per work-group
                               on the even-numbered work-groups take 1/32, from 48 blocks on 1/16
                               more and the odd-numbered ones as much less: they run on dies of
                               different speed) and a row is cut only where one share ends and
                               the next begins                                                   */
    float   softmax_scale;  /* 0 means 1/sqrt(head_dim)                                         */
    int32_t device;         /* HIP device ordinal the handle is bound to                        */
} lamina_attn_config;

/*
 * Per-call arguments that are not tensors.  Strides are in ELEMENTS of the cache dtype;
 * the innermost (head_dim) stride is always 1 and every row start must be 16-byte aligned.
 */
typedef struct {
    int32_t batch;               /* R: requests in this call, 0 <= R <= max_batch              */
    int64_t kv_stride_req;       /* contiguous mode: distance between requests                 */
    int64_t kv_stride_head;      /* contiguous mode: distance between kv heads                 */
    int64_t kv_stride_tok;       /* contiguous mode: distance between tokens (>= head_dim)     */
    int64_t pool_stride_block;   /* paged mode: distance between pool blocks                   */
    int64_t pool_stride_head;    /* paged mode: distance between kv heads inside a block;
                                    tokens of one (block, head) are block_size rows of head_dim */
    int32_t block_table_stride;  /* paged mode: entries per request row of block_table         */
    const float *k_scale;        /* device [R][num_kv_heads]; fp8 only, else NULL              */
    const float *v_scale;        /* device [R][num_kv_heads]; fp8 only, else NULL              */
    void *stream;                /* hipStream_t; NULL = the default stream                     */
} lamina_call_params;

/*
 * Create a handle for one layer-share on cfg->device.  Validates cfg, picks the partitioning
 * and allocates the handle-owned workspace for partial results (see
 * lamina_attn_workspace_bytes; nothing when rows are never cut).
 * On success *out_handle is set.  Errors: INVALID_ARG (NULL, non-positive sizes,
 * num_q_heads % num_kv_heads != 0, unknown dtype), UNSUPPORTED (head_dim != 128,
 * block_size not in {0, 16}, group size not in {1,2,4,8,16}, num_splits > 1 with
 * max_batch > 1024, max_batch * num_kv_heads * partitions per row above 2^30), HIP, WORKSPACE.
 * With num_splits == 0 and max_batch > 1024 rows are never cut.
 */
int lamina_attn_create(const lamina_attn_config *cfg, lamina_attn_t *out_handle);

/*
 * One decode-attention call (Sec. 2.1 starred equation per request and head; split-KV
 * partials merged by the identity of Sec. 4.2.2 when the handle uses more than one
 * partition).
 *
 *   q            device bf16  [R][num_q_heads][128], dense
 *   k_cache      device; contiguous mode: rows K[r][g][j][0..127] at
 *                r*kv_stride_req + g*kv_stride_head + j*kv_stride_tok;
 *                paged mode: pool, token j of request r lives in pool block
 *                block_table[r][j / 16] at row j % 16:
 *                blk*pool_stride_block + g*pool_stride_head + (j%16)*128
 *   v_cache      device; same dtype and layout as k_cache
 *   seq_lens     device int32 [R]: tokens to attend, INCLUDING the token being decoded
 *                (whose k, v the caller has already written).  Never read by the host; a value
 *                above max_seq_len (or, paged, above 16 * block_table_stride) is treated as
 *                that limit, a negative one as 0, so a bad length cannot cause a read outside
 *                the cache extent the call was given.
 *   block_table  device int32 [R][block_table_stride]; only entries below
 *                ceil(seq_lens[r]/16) are read.  NULL in contiguous mode.
 *   out          device [R][num_q_heads][128] of out_dtype, dense
 *   lse          device fp32 [R][num_q_heads], or NULL if not wanted
 *
 * fp8 caches hold OCP e4m3fn bytes; the value of an element is decode(byte) * k_scale[r][g]
 * (resp. v_scale[r][g]).  Rows at or beyond seq_lens[r], the tail of a request's last
 * block and unreferenced pool blocks may hold anything (including NaN patterns).
 * seq_lens[r] == 0 gives out[r] = 0 and lse[r] = -inf.
 *
 * Errors (nothing is launched): INVALID_ARG for a NULL handle/params/required pointer,
 * batch < 0 or > max_batch, paged mode without block_table, fp8 without scales, strides
 * that break the alignment rule; HIP if a launch fails.  batch == 0 is a no-op.
 * One handle must not be used from two streams at once (they would share the workspace).
 */
int lamina_decode_attention(lamina_attn_t h,
                            const void *q,
                            const void *k_cache,
                            const void *v_cache,
                            const int32_t *seq_lens,
                            const int32_t *block_table,
                            void *out,
                            float *lse,
                            const lamina_call_params *p);

/* Free the handle and its workspace.  NULL is accepted.  Does not synchronise: the caller
 * makes sure no call on this handle is still running. */
int lamina_attn_destroy(lamina_attn_t h);

/* Message for the last error on this handle (or, with h == NULL, for the last failed
 * lamina_attn_create on this thread).  Owned by the library; valid until the next call. */
const char *lamina_attn_last_error(lamina_attn_t h);

/* Bytes of device workspace a handle made from cfg would own, or 0 if cfg is invalid or rows are
 * never cut.  It holds one partial result (G x (head_dim + 1) fp32) per piece a call can produce
 * -- max_batch * num_kv_heads * N pieces plus max_batch + 1 int32 prefix sums for fixed
 * partitions; 2048 pieces (two per work-group of the largest grid) plus 16 KiB of per-work-group
 * records for balanced shares, whatever the batch.  Does not touch the GPU. */
size_t lamina_attn_workspace_bytes(const lamina_attn_config *cfg);

/* Partitioning chosen at creation.  lamina_attn_num_splits: 1 = rows are never cut, N > 1 = fixed
 * partitions, 0 = balanced shares decided per call.  lamina_attn_split_tokens: tokens per fixed
 * partition, or the granularity of balanced shares (128 tokens for bf16, 256 for fp8 caches), or
 * 0 when rows are never cut. */
int lamina_attn_num_splits(lamina_attn_t h);
int lamina_attn_split_tokens(lamina_attn_t h);

/* Number of per-query-head partial results ((head_dim + 1) fp32 each, written once by the main
 * pass and read once by the merge) that a call with these lengths produces on this handle: rows
 * that are not cut produce none.  For callers that account for the operator's memory traffic.
 * host_seq_lens is a HOST array of `batch` lengths; nothing touches the GPU.  Returns a negative
 * error code for a NULL argument or batch outside [0, max_batch]. */
int64_t lamina_attn_count_partials(lamina_attn_t h, const int32_t *host_seq_lens, int32_t batch);

/*
 * The two steps either side of the hot path on the attention device when the new token's
 * k, v arrive after its q (Sec. 4.2.2, "resource utilization overlapping": the token set
 * is split into all previous tokens and the newly generated one; [A_q(prev), S_q(prev)] is
 * computed as soon as q is there -- that is lamina_decode_attention with seq_lens counting
 * the previous tokens only, fp32 output and lse -- and k_n, v_n are folded in afterwards).
 *
 * lamina_append_kv writes the new token's rows into the cache:
 *   k_new, v_new  device bf16 [R][num_kv_heads][128], dense
 *   positions     device int32 [R]: token index the rows go to (normally the request's
 *                 previous length); in paged mode block_table[r][positions[r] / 16] must
 *                 already name the destination block
 *   k_cache, v_cache, block_table, p: as for lamina_decode_attention (p->k_scale / v_scale
 *                 are required for fp8 caches: the quotient x / scale is formed in fp32 by a
 *                 correctly rounded IEEE division, clamped to +-448 and rounded to nearest even
 *                 on the e4m3fn grid)
 * positions[r] < 0 skips request r; so does a position at or beyond max_seq_len (paged: beyond
 * the block table row, or in a block whose table entry is negative).  Nothing else in the cache
 * is touched.
 *
 * lamina_fold_new_token combines a result over the previous tokens with the single new token:
 *   q             device bf16 [R][num_q_heads][128]
 *   k_new, v_new  device bf16 [R][num_kv_heads][128]
 *   out_prev      device fp32 [R][num_q_heads][128], lse_prev device fp32 [R][num_q_heads]:
 *                 A_q(prev) and ln S_q(prev); lse_prev = -inf (no previous tokens) is allowed
 *   out           device [R][num_q_heads][128] of out_dtype, lse device fp32 or NULL
 * With s = scale * <q, k_new>:  lse = ln(e^{lse_prev} + e^s),
 *   out = (e^{lse_prev} out_prev + e^s v_new) / (e^{lse_prev} + e^s)      (Sec. 4.2.2 identity).
 * For fp8 handles k_new and v_new enter as the cache will hold them (quantised with
 * p->k_scale / p->v_scale, then dequantised), so the result equals one call over the
 * appended cache.  out may alias out_prev only if out_dtype is fp32.
 *
 * Both only enqueue work on p->stream.  Errors as for lamina_decode_attention.
 */
int lamina_append_kv(lamina_attn_t h, const void *k_new, const void *v_new, void *k_cache,
                     void *v_cache, const int32_t *positions, const int32_t *block_table,
                     const lamina_call_params *p);
int lamina_fold_new_token(lamina_attn_t h, const void *q, const void *k_new, const void *v_new,
                          const float *out_prev, const float *lse_prev, void *out, float *lse,
                          const lamina_call_params *p);

/*
 * lamina_fold_new_token followed by lamina_append_kv in ONE launch, for the attention device's
 * per-layer step in its overlapped order (Sec. 4.2.2): once k_n, v_n have arrived, the result
 * over the previous tokens is completed with the new token and the new rows go into the cache.
 * Arguments, results and errors are those of the two calls (p carries the cache layout and,
 * for fp8 caches, the scales); the cache rows written and the output are bit-identical to
 * calling them one after the other.  One small launch instead of two matters because the step
 * is a chain of launches behind a 60-400 us attention call.
 */
int lamina_fold_new_token_and_append(lamina_attn_t h, const void *q, const void *k_new,
                                     const void *v_new, const float *out_prev,
                                     const float *lse_prev, void *out, float *lse, void *k_cache,
                                     void *v_cache, const int32_t *positions,
                                     const int32_t *block_table, const lamina_call_params *p);

/*
 * lamina_decode_attention for callers that cannot allocate device memory or create a handle:
 * code under HIP graph capture, tight serving loops that must not reach hipMalloc, harnesses
 * that forbid it.  Same operator, same kernels, same arguments and argument checks as
 * lamina_decode_attention, with cfg in place of the handle; results are bit-identical to those
 * of a handle made from the same cfg.  The call allocates nothing, on the host or on the device
 * (no hipMalloc / hipFree, no handle): the partial results of cut rows go to a fixed area of
 * LAMINA_STATIC_SCRATCH_BYTES of device memory that is part of the library's code object -- each
 * GPU the library runs on holds its own copy from the first call on it until the process ends.
 *
 * Limit: lamina_attn_workspace_bytes(cfg) must not exceed LAMINA_STATIC_SCRATCH_BYTES, else
 * LAMINA_ERR_WORKSPACE is returned and nothing is launched (configurations that never cut rows
 * need no scratch at all; the five named workloads of this build need 4-17 MiB).
 * Every call on one GPU uses that GPU's one area: calls that overlap on a GPU (two streams, two
 * threads) race on it and must be serialised by the caller; calls on one stream are ordered by
 * the stream.  Nothing in the area has to start at zero -- each call writes every partial
 * result and prefix sum before its merge pass reads it -- so a call is not disturbed by what the
 * previous one left behind.
 * The first call on a device resolves the area's address and the device's compute-unit count
 * (no allocation, but not stream work either): make that call before a stream capture begins.
 * Errors as for lamina_attn_create (bad cfg) and lamina_decode_attention; the message is
 * returned by lamina_attn_last_error(NULL) on the calling thread.
 */
#define LAMINA_STATIC_SCRATCH_BYTES (32u << 20)
int lamina_decode_attention_static(const lamina_attn_config *cfg,
                                   const void *q,
                                   const void *k_cache,
                                   const void *v_cache,
                                   const int32_t *seq_lens,
                                   const int32_t *block_table,
                                   void *out,
                                   float *lse,
                                   const lamina_call_params *p);

#ifdef __cplusplus
}
#endif
#endif /* LAMINA_ATTN_H */
