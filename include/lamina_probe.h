/*
 * lamina_probe.h -- measurement aids beside the decode attention operator (not on its path):
 * a read-only streaming kernel with the launch geometry of the main pass, as a same-box
 * reference for what the memory system delivers, and the operator once more with all of its
 * arithmetic on the vector ALU, as the reference for what the matrix cores buy.
 *
 * The decode attention operator is bound by HBM bandwidth (paper Sec. 2.2.2: its arithmetic
 * intensity does not grow with the batch), so the benchmark prices it against the chip's
 * published peak.  This call measures the other end of the comparison: a kernel that does
 * nothing but read a buffer once -- a persistent grid of two 4-wavefront work-groups per
 * compute unit, every wavefront streaming 16 KiB tiles with 128-bit loads of whole lines,
 * two tiles in flight -- so that a reader can tell how much of the gap to the peak is the
 * operator's and how much no read-only kernel of this shape closes on this machine.
 *
 * Returns LAMINA_OK (0) or a negative error code of lamina_attn.h.
 */
#ifndef LAMINA_PROBE_H
#define LAMINA_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Enqueue on `stream` (hipStream_t; NULL = default stream) one pass that reads
 * buf[0 .. bytes) exactly once.
 *   buf          device memory, 16-byte aligned; bytes a positive multiple of 16
 *   nontemporal  non-zero: loads carry the non-temporal hint (as the operator's K/V loads do);
 *                zero: ordinary loads
 *   work_groups  size of the persistent grid; 0 selects two per compute unit of the current
 *                device (what the operator uses)
 *   sink         device-writable uint32 (4-byte aligned) that receives a value derived from every
 *                byte read, so that no load can be dropped; caller-owned, must not be NULL
 * Nothing is allocated and nothing synchronises.  Errors: INVALID_ARG (NULL or misaligned
 * pointer, bytes not a positive multiple of 16, negative work_groups), HIP (launch failed).
 */
int lamina_probe_stream_read(const void *buf, size_t bytes, int nontemporal, int work_groups,
                             uint32_t *sink, void *stream);

/*
 * The decode attention operator of paper Sec. 2.1 (starred equation, per head; grouped-query
 * sharing of K and V as in Sec. 2.2.2) computed WITHOUT the matrix cores: bf16 dot-product and
 * fp32 multiply-add instructions of the vector ALU only, while K and V are streamed exactly as
 * lamina_decode_attention streams them (persistent grid, 16 KiB tiles of whole rows,
 * non-temporal 128-bit loads, two tiles in flight per wavefront).  It exists so that the choice
 * of the matrix cores for a memory-bound operator can be measured on the same inputs; it is not
 * used by any other entry point.  Restricted to what that comparison needs: bf16 contiguous
 * caches, rows never cut, fp32 output, group sizes 1, 2, 4, 8.
 *   q            device bf16 [batch][num_q_heads][128], 16-byte aligned
 *   k_cache,     device bf16; element (r, g, t, c) at r*kv_stride_req + g*kv_stride_head +
 *   v_cache        t*kv_stride_tok + c (strides in elements, multiples of 8, kv_stride_tok >= 128);
 *                every request's rows must exist up to max_seq_len tokens
 *   seq_lens     device int32 [batch]; values are clamped to [0, max_seq_len] in the kernel
 *   out          device fp32 [batch][num_q_heads][128];  0 for an empty request
 *   lse          device fp32 [batch][num_q_heads], natural log of the softmax denominator of
 *                the scaled scores (-inf for an empty request); may be NULL
 *   softmax_scale  0 selects 1/sqrt(128)
 *   work_groups  size of the persistent grid; 0 selects what can be resident (two per compute
 *                unit, one for group size 8), never more than batch * num_kv_heads
 * Enqueues one kernel on `stream`; nothing is allocated, nothing synchronises.  Errors:
 * INVALID_ARG (NULL or misaligned pointer, bad head counts, strides or sizes), UNSUPPORTED
 * (group size not 1, 2, 4 or 8), HIP (launch failed).
 */
int lamina_probe_valu_attention(const void *q, const void *k_cache, const void *v_cache,
                                const int32_t *seq_lens, float *out, float *lse, int batch,
                                int num_q_heads, int num_kv_heads, int max_seq_len,
                                int64_t kv_stride_req, int64_t kv_stride_head,
                                int64_t kv_stride_tok, float softmax_scale, int work_groups,
                                void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LAMINA_PROBE_H */
