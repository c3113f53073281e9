/*
 * lamina_probe.h -- a read-only streaming kernel with the launch geometry of the decode
 * attention main pass, as a same-box reference for what the memory system delivers.
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

#ifdef __cplusplus
}
#endif
#endif /* LAMINA_PROBE_H */
