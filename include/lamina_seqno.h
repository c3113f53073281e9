/*
 * lamina_seqno.h -- C ABI of the stream-ordered sequence-number wait / signal kernels.
 *
 * The attention device receives each layer's query vectors from another device and must not
 * start the attention kernels before they have arrived -- without a CPU in between.  The
 * paper's receive path (Sec. 4.1, "FHBN recv") does this with device-side polling: a `seqno`
 * variable that the sender advances after every send (batched behind the data, so the data is
 * visible once the new value is), and a small kernel, enqueued on the receiver's stream ahead
 * of the compute kernels, that polls it.  Launching is asynchronous, so neither the wait for
 * the data nor the launch of the compute kernels involves the host.
 *
 * This header is that mechanism for a HIP stream.  The writer of a seqno can be anything whose
 * stores the polling device sees: a host thread (as in the tests), another stream of the same
 * device via lamina_seqno_signal, or a peer device / NIC writing over the fabric.  A seqno is a
 * 64-bit counter that only grows; waiting for `target` means waiting until *seqno >= target.
 *
 * All functions return LAMINA_OK (0) or a negative error code of lamina_attn.h.
 */
#ifndef LAMINA_SEQNO_H
#define LAMINA_SEQNO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    LAMINA_SEQNO_REACHED   = 0,    /* *status after a wait that saw seqno >= target            */
    LAMINA_SEQNO_TIMED_OUT = 1     /* *status after a wait that gave up                        */
};

/*
 * Allocate one seqno (initial value 0) in pinned, host-coherent memory: the returned pointer
 * is valid on the host AND on every device of the process, so a host thread can advance it
 * with an ordinary release store while a kernel polls it.  *status_out (optional, may be NULL)
 * receives a second such word for use as the `status` of lamina_seqno_wait.  Free both with
 * lamina_seqno_free (NULL accepted) once no kernel that uses them can still be running.
 * Errors: INVALID_ARG (seqno_out NULL), HIP (allocation failed).
 */
int lamina_seqno_alloc(uint64_t **seqno_out, int32_t **status_out);
int lamina_seqno_free(uint64_t *seqno, int32_t *status);

/*
 * Enqueue on `stream` (hipStream_t; NULL = default stream of the current device) a one-wavefront
 * kernel that polls *seqno with system-scope acquire loads until *seqno >= target, then exits;
 * work enqueued on the stream afterwards therefore starts only once the value -- and every
 * store the writer released before it -- is visible.  The wait is BOUNDED: after timeout_us
 * microseconds (0 selects 10 s; measured on the device's constant 100 MHz clock) the kernel
 * gives up and exits all the same, so the stream never hangs on a writer that died; later work
 * on the stream still runs, and the caller finds out from *status.
 *   seqno    any address the device can read coherently: pinned host memory (lamina_seqno_alloc),
 *            fine-grained or peer-mapped device memory
 *   status   device-writable int32 or NULL: set to LAMINA_SEQNO_REACHED or LAMINA_SEQNO_TIMED_OUT
 *            by the kernel before it exits
 * Never blocks the host.  Errors: INVALID_ARG (seqno NULL), HIP (launch failed).
 */
int lamina_seqno_wait(const uint64_t *seqno, uint64_t target, uint32_t timeout_us,
                      int32_t *status, void *stream);

/*
 * Enqueue on `stream` a kernel that sets *seqno = value with a system-scope release store
 * (the caller passes growing values; a seqno has one writer at a time).  Being stream-ordered,
 * it runs after all work enqueued before it has finished, so a waiter that sees `value` also
 * sees that work's results: the sender side of the same protocol when the sender is a HIP
 * stream.
 * Errors: INVALID_ARG (seqno NULL), HIP (launch failed).
 */
int lamina_seqno_signal(uint64_t *seqno, uint64_t value, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LAMINA_SEQNO_H */
