// Stream-ordered sequence-number wait / signal for gfx950: the device-side polling receive of
// the paper's host-bypassed network stack (Sec. 4.1, "FHBN recv"), with the writer left open
// (host thread, another stream, a peer device).  Declared in lamina_seqno.h.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "lamina_attn.h"
#include "lamina_seqno.h"

namespace {

constexpr unsigned long long kTicksPerMicrosecond = 100;      // s_memrealtime: constant 100 MHz
constexpr uint32_t kDefaultTimeoutUs = 10u * 1000u * 1000u;

// One wavefront; lane 0 polls.  Every path leaves the loop: the value arrives or the clock
// runs out.  System scope: the load must not be served from a cache the writer cannot reach.
__global__ __launch_bounds__(64) void seqno_wait_kernel(const uint64_t *seqno, uint64_t target,
                                                       unsigned long long timeout_ticks,
                                                       int32_t *status)
{
    if (threadIdx.x != 0)
        return;
    const unsigned long long start = __builtin_amdgcn_s_memrealtime();
    int32_t result = LAMINA_SEQNO_TIMED_OUT;
    for (;;) {
        const uint64_t seen =
            __hip_atomic_load(seqno, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM);
        if (seen >= target) {
            result = LAMINA_SEQNO_REACHED;
            break;
        }
        if (__builtin_amdgcn_s_memrealtime() - start >= timeout_ticks)
            break;
        __builtin_amdgcn_s_sleep(32);                         // ~0.5 us between polls
    }
    if (status)
        __hip_atomic_store(status, result, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ __launch_bounds__(64) void seqno_signal_kernel(uint64_t *seqno, uint64_t value)
{
    if (threadIdx.x != 0)
        return;
    // a plain release store: the target may be host memory, where read-modify-write atomics
    // need PCIe support that cannot be taken for granted
    __hip_atomic_store(seqno, value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

}  // namespace

extern "C" {

int lamina_seqno_alloc(uint64_t **seqno_out, int32_t **status_out)
{
    if (!seqno_out)
        return LAMINA_ERR_INVALID_ARG;
    *seqno_out = nullptr;
    if (status_out)
        *status_out = nullptr;
    // one pinned, coherent 128-byte line: the seqno at offset 0, the status word at offset 64
    void *mem = nullptr;
    if (hipHostMalloc(&mem, 128, hipHostMallocMapped | hipHostMallocCoherent) != hipSuccess) {
        (void)hipGetLastError();
        return LAMINA_ERR_HIP;
    }
    volatile uint64_t *words = static_cast<volatile uint64_t *>(mem);
    for (int i = 0; i < 16; ++i)
        words[i] = 0;
    *seqno_out = static_cast<uint64_t *>(mem);
    if (status_out)
        *status_out = reinterpret_cast<int32_t *>(static_cast<char *>(mem) + 64);
    return LAMINA_OK;
}

int lamina_seqno_free(uint64_t *seqno, int32_t *status)
{
    (void)status;                                             // lives in the seqno's allocation
    if (!seqno)
        return LAMINA_OK;
    return hipHostFree(seqno) == hipSuccess ? LAMINA_OK : LAMINA_ERR_HIP;
}

int lamina_seqno_wait(const uint64_t *seqno, uint64_t target, uint32_t timeout_us,
                      int32_t *status, void *stream)
{
    if (!seqno)
        return LAMINA_ERR_INVALID_ARG;
    const unsigned long long ticks =
        (unsigned long long)(timeout_us ? timeout_us : kDefaultTimeoutUs) * kTicksPerMicrosecond;
    hipLaunchKernelGGL(seqno_wait_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                       seqno, target, ticks, status);
    return hipGetLastError() == hipSuccess ? LAMINA_OK : LAMINA_ERR_HIP;
}

int lamina_seqno_signal(uint64_t *seqno, uint64_t value, void *stream)
{
    if (!seqno)
        return LAMINA_ERR_INVALID_ARG;
    hipLaunchKernelGGL(seqno_signal_kernel, dim3(1), dim3(64), 0,
                       static_cast<hipStream_t>(stream), seqno, value);
    return hipGetLastError() == hipSuccess ? LAMINA_OK : LAMINA_ERR_HIP;
}

}  // extern "C"
