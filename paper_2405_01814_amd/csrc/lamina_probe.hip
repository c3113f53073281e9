// Read-only streaming kernel with the launch geometry of the decode attention main pass
// (declared in lamina_probe.h): the same-box reference for the HBM roofline the operator is
// priced against (paper Sec. 2.2.2: the operator is bound by memory bandwidth).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "lamina_attn.h"
#include "lamina_probe.h"

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;                  // wavefronts per work-group, as in the main pass
constexpr int kLoads = 16;                 // 128-bit loads per lane and tile: 16 KiB per wavefront
constexpr size_t kTileVecs = (size_t)kLoads * 64;   // 16-byte vectors per tile

template <bool NT>
__device__ __forceinline__ u32x4 load_vec(const u32x4 *p)
{
    return NT ? __builtin_nontemporal_load(p) : *p;
}

// Work-group j reads a contiguous share of the buffer (shares equal to within one tile); its
// wavefronts take tiles w, w+4, ... of the share.  Each wavefront keeps two register sets of
// one tile in flight and refills a set as soon as it has been read, like the main pass.
// Vectors beyond the end of the share are redirected to its last vector and not counted.
template <bool NT>
__global__ __launch_bounds__(kWaves * 64, 2) void stream_read_kernel(const u32x4 *buf, size_t nvec,
                                                                    unsigned *sink)
{
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const size_t ntiles = (nvec + kTileVecs - 1) / kTileVecs;
    const size_t q = ntiles / gridDim.x, rem = ntiles % gridDim.x;
    const size_t j = blockIdx.x;
    const size_t t0 = j * q + (j < rem ? j : rem);
    const size_t t1 = t0 + q + (j < rem ? 1 : 0);
    if (t0 + w >= t1)
        return;
    const size_t last = nvec - 1;
    unsigned acc = 0;
    u32x4 a[kLoads], b[kLoads];
    auto issue = [&](size_t tile, u32x4(&r)[kLoads]) {
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            size_t at = tile * kTileVecs + (size_t)i * 64 + lane;
            at = at < last ? at : last;
            r[i] = load_vec<NT>(buf + at);
        }
    };
    auto fold = [&](size_t tile, const u32x4(&r)[kLoads]) {
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            const size_t at = tile * kTileVecs + (size_t)i * 64 + lane;
            const unsigned x = r[i][0] ^ r[i][1] ^ r[i][2] ^ r[i][3];
            acc ^= (tile < t1 && at <= last) ? x : 0u;
        }
    };
    size_t t = t0 + w;
    issue(t, a);
    __builtin_amdgcn_sched_barrier(0);
    issue(t + kWaves, b);
    __builtin_amdgcn_sched_barrier(0);
    for (; t < t1; t += 2 * kWaves) {
        fold(t, a);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 2 * kWaves < t1)
            issue(t + 2 * kWaves, a);
        __builtin_amdgcn_sched_barrier(0);
        fold(t + kWaves, b);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 3 * kWaves < t1)
            issue(t + 3 * kWaves, b);
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        acc ^= __shfl_xor(acc, off);
    if (lane == 0 && acc == 0x9e3779b9u)                  // practically never: keeps the loads alive
        *sink = acc;
    if (lane == 0 && j == 0 && w == 0)
        *sink = acc | 1u;
}

}  // namespace

extern "C" int lamina_probe_stream_read(const void *buf, size_t bytes, int nontemporal,
                                        int work_groups, uint32_t *sink, void *stream)
{
    if (!buf || !sink || bytes == 0 || bytes % 16 != 0 || (uintptr_t)buf % 16 != 0 ||
        (uintptr_t)sink % 4 != 0 || work_groups < 0)
        return LAMINA_ERR_INVALID_ARG;
    int wgs = work_groups;
    if (wgs == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus <= 0)
            return LAMINA_ERR_HIP;
        wgs = 2 * cus;
    }
    const size_t nvec = bytes / 16;
    const u32x4 *p = static_cast<const u32x4 *>(buf);
    if (nontemporal)
        hipLaunchKernelGGL(stream_read_kernel<true>, dim3((unsigned)wgs), dim3(kWaves * 64), 0,
                           static_cast<hipStream_t>(stream), p, nvec, sink);
    else
        hipLaunchKernelGGL(stream_read_kernel<false>, dim3((unsigned)wgs), dim3(kWaves * 64), 0,
                           static_cast<hipStream_t>(stream), p, nvec, sink);
    return hipGetLastError() == hipSuccess ? LAMINA_OK : LAMINA_ERR_HIP;
}
