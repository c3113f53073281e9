// Measurement aids declared in lamina_probe.h, neither of them on the product path:
//   * a read-only streaming kernel with the launch geometry of the decode attention main pass,
//     the same-box reference for the HBM roofline the operator is priced against (paper
//     Sec. 2.2.2: the operator is bound by memory bandwidth);
//   * the same operator (Sec. 2.1 starred equation, GQA per Sec. 2.2.2) with every product on
//     the vector ALU instead of the matrix cores, streaming K and V exactly as the main pass
//     does, so that what the matrix cores buy can be measured rather than argued.
#include <hip/hip_runtime.h>

#include <cmath>
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


// -------------------------------------------------------------------------------------------
// Decode attention on the vector ALU (bf16 contiguous caches, rows never cut, fp32 output).
//
// Streaming is the main pass's: a persistent grid of 4-wavefront work-groups, a work-group per
// (request, kv head) row, wavefront w taking the 32-token tiles w, w+4, ..., every tile 8 + 8
// non-temporal 128-bit loads per lane that cover whole rows, two tiles in flight, refills
// beyond the row's end redirected to its last token.  Only the arithmetic differs:
//   * a load leaves the lane with 8 consecutive dims (piece = lane % 16) of token
//     i*4 + lane/16 of the tile; q.k is four bf16 dot-product instructions per head and load
//     followed by a sum over the 16 lanes of the row (four DPP additions);
//   * the softmax runs per lane for its row group's 8 tokens of the tile (the maximum is taken
//     over the whole tile, so all lanes rescale alike);
//   * p.V is 8 fp32 multiply-adds per head and load into the lane's 8 output dims; the four
//     row groups' partial sums meet once, at the end of the row.
// The four wavefronts' (max, denominator, output) triples are combined through LDS.
// -------------------------------------------------------------------------------------------
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct ValuParams {
    const unsigned char *q;            // bf16 [R][Hq][128]
    const unsigned char *k;            // bf16, strides below
    const unsigned char *v;
    const int32_t *seq_lens;
    float *out;                        // fp32 [R][Hq][128]
    float *lse;                        // fp32 [R][Hq], natural log
    long long stride_req_b, stride_head_b, stride_tok_b;
    int R, Hq, Hkv;
    int len_cap;
    float scale_log2;
};

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}

// Sum over the 16 lanes of a row; every lane of the row ends up with the total.
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_move<0xB1>(x);                               // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);                               // quad_perm [2,3,0,1]
    x += dpp_move<0x141>(x);                              // row_half_mirror
    x += dpp_move<0x140>(x);                              // row_mirror
    return x;
}

template <int G>
__global__ __launch_bounds__(kWaves * 64, G == 8 ? 1 : 2) void valu_attention_kernel(const ValuParams prm)
{
    constexpr int TILE = 32;
    constexpr int NL = 8;                                 // K (and V) loads per lane and tile
    __shared__ float s_o[kWaves][G][128];
    __shared__ float s_m[kWaves][G];
    __shared__ float s_l[kWaves][G];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int piece = lane & 15;                          // dims piece*8 .. piece*8+7
    const int rg = lane >> 4;                             // row group: token i*4 + rg of a tile
    const int rows = prm.R * prm.Hkv;
    for (int row = blockIdx.x; row < rows; row += gridDim.x) {
        const int r = row / prm.Hkv, g = row % prm.Hkv;
        const int len = min(max(prm.seq_lens[r], 0), prm.len_cap);
        const unsigned char *kb = prm.k + (long long)r * prm.stride_req_b + (long long)g * prm.stride_head_b;
        const unsigned char *vb = prm.v + (long long)r * prm.stride_req_b + (long long)g * prm.stride_head_b;
        u32x4 qv[G];
#pragma unroll
        for (int h = 0; h < G; ++h)
            qv[h] = *reinterpret_cast<const u32x4 *>(
                prm.q + ((size_t)r * prm.Hq + (size_t)g * G + h) * 256 + piece * 16);
        float m[G], l[G], o[G][8];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            m[h] = -INFINITY;
            l[h] = 0.0f;
#pragma unroll
            for (int d = 0; d < 8; ++d)
                o[h][d] = 0.0f;
        }
        const int ntiles = (len + TILE - 1) / TILE;
        const int mine = ntiles > w ? (ntiles - w + kWaves - 1) / kWaves : 0;   // this wavefront's tiles
        const int n_even = (mine + 1) & ~1;
        const int last = len - 1;                         // >= 0 whenever a load is issued
        u32x4 kA[NL], vA[NL], kB[NL], vB[NL];
        auto issue = [&](int k_th, u32x4(&kr)[NL], u32x4(&vr)[NL]) {
            const int ts = (w + k_th * kWaves) * TILE;
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int tok = min(ts + i * 4 + rg, last);
                kr[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(
                    kb + (long long)tok * prm.stride_tok_b + piece * 16));
            }
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int tok = min(ts + i * 4 + rg, last);
                vr[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(
                    vb + (long long)tok * prm.stride_tok_b + piece * 16));
            }
        };
        auto compute = [&](int k_th, const u32x4(&kr)[NL], const u32x4(&vr)[NL]) {
            const int ts = (w + k_th * kWaves) * TILE;
            float s[G][NL];
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const bool valid = ts + i * 4 + rg < len;
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    float acc = 0.0f;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        // (elements are copied to scalars first: a bit cast applied directly
                        // to a vector element reads element 0 with this compiler)
                        const unsigned kk = kr[i][c], qq = qv[h][c];
                        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kk),
                                                              __builtin_bit_cast(bf16x2, qq), acc,
                                                              false);
                    }
                    acc = row16_sum(acc);
                    s[h][i] = valid ? acc * prm.scale_log2 : -INFINITY;
                }
            }
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float tmax = s[h][0];
#pragma unroll
                for (int i = 1; i < NL; ++i)
                    tmax = fmaxf(tmax, s[h][i]);
                tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
                tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
                const float m_new = fmaxf(m[h], tmax);    // finite: a wavefront's first tile holds a token
                const float alpha = exp2f(m[h] - m_new);
                m[h] = m_new;
                float ps = 0.0f;
#pragma unroll
                for (int i = 0; i < NL; ++i) {
                    s[h][i] = exp2f(s[h][i] - m_new);     // the probability, in place
                    ps += s[h][i];
                }
                l[h] = l[h] * alpha + ps;
#pragma unroll
                for (int d = 0; d < 8; ++d)
                    o[h][d] *= alpha;
            }
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                float vf[8];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    vf[2 * c] = __builtin_bit_cast(float, vr[i][c] << 16);
                    vf[2 * c + 1] = __builtin_bit_cast(float, vr[i][c] & 0xffff0000u);
                }
#pragma unroll
                for (int h = 0; h < G; ++h)
#pragma unroll
                    for (int d = 0; d < 8; ++d)
                        o[h][d] = fmaf(s[h][i], vf[d], o[h][d]);
            }
        };
        if (n_even > 0) {
            issue(0, kA, vA);
            __builtin_amdgcn_sched_barrier(0);
            issue(1, kB, vB);
            __builtin_amdgcn_sched_barrier(0);
        }
        for (int k_th = 0; k_th < n_even; k_th += 2) {
            compute(k_th, kA, vA);
            __builtin_amdgcn_sched_barrier(0);
            issue(k_th + 2, kA, vA);
            __builtin_amdgcn_sched_barrier(0);
            compute(k_th + 1, kB, vB);
            __builtin_amdgcn_sched_barrier(0);
            issue(k_th + 3, kB, vB);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the four row groups hold partial sums over different tokens
#pragma unroll
        for (int h = 0; h < G; ++h) {
            l[h] += __shfl_xor(l[h], 16);
            l[h] += __shfl_xor(l[h], 32);
#pragma unroll
            for (int d = 0; d < 8; ++d) {
                o[h][d] += __shfl_xor(o[h][d], 16);
                o[h][d] += __shfl_xor(o[h][d], 32);
            }
        }
        if (rg == 0) {
#pragma unroll
            for (int h = 0; h < G; ++h) {
#pragma unroll
                for (int d = 0; d < 8; ++d)
                    s_o[w][h][piece * 8 + d] = o[h][d];
                if (piece == 0) {
                    s_m[w][h] = m[h];
                    s_l[w][h] = l[h];
                }
            }
        }
        __syncthreads();
        for (int idx = tid; idx < G * 128; idx += kWaves * 64) {
            const int h = idx >> 7, d = idx & 127;
            float M = -INFINITY;
#pragma unroll
            for (int ww = 0; ww < kWaves; ++ww)
                M = fmaxf(M, s_m[ww][h]);
            float W = 0.0f, O = 0.0f;
            if (M > -INFINITY) {
#pragma unroll
                for (int ww = 0; ww < kWaves; ++ww) {
                    const float e = exp2f(s_m[ww][h] - M);   // 0 for a wavefront without tiles
                    W += s_l[ww][h] * e;
                    O += s_o[ww][h][d] * e;
                }
            }
            const size_t at = (size_t)r * prm.Hq + (size_t)g * G + h;
            prm.out[at * 128 + d] = W > 0.0f ? O / W : 0.0f;
            if (d == 0 && prm.lse)
                prm.lse[at] = W > 0.0f ? (M + log2f(W)) * 0.6931471805599453f : -INFINITY;
        }
        __syncthreads();
    }
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


extern "C" int lamina_probe_valu_attention(const void *q, const void *k_cache, const void *v_cache,
                                           const int32_t *seq_lens, float *out, float *lse,
                                           int batch, int num_q_heads, int num_kv_heads,
                                           int max_seq_len, int64_t kv_stride_req,
                                           int64_t kv_stride_head, int64_t kv_stride_tok,
                                           float softmax_scale, int work_groups, void *stream)
{
    if (!q || !k_cache || !v_cache || !seq_lens || !out || batch < 0 || num_kv_heads <= 0 ||
        num_q_heads <= 0 || num_q_heads % num_kv_heads != 0 || max_seq_len <= 0 ||
        work_groups < 0 || kv_stride_tok < 128 || kv_stride_tok % 8 != 0 || kv_stride_head < 0 ||
        kv_stride_head % 8 != 0 || kv_stride_req < 0 || kv_stride_req % 8 != 0 ||
        (uintptr_t)q % 16 != 0 || (uintptr_t)k_cache % 16 != 0 || (uintptr_t)v_cache % 16 != 0 ||
        (uintptr_t)out % 4 != 0 || (long long)batch * num_kv_heads > (1ll << 30))
        return LAMINA_ERR_INVALID_ARG;
    const int G = num_q_heads / num_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8)
        return LAMINA_ERR_UNSUPPORTED;
    if (batch == 0)
        return LAMINA_OK;
    int wgs = work_groups;
    if (wgs == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus <= 0)
            return LAMINA_ERR_HIP;
        wgs = (G == 8 ? 1 : 2) * cus;                     // what can be resident at once
    }
    const long long rows = (long long)batch * num_kv_heads;
    if (wgs > rows)
        wgs = (int)rows;
    ValuParams prm;
    prm.q = static_cast<const unsigned char *>(q);
    prm.k = static_cast<const unsigned char *>(k_cache);
    prm.v = static_cast<const unsigned char *>(v_cache);
    prm.seq_lens = seq_lens;
    prm.out = out;
    prm.lse = lse;
    prm.stride_req_b = kv_stride_req * 2;
    prm.stride_head_b = kv_stride_head * 2;
    prm.stride_tok_b = kv_stride_tok * 2;
    prm.R = batch;
    prm.Hq = num_q_heads;
    prm.Hkv = num_kv_heads;
    prm.len_cap = max_seq_len;
    prm.scale_log2 = (softmax_scale > 0.0f ? softmax_scale : 1.0f / sqrtf(128.0f)) * 1.4426950408889634f;
    const dim3 grid((unsigned)wgs), block(kWaves * 64);
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (G) {
    case 1: hipLaunchKernelGGL(valu_attention_kernel<1>, grid, block, 0, st, prm); break;
    case 2: hipLaunchKernelGGL(valu_attention_kernel<2>, grid, block, 0, st, prm); break;
    case 4: hipLaunchKernelGGL(valu_attention_kernel<4>, grid, block, 0, st, prm); break;
    default: hipLaunchKernelGGL(valu_attention_kernel<8>, grid, block, 0, st, prm); break;
    }
    return hipGetLastError() == hipSuccess ? LAMINA_OK : LAMINA_ERR_HIP;
}
