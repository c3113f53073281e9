// Decode attention for gfx950 (MI355X): kernels and the C ABI declared in lamina_attn.h.
//
// The operator (paper Sec. 2.1, starred equation, per head; GQA per Sec. 2.2.2): for each
// request r and query head h, out = sum_j softmax_j(scale * q.K_j) V_j over the request's
// own KV cache.  It is a batched matrix-vector product whose arithmetic intensity does not
// grow with the batch (Sec. 2.2.2), so the kernel is organised around streaming K and V
// from HBM exactly once:
//
//   * one work-group (4 wavefronts) per (request, kv head, KV partition); the G query heads
//     of the group share every K/V tile that is loaded;
//   * every wavefront streams its own 32-token tiles with non-temporal 128-bit loads, one
//     tile ahead of the arithmetic, and never synchronises with its neighbours until the end;
//   * q.K^T and p.V run on the matrix cores (16x16x32 bf16 MFMA, the G heads padded to 16
//     columns) so that the vector ALU only does the softmax; K goes from HBM straight into
//     the MFMA operand layout, V is staged through LDS and read back transposed;
//   * partitions keep (A_q(I), ln S_q(I)) of Sec. 4.2.2 and a second kernel combines them
//     with the divide-and-conquer identity of that section.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <new>

#include "lamina_attn.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
// Read-only index arrays are read through the constant address space so that uniform reads
// stay on the scalar unit (and off the in-order vector-memory counter) inside the tile loop.
typedef const __attribute__((address_space(4))) int32_t *const_i32_ptr;

constexpr int kHeadDim = 128;
constexpr int kWaves = 4;              // wavefronts per work-group
constexpr int kThreads = kWaves * 64;
constexpr int kChunkAlign = 256;       // partition sizes are multiples of 4 wavefronts x 64 tokens
constexpr int kMaxGroup = 16;          // query heads per kv head the MFMA tile can hold
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct MainParams {
    const void *q;
    const unsigned char *k;
    const unsigned char *v;
    const int32_t *seq_lens;
    const int32_t *block_table;
    void *out;
    float *lse;
    float *part_out;                   // [R][Hq][P][128], normalised partial outputs
    float *part_lse;                   // [R][Hq][P], natural-log partial denominators
    const float *k_scale;
    const float *v_scale;
    long long stride_req_b, stride_head_b, stride_tok_b;     // bytes (contiguous mode)
    long long pool_stride_block_b, pool_stride_head_b;       // bytes (paged mode)
    int bt_stride;
    int Hq, Hkv, G;
    int P, chunk;
    int out_is_bf16;
    float scale_log2;                  // softmax scale times log2(e)
};

struct MergeParams {
    const float *part_out;
    const float *part_lse;
    const int32_t *seq_lens;
    void *out;
    float *lse;
    int Hq, P, chunk;
    int out_is_bf16;
};

__device__ __forceinline__ u32x4 load_stream_128(const unsigned char *p)
{
    // KV bytes are used once: keep them from displacing anything in the caches.
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ unsigned short bf16_bits(float x)
{
    return __builtin_bit_cast(unsigned short, static_cast<__bf16>(x));
}

// Four e4m3fn bytes -> four bf16 values (exact: every e4m3fn value is a bf16 value).
__device__ __forceinline__ bf16x4 fp8x4_to_bf16(unsigned word)
{
    const bf16x2 lo = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(word, 1.0f, false);   // bytes 0, 1
    const bf16x2 hi = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(word, 1.0f, true);    // bytes 2, 3
    bf16x4 r;
    r[0] = lo[0];
    r[1] = lo[1];
    r[2] = hi[0];
    r[3] = hi[1];
    return r;
}

__device__ __forceinline__ bf16x8 join_bf16x4(bf16x4 a, bf16x4 b)
{
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ void store_out(void *out, int out_is_bf16, size_t idx, float x)
{
    if (out_is_bf16)
        static_cast<unsigned short *>(out)[idx] = bf16_bits(x);
    else
        static_cast<float *>(out)[idx] = x;
}

// -------------------------------------------------------------------------------------------
// Main pass.  Grid: batch * Hkv * P work-groups of 256 threads; work-group id decodes to
// (request r, kv head g, partition p), p fastest.  Partition p owns tokens
// [p*chunk, min((p+1)*chunk, seq_lens[r])); a work-group whose range is empty exits at once.
//
// Lane roles inside a wavefront (col = lane % 16, quad = lane / 16):
//   scores   S^T[token][head] = K[token][:] . Q[head][:]  -- MFMA A = K sub-tile (row = token
//            col, the lane holds 8 consecutive dims), B = Q (column = head col); the result
//            leaves each lane with 4 tokens (quad*4 + v) of ONE head (col), so the softmax
//            statistics of a head live in the 4 lanes {col, col+16, col+32, col+48}.
//   output   O^T[dim][head] += V^T[dim][token] . P^T[token][head] -- MFMA A = V^T (row = dim
//            col, 8 token slots), B = P^T (column = head col, 8 token slots).  The score
//            layout above already IS that B layout, so probabilities never cross lanes; V^T
//            comes from a transposing LDS read.  The accumulator keeps head = col, so the
//            running rescale is lane-local.
// -------------------------------------------------------------------------------------------
template <bool FP8, bool PAGED>
__global__ __launch_bounds__(kThreads, 2) void decode_mfma_kernel(const MainParams prm)
{
    constexpr int TILE = FP8 ? 64 : 32;                   // tokens per wavefront tile (16 KiB of K+V)
    constexpr int NSUB = TILE / 16;                       // 16-token MFMA sub-tiles per tile
    constexpr int NPAIR = NSUB / 2;                       // 32-token contraction steps for p.V
    constexpr int ROWB = FP8 ? 128 : 256;                 // bytes of one K or V row
    constexpr int VSTRIDE = ROWB + (FP8 ? 16 : 32);       // LDS row pitch (bank spreading)
    constexpr int KR = 8;                                 // 128-bit K loads per lane per tile
    constexpr int VR = 8;                                 // 128-bit V loads per lane per tile
    constexpr int KPS = KR / NSUB;                        // K loads per sub-tile
    constexpr int LPR = ROWB / 16;                        // lanes that cover one V row
    constexpr int RPI = 64 / LPR;                         // V rows per load instruction
    constexpr int VBUF = TILE * VSTRIDE;                  // V staging bytes per wavefront
    constexpr bool SPLIT_P = !FP8;                        // carry p as hi + lo bf16 halves
    constexpr int MERGE_BYTES = kWaves * kMaxGroup * (kHeadDim + 2) * 4;
    constexpr int SMEM = (kWaves * VBUF > MERGE_BYTES) ? kWaves * VBUF : MERGE_BYTES;
    static_assert(VR * RPI == TILE && KR % NSUB == 0, "tile geometry");
    __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15;
    const int quad = lane >> 4;
    const int G = prm.G;

    int id = blockIdx.x;
    const int p = id % prm.P;
    id /= prm.P;
    const int g = id % prm.Hkv;
    const int r = id / prm.Hkv;
    const int len = prm.seq_lens[r];
    const int t0 = p * prm.chunk;
    const int hq0 = g * G;                                // first query head of this group

    if (t0 >= len) {
        // Empty partition.  Unsplit and an empty context: the result is defined as 0 / -inf.
        if (prm.P == 1) {
            for (int i = tid; i < G * kHeadDim; i += kThreads)
                store_out(prm.out, prm.out_is_bf16,
                          ((size_t)r * prm.Hq + hq0) * kHeadDim + i, 0.0f);
            if (prm.lse && tid < G)
                prm.lse[(size_t)r * prm.Hq + hq0 + tid] = -INFINITY;
        }
        return;
    }
    const int t1 = min(len, t0 + prm.chunk);
    const int last = t1 - 1;                              // loads never go past this token

    // ---- Q as MFMA B operand: column = head col, k-step s holds 8 dims --------------------
    bf16x8 qop[4];
    {
        const __bf16 *qrow =
            static_cast<const __bf16 *>(prm.q) + ((size_t)r * prm.Hq + hq0 + col) * kHeadDim;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            // The dims a lane holds in step s must be the dims its K register holds there.
            const int chunk8 = FP8 ? (((s >> 1) * 4 + quad) * 2 + (s & 1)) : (s * 4 + quad);
            bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
            qop[s] = z;
            if (col < G)
                qop[s] = *reinterpret_cast<const bf16x8 *>(qrow + chunk8 * 8);
        }
    }
    float c_log2 = prm.scale_log2;
    if (FP8)
        c_log2 *= prm.k_scale[(size_t)r * prm.Hkv + g];   // K scale folds into the score scale

    const unsigned char *kbase;
    const unsigned char *vbase;
    const_i32_ptr bt_row = nullptr;
    if (PAGED) {
        kbase = prm.k + (long long)g * prm.pool_stride_head_b;
        vbase = prm.v + (long long)g * prm.pool_stride_head_b;
        bt_row = (const_i32_ptr)(prm.block_table + (size_t)r * prm.bt_stride);
    } else {
        const long long off = (long long)r * prm.stride_req_b + (long long)g * prm.stride_head_b;
        kbase = prm.k + off;
        vbase = prm.v + off;
    }

    unsigned char *vbuf = smem + w * VBUF;                // this wavefront's V staging area

    // Pool blocks of the 16-token pages of the tile starting at ts (wave-uniform, scalar
    // loads).  Looked up one tile ahead of the loads that need them.
    auto fetch_pages = [&](int ts, int(&pg)[NSUB]) {
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
            pg[sub] = PAGED ? bt_row[min(ts + sub * 16, last) >> 4] : 0;
    };

    // Issue all loads of the tile starting at token ts.  Tokens beyond the partition are
    // redirected to its last valid row so that no byte outside the request is touched;
    // their scores are masked later.
    auto issue_loads = [&](int ts, const int(&pg)[NSUB], u32x4(&kr)[KR], u32x4(&vr)[VR]) {
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub) {
            const int tok = min(ts + sub * 16 + col, last);
            const unsigned char *row =
                PAGED ? kbase + (long long)pg[sub] * prm.pool_stride_block_b + (tok & 15) * ROWB
                      : kbase + (long long)tok * prm.stride_tok_b;
#pragma unroll
            for (int s = 0; s < KPS; ++s)
                kr[sub * KPS + s] = load_stream_128(row + (s * 4 + quad) * 16);
        }
#pragma unroll
        for (int i = 0; i < VR; ++i) {
            const int tok = min(ts + i * RPI + lane / LPR, last);
            const int sub = (i * RPI) / 16;               // compile-time per instruction
            const unsigned char *row =
                PAGED ? vbase + (long long)pg[sub] * prm.pool_stride_block_b + (tok & 15) * ROWB
                      : vbase + (long long)tok * prm.stride_tok_b;
            vr[i] = load_stream_128(row + (lane % LPR) * 16);
        }
    };

    float m_run = -INFINITY;        // running max of log2-domain scores, head = col
    float l_run = 0.0f;             // this lane's share of the running denominator
    f32x4 o_acc[8];                 // O^T[dim = db*16 + quad*4 + v][head = col]
#pragma unroll
    for (int db = 0; db < 8; ++db) {
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
        o_acc[db] = z;
    }

    // First half of a tile: everything that reads the tile's load registers.
    auto consume = [&](const u32x4(&kr)[KR], const u32x4(&vr)[VR], f32x4(&sc)[NSUB]) {
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            if (FP8) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const u32x4 raw = kr[sub * 2 + s2];
                    const bf16x8 lo = join_bf16x4(fp8x4_to_bf16(raw[0]), fp8x4_to_bf16(raw[1]));
                    const bf16x8 hi = join_bf16x4(fp8x4_to_bf16(raw[2]), fp8x4_to_bf16(raw[3]));
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo, qop[2 * s2], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi, qop[2 * s2 + 1], acc, 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const bf16x8 kop = __builtin_bit_cast(bf16x8, kr[sub * 4 + s]);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop, qop[s], acc, 0, 0, 0);
                }
            }
            sc[sub] = acc;
        }
        // stage V in LDS (row-major, padded pitch)
#pragma unroll
        for (int i = 0; i < VR; ++i) {
            const int trow = i * RPI + lane / LPR;
            *reinterpret_cast<u32x4 *>(vbuf + trow * VSTRIDE + (lane % LPR) * 16) = vr[i];
        }
    };

    // Second half: online softmax in the log2 domain, then O^T += V^T . P^T from LDS.
    auto finish = [&](int ts, const f32x4(&sc)[NSUB]) {
        float x[NSUB * 4];
        float tmax = -INFINITY;
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int tok = ts + sub * 16 + quad * 4 + v;
                float s = sc[sub][v] * c_log2;
                s = (tok < t1) ? s : -INFINITY;
                x[sub * 4 + v] = s;
                tmax = fmaxf(tmax, s);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax);           // finite from the first tile on
        const float alpha = fast_exp2(m_run - m_new);     // exp2(-inf) = 0 on the first tile
        m_run = m_new;
        float psum = 0.0f;
        bf16x8 p_hi[NPAIR], p_lo[NPAIR];
#pragma unroll
        for (int j = 0; j < NSUB * 4; ++j) {
            const float pj = fast_exp2(x[j] - m_new);
            psum += pj;
            // p = hi + lo with both halves bf16: keeps ~16 significant bits through the MFMA
            const __bf16 h = static_cast<__bf16>(pj);
            p_hi[j >> 3][j & 7] = h;
            if (SPLIT_P)
                p_lo[j >> 3][j & 7] = static_cast<__bf16>(pj - static_cast<float>(h));
        }
        l_run = l_run * alpha + psum;
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int db = 0; db < 8; ++db)
                o_acc[db] *= alpha;
        }
#pragma unroll
        for (int db = 0; db < 8; ++db) {
#pragma unroll
            for (int pp = 0; pp < NPAIR; ++pp) {
                bf16x8 vop;
                if (FP8) {
                    // 8 rows x 16 byte-columns per 16-lane block; lane supplies row col/2
                    const int rr = col >> 1;
                    const int trow =
                        pp * 32 + ((rr < 4) ? (quad * 4 + rr) : (16 + quad * 4 + rr - 4));
                    const unsigned char *a = vbuf + trow * VSTRIDE + db * 16 + (col & 1) * 8;
                    const i32x2 raw = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                        (i32x2 __attribute__((address_space(3))) *)(a));
                    vop = join_bf16x4(fp8x4_to_bf16((unsigned)raw[0]),
                                      fp8x4_to_bf16((unsigned)raw[1]));
                } else {
                    // 4 rows x 16 columns per 16-lane block; lane supplies row col/4, 4 columns
                    const unsigned char *a = vbuf + (pp * 32 + quad * 4 + (col >> 2)) * VSTRIDE +
                                             db * 32 + (col & 3) * 8;
                    const s16x4 ra = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3))) *)(a));
                    const s16x4 rb = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3))) *)(a + 16 * VSTRIDE));
                    vop = join_bf16x4(__builtin_bit_cast(bf16x4, ra),
                                      __builtin_bit_cast(bf16x4, rb));
                }
                o_acc[db] =
                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, p_hi[pp], o_acc[db], 0, 0, 0);
                if (SPLIT_P)
                    o_acc[db] =
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, p_lo[pp], o_acc[db], 0, 0, 0);
            }
        }
    };

    // ---- stream this wavefront's tiles --------------------------------------------------------
    // Tiles w, w+4, w+8, ... of the partition.  Two register sets (A, B) alternate; a set is
    // refilled with the tile two steps ahead as soon as its registers have been read, so one
    // to two tiles (16-32 KiB per wavefront) are always in flight.  The loop body is a single
    // basic block: a wavefront with an odd tile count runs one fully masked tile, and the
    // refills past the end are redirected to the last valid row.
    {
        constexpr int step = kWaves * TILE;
        int ts = t0 + w * TILE;
        if (ts < t1) {
            const int ntiles = (t1 - ts + step - 1) / step;
            u32x4 kA[KR], vA[VR], kB[KR], vB[VR];
            int pg[NSUB];
            f32x4 sc[NSUB];
            fetch_pages(ts, pg);
            issue_loads(ts, pg, kA, vA);
            __builtin_amdgcn_sched_barrier(0);            // A must be the older set
            fetch_pages(ts + step, pg);
            issue_loads(ts + step, pg, kB, vB);
            fetch_pages(ts + 2 * step, pg);
            __builtin_amdgcn_sched_barrier(0);
            for (int it = 0; it < ntiles; it += 2) {
                consume(kA, vA, sc);
                __builtin_amdgcn_sched_barrier(0);
                issue_loads(ts + 2 * step, pg, kA, vA);
                fetch_pages(ts + 3 * step, pg);
                __builtin_amdgcn_sched_barrier(0);
                finish(ts, sc);
                __builtin_amdgcn_sched_barrier(0);
                consume(kB, vB, sc);
                __builtin_amdgcn_sched_barrier(0);
                issue_loads(ts + 3 * step, pg, kB, vB);
                fetch_pages(ts + 4 * step, pg);
                __builtin_amdgcn_sched_barrier(0);
                finish(ts + step, sc);
                __builtin_amdgcn_sched_barrier(0);
                ts += 2 * step;
            }
        }
    }

    // ---- combine the four wavefronts (same identity as the cross-partition merge) -----------
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    __syncthreads();                                      // everyone is done with V staging
    float *mo = reinterpret_cast<float *>(smem);          // [kWaves][kMaxGroup][128]
    float *mm = mo + kWaves * kMaxGroup * kHeadDim;       // [kWaves][kMaxGroup] running max
    float *ml = mm + kWaves * kMaxGroup;                  // [kWaves][kMaxGroup] denominators
    if (col < G) {
#pragma unroll
        for (int db = 0; db < 8; ++db)
            *reinterpret_cast<f32x4 *>(mo + ((w * kMaxGroup + col) * kHeadDim) + db * 16 +
                                       quad * 4) = o_acc[db];
        if (quad == 0) {
            mm[w * kMaxGroup + col] = m_run;
            ml[w * kMaxGroup + col] = l_run;
        }
    }
    __syncthreads();
    const float vs = FP8 ? prm.v_scale[(size_t)r * prm.Hkv + g] : 1.0f;
    for (int i = tid; i < G * kHeadDim; i += kThreads) {
        const int h = i >> 7;
        const int d = i & 127;
        float M = -INFINITY;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww)
            M = fmaxf(M, mm[ww * kMaxGroup + h]);
        float L = 0.0f, o = 0.0f;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) {
            const float e = fast_exp2(mm[ww * kMaxGroup + h] - M);   // idle wavefront: 0
            L += e * ml[ww * kMaxGroup + h];
            o += e * mo[(ww * kMaxGroup + h) * kHeadDim + d];
        }
        o = o / L * vs;
        const size_t row = (size_t)r * prm.Hq + hq0 + h;
        const float lse_nat = (M + log2f(L)) * kLn2;
        if (prm.P == 1) {
            store_out(prm.out, prm.out_is_bf16, row * kHeadDim + d, o);
            if (d == 0 && prm.lse)
                prm.lse[row] = lse_nat;
        } else {
            prm.part_out[(row * prm.P + p) * kHeadDim + d] = o;
            if (d == 0)
                prm.part_lse[row * prm.P + p] = lse_nat;
        }
    }
}

// -------------------------------------------------------------------------------------------
// Cross-partition merge (Sec. 4.2.2 identity, P parts, log-sum-exp form):
//   lse = ln sum_p e^{lse_p},  out = sum_p e^{lse_p - lse} out_p.
// One work-group of 128 threads per (request, query head); thread d owns output column d.
// Only the first ceil(len / chunk) partitions were written by the main pass.
// -------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kHeadDim) void merge_partials_kernel(const MergeParams prm)
{
    const int row = blockIdx.x;                           // r * Hq + h
    const int r = row / prm.Hq;
    const int d = threadIdx.x;
    const int len = prm.seq_lens[r];
    const int np = min(prm.P, (len + prm.chunk - 1) / prm.chunk);
    const float *pl = prm.part_lse + (size_t)row * prm.P;
    const float *po = prm.part_out + (size_t)row * prm.P * kHeadDim;
    float M = -INFINITY;
    for (int p = 0; p < np; ++p)
        M = fmaxf(M, pl[p]);
    float W = 0.0f, o = 0.0f;
    for (int p = 0; p < np; ++p) {
        const float e = __expf(pl[p] - M);
        W += e;
        o += e * po[(size_t)p * kHeadDim + d];
    }
    const bool empty = (np == 0);
    store_out(prm.out, prm.out_is_bf16, (size_t)row * kHeadDim + d, empty ? 0.0f : o / W);
    if (d == 0 && prm.lse)
        prm.lse[row] = empty ? -INFINITY : M + logf(W);
}

}  // namespace

// ============================================================================================
// Host side: handle, validation, launch.
// ============================================================================================
struct lamina_attn {
    lamina_attn_config cfg;
    int group;
    int num_splits;
    int split_tokens;
    float scale;
    float *workspace;            // part_out followed by part_lse; nullptr when unsplit
    size_t workspace_bytes;
    char err[256];
};

namespace {

thread_local char g_create_err[256] = "";

int round_up(int x, int m) { return (x + m - 1) / m * m; }

struct Plan {
    int num_splits;
    int split_tokens;
};

// Partitioning.  Explicit num_splits is honoured; otherwise partitions of about 1024 tokens
// (512 when that still leaves the chip short of work-groups), unsplit when one covers it all.
Plan make_plan(const lamina_attn_config &c)
{
    Plan pl;
    int P;
    if (c.num_splits >= 1) {
        P = c.num_splits;
    } else {
        const long long pairs = (long long)c.max_batch * c.num_kv_heads;
        int target = 1024;
        if (pairs * ((c.max_seq_len + target - 1) / target) < 1024)
            target = 512;
        P = (c.max_seq_len + target - 1) / target;
        if (P < 1)
            P = 1;
    }
    int chunk = round_up((c.max_seq_len + P - 1) / P, kChunkAlign);
    if (chunk < kChunkAlign)
        chunk = kChunkAlign;
    if (c.num_splits < 1)
        P = (c.max_seq_len + chunk - 1) / chunk;          // drop partitions the rounding emptied
    if (P < 1)
        P = 1;
    pl.num_splits = P;
    pl.split_tokens = chunk;
    return pl;
}

const char *check_config(const lamina_attn_config *c, int *code)
{
    *code = LAMINA_ERR_INVALID_ARG;
    if (!c)
        return "config is NULL";
    if (c->num_q_heads <= 0 || c->num_kv_heads <= 0 || c->head_dim <= 0)
        return "head counts and head_dim must be positive";
    if (c->num_q_heads % c->num_kv_heads != 0)
        return "num_q_heads must be a multiple of num_kv_heads";
    if (c->max_batch <= 0 || c->max_seq_len <= 0)
        return "max_batch and max_seq_len must be positive";
    if (c->kv_dtype != LAMINA_BF16 && c->kv_dtype != LAMINA_FP8_E4M3)
        return "kv_dtype must be LAMINA_BF16 or LAMINA_FP8_E4M3";
    if (c->out_dtype != LAMINA_BF16 && c->out_dtype != LAMINA_F32)
        return "out_dtype must be LAMINA_BF16 or LAMINA_F32";
    if (c->num_splits < 0 || c->device < 0)
        return "num_splits and device must be non-negative";
    if (!(c->softmax_scale >= 0.0f) || std::isinf(c->softmax_scale))
        return "softmax_scale must be finite and non-negative (0 selects 1/sqrt(head_dim))";
    *code = LAMINA_ERR_UNSUPPORTED;
    if (c->head_dim != kHeadDim)
        return "only head_dim 128 is supported";
    if (c->block_size != 0 && c->block_size != 16)
        return "block_size must be 0 (contiguous) or 16 (paged)";
    const int G = c->num_q_heads / c->num_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8 && G != 16)
        return "group size num_q_heads/num_kv_heads must be 1, 2, 4, 8 or 16";
    if (c->kernel != LAMINA_KERNEL_MFMA)
        return "unknown kernel family";
    if (c->num_splits > 4096)
        return "num_splits above 4096";
    *code = LAMINA_OK;
    return nullptr;
}

size_t workspace_bytes_for(const lamina_attn_config &c, const Plan &pl)
{
    if (pl.num_splits <= 1)
        return 0;
    return (size_t)c.max_batch * c.num_q_heads * pl.num_splits * (kHeadDim + 1) * sizeof(float);
}

int fail(lamina_attn *h, int code, const char *msg)
{
    snprintf(h->err, sizeof h->err, "%s", msg);
    return code;
}

int fail_hip(lamina_attn *h, const char *what, hipError_t e)
{
    snprintf(h->err, sizeof h->err, "%s: %s", what, hipGetErrorString(e));
    return LAMINA_ERR_HIP;
}

class DeviceGuard {
  public:
    explicit DeviceGuard(int dev) : prev_(-1), ok_(true)
    {
        if (hipGetDevice(&prev_) != hipSuccess)
            prev_ = -1;
        if (prev_ != dev)
            ok_ = (hipSetDevice(dev) == hipSuccess);
        else
            prev_ = -1;
    }
    ~DeviceGuard()
    {
        if (prev_ >= 0)
            (void)hipSetDevice(prev_);
    }
    bool ok() const { return ok_; }

  private:
    int prev_;
    bool ok_;
};

}  // namespace

extern "C" {

size_t lamina_attn_workspace_bytes(const lamina_attn_config *cfg)
{
    int code;
    if (check_config(cfg, &code))
        return 0;
    return workspace_bytes_for(*cfg, make_plan(*cfg));
}

int lamina_attn_create(const lamina_attn_config *cfg, lamina_attn_t *out_handle)
{
    int code;
    if (!out_handle) {
        snprintf(g_create_err, sizeof g_create_err, "out_handle is NULL");
        return LAMINA_ERR_INVALID_ARG;
    }
    *out_handle = nullptr;
    if (const char *msg = check_config(cfg, &code)) {
        snprintf(g_create_err, sizeof g_create_err, "%s", msg);
        return code;
    }
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || cfg->device >= ndev) {
        snprintf(g_create_err, sizeof g_create_err, "device %d not available (%s)", cfg->device,
                 e == hipSuccess ? "ordinal out of range" : hipGetErrorString(e));
        return LAMINA_ERR_HIP;
    }
    lamina_attn *h = new (std::nothrow) lamina_attn();
    if (!h) {
        snprintf(g_create_err, sizeof g_create_err, "out of host memory");
        return LAMINA_ERR_WORKSPACE;
    }
    h->cfg = *cfg;
    h->group = cfg->num_q_heads / cfg->num_kv_heads;
    const Plan pl = make_plan(*cfg);
    h->num_splits = pl.num_splits;
    h->split_tokens = pl.split_tokens;
    h->scale = cfg->softmax_scale > 0.0f ? cfg->softmax_scale : 1.0f / sqrtf((float)cfg->head_dim);
    h->workspace = nullptr;
    h->workspace_bytes = workspace_bytes_for(*cfg, pl);
    h->err[0] = 0;
    if (h->workspace_bytes) {
        DeviceGuard guard(cfg->device);
        e = guard.ok() ? hipMalloc((void **)&h->workspace, h->workspace_bytes) : hipErrorInvalidDevice;
        if (e != hipSuccess) {
            snprintf(g_create_err, sizeof g_create_err, "workspace of %zu bytes: %s",
                     h->workspace_bytes, hipGetErrorString(e));
            (void)hipGetLastError();
            delete h;
            return LAMINA_ERR_WORKSPACE;
        }
    }
    *out_handle = h;
    return LAMINA_OK;
}

int lamina_attn_destroy(lamina_attn_t h)
{
    if (!h)
        return LAMINA_OK;
    int rc = LAMINA_OK;
    if (h->workspace) {
        DeviceGuard guard(h->cfg.device);
        if (hipFree(h->workspace) != hipSuccess)
            rc = LAMINA_ERR_HIP;
    }
    delete h;
    return rc;
}

const char *lamina_attn_last_error(lamina_attn_t h) { return h ? h->err : g_create_err; }

int lamina_attn_num_splits(lamina_attn_t h) { return h ? h->num_splits : 0; }

int lamina_attn_split_tokens(lamina_attn_t h) { return h ? h->split_tokens : 0; }

int lamina_decode_attention(lamina_attn_t h, const void *q, const void *k_cache,
                            const void *v_cache, const int32_t *seq_lens,
                            const int32_t *block_table, void *out, float *lse,
                            const lamina_call_params *p)
{
    if (!h)
        return LAMINA_ERR_INVALID_ARG;
    h->err[0] = 0;
    if (!p)
        return fail(h, LAMINA_ERR_INVALID_ARG, "call params are NULL");
    const lamina_attn_config &c = h->cfg;
    if (p->batch < 0 || p->batch > c.max_batch)
        return fail(h, LAMINA_ERR_INVALID_ARG, "batch is negative or exceeds max_batch");
    if (p->batch == 0)
        return LAMINA_OK;
    if (!q || !k_cache || !v_cache || !seq_lens || !out)
        return fail(h, LAMINA_ERR_INVALID_ARG, "q, k_cache, v_cache, seq_lens and out must be non-NULL");
    const bool fp8 = c.kv_dtype == LAMINA_FP8_E4M3;
    const bool paged = c.block_size != 0;
    const int esz = fp8 ? 1 : 2;
    if (paged && !block_table)
        return fail(h, LAMINA_ERR_INVALID_ARG, "paged cache needs a block_table");
    if (fp8 && (!p->k_scale || !p->v_scale))
        return fail(h, LAMINA_ERR_INVALID_ARG, "fp8 cache needs k_scale and v_scale");
    auto misaligned = [&](long long stride_elems) { return (stride_elems * esz) % 16 != 0; };
    if (((uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)out) % 16 != 0)
        return fail(h, LAMINA_ERR_INVALID_ARG, "q, k_cache, v_cache and out must be 16-byte aligned");
    if (paged) {
        if (p->pool_stride_head < (long long)c.block_size * kHeadDim || p->pool_stride_block <= 0 ||
            p->block_table_stride <= 0 || misaligned(p->pool_stride_head) ||
            misaligned(p->pool_stride_block))
            return fail(h, LAMINA_ERR_INVALID_ARG, "bad pool strides or block_table_stride");
    } else {
        if (p->kv_stride_tok < kHeadDim || p->kv_stride_req < 0 || p->kv_stride_head < 0 ||
            misaligned(p->kv_stride_tok) || misaligned(p->kv_stride_req) ||
            misaligned(p->kv_stride_head))
            return fail(h, LAMINA_ERR_INVALID_ARG, "bad contiguous-cache strides");
    }

    MainParams mp;
    memset(&mp, 0, sizeof mp);
    mp.q = q;
    mp.k = static_cast<const unsigned char *>(k_cache);
    mp.v = static_cast<const unsigned char *>(v_cache);
    mp.seq_lens = seq_lens;
    mp.block_table = block_table;
    mp.out = out;
    mp.lse = lse;
    mp.k_scale = p->k_scale;
    mp.v_scale = p->v_scale;
    mp.stride_req_b = p->kv_stride_req * esz;
    mp.stride_head_b = p->kv_stride_head * esz;
    mp.stride_tok_b = p->kv_stride_tok * esz;
    mp.pool_stride_block_b = p->pool_stride_block * esz;
    mp.pool_stride_head_b = p->pool_stride_head * esz;
    mp.bt_stride = p->block_table_stride;
    mp.Hq = c.num_q_heads;
    mp.Hkv = c.num_kv_heads;
    mp.G = h->group;
    mp.P = h->num_splits;
    mp.chunk = h->split_tokens;
    mp.out_is_bf16 = c.out_dtype == LAMINA_BF16;
    mp.scale_log2 = h->scale * kLog2e;
    if (h->num_splits > 1) {
        mp.part_out = h->workspace;
        mp.part_lse = h->workspace + (size_t)c.max_batch * c.num_q_heads * h->num_splits * kHeadDim;
    }

    DeviceGuard guard(c.device);
    if (!guard.ok())
        return fail(h, LAMINA_ERR_HIP, "cannot select the handle's device");
    hipStream_t stream = static_cast<hipStream_t>(p->stream);
    const long long wgs = (long long)p->batch * c.num_kv_heads * h->num_splits;
    if (wgs > 0x7fffffffLL)
        return fail(h, LAMINA_ERR_UNSUPPORTED, "grid too large");
    const dim3 grid((unsigned)wgs), block(kThreads);
    if (fp8 && paged)
        hipLaunchKernelGGL((decode_mfma_kernel<true, true>), grid, block, 0, stream, mp);
    else if (fp8)
        hipLaunchKernelGGL((decode_mfma_kernel<true, false>), grid, block, 0, stream, mp);
    else if (paged)
        hipLaunchKernelGGL((decode_mfma_kernel<false, true>), grid, block, 0, stream, mp);
    else
        hipLaunchKernelGGL((decode_mfma_kernel<false, false>), grid, block, 0, stream, mp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(h, "main kernel launch", e);
    if (h->num_splits > 1) {
        MergeParams gp;
        gp.part_out = mp.part_out;
        gp.part_lse = mp.part_lse;
        gp.seq_lens = seq_lens;
        gp.out = out;
        gp.lse = lse;
        gp.Hq = c.num_q_heads;
        gp.P = h->num_splits;
        gp.chunk = h->split_tokens;
        gp.out_is_bf16 = mp.out_is_bf16;
        hipLaunchKernelGGL(merge_partials_kernel, dim3((unsigned)(p->batch * c.num_q_heads)),
                           dim3(kHeadDim), 0, stream, gp);
        e = hipGetLastError();
        if (e != hipSuccess)
            return fail_hip(h, "merge kernel launch", e);
    }
    return LAMINA_OK;
}

}  // extern "C"
