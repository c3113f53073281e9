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
constexpr int kMaxSplitBatch = 1024;   // requests per call when the KV range is partitioned
constexpr int kTableSlots = 256;       // work items one work-group can be dealt per call
constexpr int kCoarsenSteps = 4;       // the kernel may double the base partition size this often
constexpr int kItemsPerGroup = 4;      // ... while an item stays below 1/4 of a work-group's share
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
    int P, chunk;                      // partitions per request at most, base partition size
    int adapt;                         // 1: the kernel may coarsen the partition size
    int *chunk_used;                   // device scalar: partition size the kernel settled on
    int batch;
    int out_is_bf16;
    float scale_log2;                  // softmax scale times log2(e)
};

struct MergeParams {
    const float *part_out;
    const float *part_lse;
    const int32_t *seq_lens;
    void *out;
    float *lse;
    int Hq, P;
    const int *chunk_used;             // partition size the main pass settled on
    int rows;
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

// Work-group barrier that orders LDS traffic only.  Unlike __syncthreads() it does not wait
// for outstanding global loads or stores, so prefetched K/V tiles stay in flight across it.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Wait until every vector-memory operation this wavefront has issued is complete.
__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }

__device__ __forceinline__ void store_out(void *out, int out_is_bf16, size_t idx, float x)
{
    if (out_is_bf16)
        static_cast<unsigned short *>(out)[idx] = bf16_bits(x);
    else
        static_cast<float *>(out)[idx] = x;
}

// -------------------------------------------------------------------------------------------
// Main pass: a persistent kernel.  The grid is a fixed number of work-groups (two per compute
// unit) that stay resident and share out a compact list of work items.
//
// Work items.  Request r is cut into n(r) = max(1, ceil(seq_lens[r] / chunk)) partitions of
// `chunk` tokens (one partition when the handle is unsplit); an item is (partition, kv head).
// Items are numbered with the kv head fastest and requests in order, skipping nothing but
// the partitions a request is too short to have; work-group j takes items j, j + grid,
// j + 2 grid, ...  Every work-group derives the numbering itself from seq_lens (a prefix sum
// and a table of its own items in LDS), so the host never reads seq_lens and no planning
// kernel runs.  Equal-sized items dealt round-robin keep skewed batches balanced.
//
// Inside an item the four wavefronts take 32-token (bf16) or 64-token (fp8) tiles
// w, w+4, w+8, ... and never synchronise until the item ends, where they combine their
// (max, denominator, output) triples through LDS -- the same identity as the cross-partition
// merge.  A request with a single partition is written straight to out/lse; otherwise the
// item writes the partial pair (A_q(I), ln S_q(I)) of Sec. 4.2.2 to the workspace.
//
// Streaming.  Each wavefront keeps two register sets of 16 KiB of K+V in flight and refills a
// set as soon as its registers have been read.  When an item runs out of tiles the refills
// continue with the first two tiles of the wavefront's NEXT item, so the memory pipeline
// never drains at an item boundary; the steady-state loop body is one basic block (which set
// of addresses a refill uses is a scalar select, not a branch).
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
template <bool FP8, bool PAGED, int GQ>
__global__ __launch_bounds__(kThreads, 2) void decode_mfma_kernel(const MainParams prm)
{
    constexpr int TILE = FP8 ? 64 : 32;                   // tokens per wavefront tile (16 KiB of K+V)
    constexpr int NSUB = TILE / 16;                       // 16-token MFMA sub-tiles per tile
    constexpr int NPAIR = NSUB / 2;                       // 32-token contraction steps for p.V
    constexpr int ROWB = FP8 ? 128 : 256;                 // bytes of one K or V row
    constexpr int VSTRIDE = ROWB + (FP8 ? 16 : 32);       // LDS row pitch of staged V (bank spreading)
    constexpr int KSTRIDE = ROWB + 16;                    // LDS row pitch of staged K
    constexpr int KR = 8;                                 // 128-bit K loads per lane per tile
    constexpr int VR = 8;                                 // 128-bit V loads per lane per tile
    constexpr int LPR = ROWB / 16;                        // lanes that cover one V row
    constexpr int RPI = 64 / LPR;                         // V rows per load instruction
    constexpr int VBUF = TILE * VSTRIDE;                  // V staging bytes per wavefront
    constexpr bool SPLIT_P = !FP8;                        // carry p as hi + lo bf16 halves
    // Keep the next item's Q rows in registers for a whole item?  Only where the register
    // file has room (not with the fp8 tile, not with 16 head rows); otherwise the rows are
    // fetched when the item starts, which costs that wavefront one exposed cache latency.
    constexpr bool Q_AHEAD = !FP8 && GQ <= 2;
    constexpr int step = kWaves * TILE;                   // token stride between a wave's tiles
    constexpr int TRIP = kMaxGroup * kHeadDim + 2 * kMaxGroup;   // floats: O, then max, then sum
    static_assert(VR * RPI == TILE && KR == VR && KSTRIDE <= VSTRIDE, "tile geometry");
    __shared__ __attribute__((aligned(16))) unsigned char smem[kWaves * VBUF];
    __shared__ __attribute__((aligned(16))) float s_trip[kWaves * TRIP];   // end-of-item triples
    __shared__ int s_busy[kWaves];                        // 1 while s_trip[w] awaits the combine
    __shared__ int s_count;                               // wavefronts that finished the item
    __shared__ int s_cum[kMaxSplitBatch + 1];             // partitions before request r
    __shared__ int s_tab_r[kTableSlots];                  // this work-group's items: request
    __shared__ int s_tab_c[kTableSlots];                  //                          partition
    __shared__ int s_tab_len[kTableSlots];                //                          seq_lens[request]
    __shared__ float s_wgt[kWaves * kMaxGroup];           // combine weights of the four triples
    __shared__ int s_wsum[kWaves];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15;
    const int quad = lane >> 4;
    const int G = prm.G;
    const int R = prm.batch;
    int C = prm.chunk;
    const int Hkv = prm.Hkv;
    const bool split = prm.P > 1;
    const int j = blockIdx.x;
    const int nwg = gridDim.x;
    const const_i32_ptr lens = (const_i32_ptr)prm.seq_lens;

    auto nparts = [&](int len) { return min(prm.P, max(1, (len + C - 1) / C)); };
    unsigned char *vbuf = smem + w * VBUF;                // this wavefront's V staging area

    if (tid < kWaves)
        s_busy[tid] = 0;
    if (tid == 0)
        s_count = 0;
    __syncthreads();

    // ---- the work list ---------------------------------------------------------------------
    int total_items;
    if (split) {
        const int per = (R + kThreads - 1) / kThreads;
        const int b = tid * per;
        const int e = min(R, b + per);
        if (prm.adapt) {
            // Partition size for THIS batch: the base size doubled as often as keeps an item
            // below a quarter of a work-group's average share of the batch's tokens.  Few,
            // long items waste nothing at item boundaries; many, short ones are what balances
            // skewed or small batches.  Every work-group takes the same decision from the
            // same seq_lens.
            int toks = 0;
            for (int i = b; i < e; ++i)
                toks += prm.seq_lens[i];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1)
                toks += __shfl_xor(toks, off);
            if (lane == 0)
                s_wsum[w] = toks;
            __syncthreads();
            long long total = 0;
#pragma unroll
            for (int ww = 0; ww < kWaves; ++ww)
                total += s_wsum[ww];
            __syncthreads();                              // s_wsum is reused by the scan below
            const long long share = total * Hkv / nwg;    // tokens per work-group
            int pick = 0;
#pragma unroll
            for (int k = 1; k <= kCoarsenSteps; ++k)
                if ((long long)(C << k) * kItemsPerGroup <= share)
                    pick = k;
            C <<= __builtin_amdgcn_readfirstlane(pick);
        }
        if (j == 0 && tid == 0)
            *prm.chunk_used = C;
        int sum = 0;
        for (int i = b; i < e; ++i)
            sum += nparts(prm.seq_lens[i]);
        int inc = sum;                                    // inclusive scan inside the wavefront
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int t = __shfl_up(inc, off);
            if (lane >= off)
                inc += t;
        }
        if (lane == 63)
            s_wsum[w] = inc;
        __syncthreads();
        int wbase = 0, tot = 0;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) {
            const int v = s_wsum[ww];
            wbase += (ww < w) ? v : 0;
            tot += v;
        }
        int run = wbase + inc - sum;
        for (int i = b; i < e; ++i) {
            s_cum[i] = run;
            run += nparts(prm.seq_lens[i]);
        }
        if (tid == 0)
            s_cum[R] = tot;
        __syncthreads();
        total_items = __builtin_amdgcn_readfirstlane(tot) * Hkv;
    } else {
        total_items = R * Hkv;
    }
    const int nslots = (j < total_items) ? (total_items - j + nwg - 1) / nwg : 0;
    if (nslots == 0)
        return;
    if (split) {
        for (int sl = tid; sl < nslots; sl += kThreads) {  // nslots <= kTableSlots (host check)
            const int cidx = (j + sl * nwg) / Hkv;
            int lo = 0, hi = R;                           // largest r with cum[r] <= cidx
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_cum[mid] <= cidx)
                    lo = mid;
                else
                    hi = mid;
            }
            s_tab_r[sl] = lo;
            s_tab_c[sl] = cidx - s_cum[lo];
            s_tab_len[sl] = prm.seq_lens[lo];
        }
        __syncthreads();
    }

    // Wave-uniform description of the tiles one wavefront owns in one item.
    struct Desc {
        int slot;                     // -1: none
        int r, g;
        int t0w;                      // first token of this wavefront's first tile
        int t1;                       // end of the item's token range
        int n_even;                   // tile slots this wavefront runs here (tiles rounded up to even)
        const unsigned char *kbase;
        const unsigned char *vbase;
        const_i32_ptr bt;
    };
    auto identify = [&](int slot, int &r, int &g, int &c, int &len) {
        const int it = j + slot * nwg;
        g = it % Hkv;
        if (split) {
            r = __builtin_amdgcn_readfirstlane(s_tab_r[slot]);
            c = __builtin_amdgcn_readfirstlane(s_tab_c[slot]);
            len = __builtin_amdgcn_readfirstlane(s_tab_len[slot]);
        } else {
            r = it / Hkv;
            c = 0;
            len = lens[r];
        }
    };
    auto describe = [&](int slot, Desc &d) {
        int r, g, c, len;
        identify(slot, r, g, c, len);
        d.slot = slot;
        d.r = r;
        d.g = g;
        d.t0w = c * C + w * TILE;
        d.t1 = min(len, c * C + C);
        const int nt = (d.t0w < d.t1) ? (d.t1 - d.t0w + step - 1) / step : 0;
        d.n_even = (nt + 1) & ~1;
        if (PAGED) {
            d.kbase = prm.k + (long long)g * prm.pool_stride_head_b;
            d.vbase = prm.v + (long long)g * prm.pool_stride_head_b;
            d.bt = (const_i32_ptr)(prm.block_table + (size_t)r * prm.bt_stride);
        } else {
            const long long off =
                (long long)r * prm.stride_req_b + (long long)g * prm.stride_head_b;
            d.kbase = prm.k + off;
            d.vbase = prm.v + off;
            d.bt = nullptr;
        }
    };
    // First item at or after `from` in which this wavefront has at least one tile.
    auto find_next = [&](int from, Desc &d) {
        d.slot = -1;
        for (int sl = from; sl < nslots; ++sl) {
            Desc t;
            describe(sl, t);
            if (t.n_even > 0) {
                d = t;
                return;
            }
        }
    };

    // Pool blocks of the 16-token pages of the tile starting at ts (wave-uniform scalar
    // loads), looked up one refill ahead of the loads that need them.
    auto fetch_pages = [&](const_i32_ptr bt, int ts, int last, int(&pg)[NSUB]) {
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
            pg[sub] = PAGED ? bt[min(ts + sub * 16, last) >> 4] : 0;
    };

    // Issue all loads of the tile starting at token ts.  Tokens beyond `last` (the item's
    // last valid token) are redirected to that row, so no byte outside the request is
    // touched; their scores are masked later.
    auto issue_loads = [&](const unsigned char *kbase, const unsigned char *vbase, int ts,
                           int last, const int(&pg)[NSUB], u32x4(&kr)[KR], u32x4(&vr)[VR]) {
        // Addresses are a wave-uniform 64-bit base (request/head, or pool page) plus a 32-bit
        // per-lane byte offset, which keeps address arithmetic and registers small.
        // K and V use the same lane mapping: an instruction covers whole rows (full 128-byte
        // lines).  Partial-line accesses lose what the non-temporal hint gains.
#pragma unroll
        for (int i = 0; i < KR; ++i) {
            const int tok = min(ts + i * RPI + lane / LPR, last);
            const int sub = (i * RPI) / 16;               // compile-time per instruction
            const unsigned char *base =
                PAGED ? kbase + (long long)pg[sub] * prm.pool_stride_block_b : kbase;
            const unsigned off = PAGED ? (unsigned)((tok & 15) * ROWB + (lane % LPR) * 16)
                                       : (unsigned)tok * (unsigned)prm.stride_tok_b +
                                             (lane % LPR) * 16;
            kr[i] = load_stream_128(base + off);
        }
#pragma unroll
        for (int i = 0; i < VR; ++i) {
            const int tok = min(ts + i * RPI + lane / LPR, last);
            const int sub = (i * RPI) / 16;               // compile-time per instruction
            const unsigned char *base =
                PAGED ? vbase + (long long)pg[sub] * prm.pool_stride_block_b : vbase;
            const unsigned off = PAGED ? (unsigned)((tok & 15) * ROWB + (lane % LPR) * 16)
                                       : (unsigned)tok * (unsigned)prm.stride_tok_b +
                                             (lane % LPR) * 16;
            vr[i] = load_stream_128(base + off);
        }
    };

    // Q as MFMA B operand: column = head col, k-step s holds 8 dims.  It is fetched as whole
    // rows -- one 1 KiB load instruction per four heads, lane = (head, 16-byte piece) -- and
    // turned into the operand layout through this wavefront's (idle between items) staging
    // area, because vector-memory instructions, not bytes, are what an item boundary costs.
    bf16x8 qop[4];
    auto request_q = [&](int r, int g, u32x4(&raw)[GQ]) {
        const unsigned char *qg = static_cast<const unsigned char *>(prm.q) +
                                  ((size_t)r * prm.Hq + g * G) * (kHeadDim * 2);
#pragma unroll
        for (int i = 0; i < GQ; ++i) {
            u32x4 z = {0u, 0u, 0u, 0u};
            raw[i] = z;
            if (i * 4 + (lane >> 4) < G)
                raw[i] = *reinterpret_cast<const u32x4 *>(qg + (i * 4 + (lane >> 4)) * 256 +
                                                          (lane & 15) * 16);
        }
    };
    auto install_q = [&](const u32x4(&raw)[GQ]) {
#pragma unroll
        for (int i = 0; i < GQ; ++i)
            *reinterpret_cast<u32x4 *>(vbuf + (i * 4 + (lane >> 4)) * 256 + (lane & 15) * 16) = raw[i];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            // The dims a lane holds in step s must be the dims its K register holds there.
            const int chunk8 = FP8 ? (((s >> 1) * 4 + quad) * 2 + (s & 1)) : (s * 4 + quad);
            bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
            qop[s] = z;
            if (col < GQ * 4)                             // rows at or above G hold zeros
                qop[s] = *reinterpret_cast<const bf16x8 *>(vbuf + col * 256 + chunk8 * 16);
        }
    };
    auto score_scale = [&](int r, int g) {
        float c = prm.scale_log2;
        if (FP8)                                          // K scale folds into the score scale
            c *= ((const __attribute__((address_space(4))) float *)prm.k_scale)[(size_t)r * Hkv + g];
        return c;
    };

    float m_run = -INFINITY;        // running max of log2-domain scores, head = col
    float l_run = 0.0f;             // this lane's share of the running denominator
    f32x4 o_acc[8];                 // O^T[dim = db*16 + quad*4 + v][head = col]
#pragma unroll
    for (int db = 0; db < 8; ++db) {
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
        o_acc[db] = z;
    }
    float c_log2 = 0.0f;
    int cur_t1 = 0;

    // First half of a tile: everything that reads the tile's load registers.
    auto consume = [&](const u32x4(&kr)[KR], const u32x4(&vr)[VR], f32x4(&sc)[NSUB]) {
        // K rows -> LDS (pitch KSTRIDE) -> MFMA A-operand layout (row = token col, the lane
        // holds the 16-byte piece s*4 + quad of that row in k-step s).  The staging area is
        // used for K first and for V afterwards; LDS operations of a wavefront execute in
        // order, so V cannot overtake the K reads.
#pragma unroll
        for (int i = 0; i < KR; ++i) {
            const int trow = i * RPI + lane / LPR;
            *reinterpret_cast<u32x4 *>(vbuf + trow * KSTRIDE + (lane % LPR) * 16) = kr[i];
        }
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            const unsigned char *krow = vbuf + (sub * 16 + col) * KSTRIDE + quad * 16;
            if (FP8) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const u32x4 raw = *reinterpret_cast<const u32x4 *>(krow + s2 * 64);
                    const bf16x8 lo = join_bf16x4(fp8x4_to_bf16(raw[0]), fp8x4_to_bf16(raw[1]));
                    const bf16x8 hi = join_bf16x4(fp8x4_to_bf16(raw[2]), fp8x4_to_bf16(raw[3]));
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo, qop[2 * s2], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi, qop[2 * s2 + 1], acc, 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const bf16x8 kop = *reinterpret_cast<const bf16x8 *>(krow + s * 64);
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
                s = (tok < cur_t1) ? s : -INFINITY;
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
        for (int jj = 0; jj < NSUB * 4; ++jj) {
            const float pj = fast_exp2(x[jj] - m_new);
            psum += pj;
            // p = hi + lo with both halves bf16: keeps ~16 significant bits through the MFMA
            const __bf16 h = static_cast<__bf16>(pj);
            p_hi[jj >> 3][jj & 7] = h;
            if (SPLIT_P)
                p_lo[jj >> 3][jj & 7] = static_cast<__bf16>(pj - static_cast<float>(h));
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

    // End of an item for ONE wavefront.  Nobody waits at a barrier: the wavefront parks its
    // (output, max, denominator) triple in LDS, counts itself in, and moves on to its next
    // item; whichever of the four arrives last combines the triples (same identity as the
    // cross-partition merge) and writes the item's result.  A wavefront can be at most one
    // item ahead: it may not overwrite its parked triple before that item was combined.
    auto finalize = [&](int slot) {
        l_run += __shfl_xor(l_run, 16);
        l_run += __shfl_xor(l_run, 32);
        {
            // (an LDS-typed pointer: a generic volatile read would be a FLAT load and drag the
            //  vector-memory counter, i.e. the prefetched tiles, into the wait)
            volatile __attribute__((address_space(3))) int *busy =
                (volatile __attribute__((address_space(3))) int *)&s_busy[w];
            while (*busy != 0)
                __builtin_amdgcn_s_sleep(2);
        }
        float *mine = s_trip + w * TRIP;
        if (col < G) {
#pragma unroll
            for (int db = 0; db < 8; ++db)
                *reinterpret_cast<f32x4 *>(mine + col * kHeadDim + db * 16 + quad * 4) = o_acc[db];
            if (quad == 0) {
                mine[kMaxGroup * kHeadDim + col] = m_run;
                mine[kMaxGroup * kHeadDim + kMaxGroup + col] = l_run;
            }
        }
        m_run = -INFINITY;
        l_run = 0.0f;
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            f32x4 z = {0.f, 0.f, 0.f, 0.f};
            o_acc[db] = z;
        }
        int arrived = 0;
        if (lane == 0)
            s_busy[w] = 1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        if (lane == 0)
            arrived = __hip_atomic_fetch_add(&s_count, 1, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_WORKGROUP);
        arrived = __builtin_amdgcn_readfirstlane(arrived);
        if (arrived != kWaves - 1)
            return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        int r, g, c, len;
        identify(slot, r, g, c, len);
        const bool whole = nparts(len) == 1;              // the request has no other partition
        float vs = 1.0f;
        if (FP8)
            vs = ((const __attribute__((address_space(4))) float *)prm.v_scale)[(size_t)r * Hkv + g];
        {
            // weights: lane = (head col, wavefront quad)
            const float mw = s_trip[quad * TRIP + kMaxGroup * kHeadDim + col];
            const float lw = s_trip[quad * TRIP + kMaxGroup * kHeadDim + kMaxGroup + col];
            float M = fmaxf(mw, __shfl_xor(mw, 16));
            M = fmaxf(M, __shfl_xor(M, 32));
            const float e = (mw == -INFINITY) ? 0.0f : fast_exp2(mw - M);   // idle wavefront
            float L = e * lw;
            L += __shfl_xor(L, 16);
            L += __shfl_xor(L, 32);
            const bool empty = !(L > 0.0f);               // a request with no tokens at all
            s_wgt[quad * kMaxGroup + col] = empty ? 0.0f : e * vs * __builtin_amdgcn_rcpf(L);
            if (quad == 0 && col < G) {
                const float lse_nat = empty ? -INFINITY : (M + __builtin_amdgcn_logf(L)) * kLn2;
                const size_t row = (size_t)r * prm.Hq + g * G + col;
                if (whole) {
                    if (prm.lse)
                        prm.lse[row] = lse_nat;
                } else {
                    prm.part_lse[row * prm.P + c] = lse_nat;
                }
            }
        }
        // outputs: lane = four consecutive dims of one head, two heads per pass
        for (int base = 0; base < G * 32; base += 64) {
            const int idx = base + lane;
            if (idx < G * 32) {
                const int h = idx >> 5;
                const int d4 = (idx & 31) * 4;
                f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ww = 0; ww < kWaves; ++ww) {
                    const f32x4 t =
                        *reinterpret_cast<const f32x4 *>(s_trip + ww * TRIP + h * kHeadDim + d4);
                    o += s_wgt[ww * kMaxGroup + h] * t;
                }
                const size_t row = (size_t)r * prm.Hq + g * G + h;
                if (!whole) {
                    *reinterpret_cast<f32x4 *>(prm.part_out + (row * prm.P + c) * kHeadDim + d4) = o;
                } else if (prm.out_is_bf16) {
                    u32x2 pk;
                    pk[0] = (unsigned)bf16_bits(o[0]) | ((unsigned)bf16_bits(o[1]) << 16);
                    pk[1] = (unsigned)bf16_bits(o[2]) | ((unsigned)bf16_bits(o[3]) << 16);
                    *reinterpret_cast<u32x2 *>(static_cast<unsigned short *>(prm.out) +
                                               row * kHeadDim + d4) = pk;
                } else {
                    *reinterpret_cast<f32x4 *>(static_cast<float *>(prm.out) + row * kHeadDim + d4) = o;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        if (lane == 0)
            s_count = 0;
        if (lane < kWaves)
            s_busy[lane] = 0;
    };

    // ---- stream -----------------------------------------------------------------------------
    u32x4 kA[KR], vA[VR], kB[KR], vB[VR];
    int pg[NSUB];
    f32x4 sc[NSUB];
    u32x4 qn[GQ];                   // Q rows of the wavefront's next item, requested an item ahead
    float cn = 0.0f;
    Desc nxt;
    find_next(0, nxt);
    if (nxt.slot >= 0) {
        // prologue: the first two tile slots of this wavefront's first item, and its Q
        fetch_pages(nxt.bt, nxt.t0w, nxt.t1 - 1, pg);
        issue_loads(nxt.kbase, nxt.vbase, nxt.t0w, nxt.t1 - 1, pg, kA, vA);
        __builtin_amdgcn_sched_barrier(0);                // A must be the older set
        fetch_pages(nxt.bt, nxt.t0w + step, nxt.t1 - 1, pg);
        issue_loads(nxt.kbase, nxt.vbase, nxt.t0w + step, nxt.t1 - 1, pg, kB, vB);
        __builtin_amdgcn_sched_barrier(0);
        if (Q_AHEAD)
            request_q(nxt.r, nxt.g, qn);
        cn = score_scale(nxt.r, nxt.g);
        wait_vmem_all();                                  // start-up only: nothing else to do yet
    }
    for (int slot = 0; slot < nslots; ++slot) {
        if (nxt.slot == slot) {
            // Sets A and B already hold (or are receiving) this item's first two tile slots.
            const Desc cur = nxt;
            cur_t1 = cur.t1;
            c_log2 = cn;
            if (!Q_AHEAD) {
                request_q(cur.r, cur.g, qn);
                wait_vmem_all();                          // also keeps the tile loop's waits exact
            }
            install_q(qn);
            find_next(slot + 1, nxt);
            // Where refills go once this item's tiles are exhausted: the next item's first
            // two slots, or -- at the very end -- harmless reloads of this item's last row.
            const bool more = nxt.slot >= 0;
            if (more) {
                if (Q_AHEAD)
                    request_q(nxt.r, nxt.g, qn);          // needed one whole item from now
                cn = score_scale(nxt.r, nxt.g);
            }
            const unsigned char *n_kbase = more ? nxt.kbase : cur.kbase;
            const unsigned char *n_vbase = more ? nxt.vbase : cur.vbase;
            const const_i32_ptr n_bt = more ? nxt.bt : cur.bt;
            const int n_t0w = more ? nxt.t0w : cur.t1;
            const int n_last = (more ? nxt.t1 : cur.t1) - 1;
            const int c_last = cur.t1 - 1;
            const int n_even = cur.n_even;
            // refill number idx (2, 3, ...) of this item -> its addressing, by scalar selects
            auto target = [&](int idx, const unsigned char *&kb, const unsigned char *&vb,
                              const_i32_ptr &bt, int &ts, int &last) {
                const bool in_item = idx < n_even;
                kb = in_item ? cur.kbase : n_kbase;
                vb = in_item ? cur.vbase : n_vbase;
                bt = in_item ? cur.bt : n_bt;
                ts = in_item ? cur.t0w + idx * step : n_t0w + (idx - n_even) * step;
                last = in_item ? c_last : n_last;
            };
            const unsigned char *kb, *vb;
            const_i32_ptr bt;
            int rts, rlast;
            target(2, kb, vb, bt, rts, rlast);
            fetch_pages(bt, rts, rlast, pg);
            int ts = cur.t0w;
            for (int k = 0; k < n_even; k += 2) {
                consume(kA, vA, sc);
                __builtin_amdgcn_sched_barrier(0);
                target(k + 2, kb, vb, bt, rts, rlast);
                issue_loads(kb, vb, rts, rlast, pg, kA, vA);
                target(k + 3, kb, vb, bt, rts, rlast);
                fetch_pages(bt, rts, rlast, pg);
                __builtin_amdgcn_sched_barrier(0);
                finish(ts, sc);
                __builtin_amdgcn_sched_barrier(0);
                consume(kB, vB, sc);
                __builtin_amdgcn_sched_barrier(0);
                issue_loads(kb, vb, rts, rlast, pg, kB, vB);
                target(k + 4, kb, vb, bt, rts, rlast);
                fetch_pages(bt, rts, rlast, pg);
                __builtin_amdgcn_sched_barrier(0);
                finish(ts + step, sc);
                __builtin_amdgcn_sched_barrier(0);
                ts += 2 * step;
            }
        }
        finalize(slot);
    }
}

// -------------------------------------------------------------------------------------------
// Cross-partition merge (Sec. 4.2.2 identity, P parts, log-sum-exp form):
//   lse = ln sum_p e^{lse_p},  out = sum_p e^{lse_p - lse} out_p.
// One wavefront per (request, query head) row, four rows per work-group; lane d owns output
// columns 2d and 2d+1.  Lane p first holds partition p's weight (the log-sum-exp reduction is
// two wave reductions), then all lanes stream the partial outputs with independent loads.
// Only the first ceil(len / chunk) partitions were written by the main pass, and a request
// with a single partition was already written to out/lse by the main pass.
// -------------------------------------------------------------------------------------------
constexpr int kMergeRowsPerBlock = 4;

__global__ __launch_bounds__(64 * kMergeRowsPerBlock) void merge_partials_kernel(const MergeParams prm)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * kMergeRowsPerBlock + (threadIdx.x >> 6);   // r * Hq + h
    if (row >= prm.rows)
        return;
    const int r = row / prm.Hq;
    const int len = prm.seq_lens[r];
    const int chunk = *prm.chunk_used;
    const int np = min(prm.P, max(1, (len + chunk - 1) / chunk));
    if (np == 1)
        return;                                           // the main pass wrote this row itself
    const float *pl = prm.part_lse + (size_t)row * prm.P;
    const float *po = prm.part_out + (size_t)row * prm.P * kHeadDim;
    float M = -INFINITY;
    for (int p0 = 0; p0 < np; p0 += 64) {
        const float v = (p0 + lane < np) ? pl[p0 + lane] : -INFINITY;
        M = fmaxf(M, v);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        M = fmaxf(M, __shfl_xor(M, off));
    float W = 0.0f;
    float o0 = 0.0f, o1 = 0.0f;
    for (int p0 = 0; p0 < np; p0 += 64) {
        const float e = (p0 + lane < np) ? __expf(pl[p0 + lane] - M) : 0.0f;
        W += e;
        const int cnt = min(64, np - p0);
#pragma unroll 4
        for (int p = 0; p < cnt; ++p) {
            const float w = __shfl(e, p);
            const float2 t = *reinterpret_cast<const float2 *>(po + (size_t)(p0 + p) * kHeadDim +
                                                              2 * lane);
            o0 += w * t.x;
            o1 += w * t.y;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        W += __shfl_xor(W, off);
    const float inv = 1.0f / W;
    const size_t at = (size_t)row * kHeadDim + 2 * lane;
    if (prm.out_is_bf16) {
        static_cast<unsigned *>(prm.out)[at >> 1] =
            (unsigned)bf16_bits(o0 * inv) | ((unsigned)bf16_bits(o1 * inv) << 16);
    } else {
        *reinterpret_cast<float2 *>(static_cast<float *>(prm.out) + at) = make_float2(o0 * inv, o1 * inv);
    }
    if (lane == 0 && prm.lse)
        prm.lse[row] = M + logf(W);
}

// -------------------------------------------------------------------------------------------
// The new token's rows (Sec. 4.2.2: k_n, v_n arrive after q_n).
// -------------------------------------------------------------------------------------------
struct NewTokenParams {
    const unsigned short *q;           // bf16 [R][Hq][128]        (fold only)
    const unsigned short *k_new;       // bf16 [R][Hkv][128]
    const unsigned short *v_new;
    unsigned char *k_cache;            // append only
    unsigned char *v_cache;
    const int32_t *positions;
    const int32_t *block_table;
    const float *k_scale;
    const float *v_scale;
    const float *out_prev;             // fold only
    const float *lse_prev;
    void *out;
    float *lse;
    long long stride_req_b, stride_head_b, stride_tok_b;
    long long pool_stride_block_b, pool_stride_head_b;
    int bt_stride;
    int Hq, Hkv, G;
    int rows;                          // append: R * Hkv, fold: R * Hq
    int fp8, paged, out_is_bf16;
    float scale;
};

__device__ __forceinline__ float bf16_bits_to_float(unsigned short b)
{
    return __builtin_bit_cast(float, (unsigned)b << 16);
}

// x -> the value an fp8 cache holds for it: e4m3fn(rne(x / scale)) (saturating), as a byte.
__device__ __forceinline__ unsigned char quantise_e4m3fn(float x, float inv_scale)
{
    const float y = fminf(fmaxf(x * inv_scale, -448.0f), 448.0f);
    return (unsigned char)(__builtin_amdgcn_cvt_pk_fp8_f32(y, 0.0f, 0, false) & 0xFF);
}

__device__ __forceinline__ float dequantise_e4m3fn(unsigned char b, float scale)
{
    const bf16x2 v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)b, 1.0f, false);
    return static_cast<float>(v[0]) * scale;
}

// One wavefront per (request, kv head): lane i moves elements 2i and 2i+1 of the K and V rows.
__global__ __launch_bounds__(256) void append_kv_kernel(const NewTokenParams prm)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);   // r * Hkv + g
    if (row >= prm.rows)
        return;
    const int r = row / prm.Hkv;
    const int g = row % prm.Hkv;
    const int pos = prm.positions[r];
    if (pos < 0)
        return;
    const int esz = prm.fp8 ? 1 : 2;
    long long off;
    if (prm.paged) {
        const long long blk = prm.block_table[(size_t)r * prm.bt_stride + (pos >> 4)];
        off = blk * prm.pool_stride_block_b + (long long)g * prm.pool_stride_head_b +
              (long long)(pos & 15) * kHeadDim * esz;
    } else {
        off = (long long)r * prm.stride_req_b + (long long)g * prm.stride_head_b +
              (long long)pos * prm.stride_tok_b;
    }
    const unsigned kk = reinterpret_cast<const unsigned *>(prm.k_new)[(size_t)row * 64 + lane];
    const unsigned vv = reinterpret_cast<const unsigned *>(prm.v_new)[(size_t)row * 64 + lane];
    if (!prm.fp8) {
        reinterpret_cast<unsigned *>(prm.k_cache + off)[lane] = kk;
        reinterpret_cast<unsigned *>(prm.v_cache + off)[lane] = vv;
    } else {
        const float iks = 1.0f / prm.k_scale[row];
        const float ivs = 1.0f / prm.v_scale[row];
        const unsigned short kq =
            (unsigned short)quantise_e4m3fn(bf16_bits_to_float(kk & 0xFFFF), iks) |
            ((unsigned short)quantise_e4m3fn(bf16_bits_to_float(kk >> 16), iks) << 8);
        const unsigned short vq =
            (unsigned short)quantise_e4m3fn(bf16_bits_to_float(vv & 0xFFFF), ivs) |
            ((unsigned short)quantise_e4m3fn(bf16_bits_to_float(vv >> 16), ivs) << 8);
        reinterpret_cast<unsigned short *>(prm.k_cache + off)[lane] = kq;
        reinterpret_cast<unsigned short *>(prm.v_cache + off)[lane] = vq;
    }
}

// One wavefront per (request, query head): the two-part case of the Sec. 4.2.2 identity with
// I1 = previous tokens (given as A, ln S) and I2 = {new token} (A = v_new, ln S = s).
__global__ __launch_bounds__(256) void fold_new_token_kernel(const NewTokenParams prm)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);   // r * Hq + h
    if (row >= prm.rows)
        return;
    const int r = row / prm.Hq;
    const int g = (row % prm.Hq) / prm.G;
    const size_t kvrow = (size_t)r * prm.Hkv + g;
    const unsigned qq = reinterpret_cast<const unsigned *>(prm.q)[(size_t)row * 64 + lane];
    const unsigned kk = reinterpret_cast<const unsigned *>(prm.k_new)[kvrow * 64 + lane];
    const unsigned vv = reinterpret_cast<const unsigned *>(prm.v_new)[kvrow * 64 + lane];
    float k0 = bf16_bits_to_float(kk & 0xFFFF), k1 = bf16_bits_to_float(kk >> 16);
    float v0 = bf16_bits_to_float(vv & 0xFFFF), v1 = bf16_bits_to_float(vv >> 16);
    if (prm.fp8) {
        const float ks = prm.k_scale[kvrow], vs = prm.v_scale[kvrow];
        k0 = dequantise_e4m3fn(quantise_e4m3fn(k0, 1.0f / ks), ks);
        k1 = dequantise_e4m3fn(quantise_e4m3fn(k1, 1.0f / ks), ks);
        v0 = dequantise_e4m3fn(quantise_e4m3fn(v0, 1.0f / vs), vs);
        v1 = dequantise_e4m3fn(quantise_e4m3fn(v1, 1.0f / vs), vs);
    }
    float dot = bf16_bits_to_float(qq & 0xFFFF) * k0 + bf16_bits_to_float(qq >> 16) * k1;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        dot += __shfl_xor(dot, off);
    const float s = dot * prm.scale;
    const float lp = prm.lse_prev[row];
    const float m = fmaxf(lp, s);                         // s is finite, so m is
    const float wp = (lp == -INFINITY) ? 0.0f : __expf(lp - m);
    const float wn = __expf(s - m);
    const float inv = 1.0f / (wp + wn);
    const float2 op = wp > 0.0f
                          ? *reinterpret_cast<const float2 *>(prm.out_prev + (size_t)row * kHeadDim + 2 * lane)
                          : make_float2(0.0f, 0.0f);
    const float o0 = (wp * op.x + wn * v0) * inv;
    const float o1 = (wp * op.y + wn * v1) * inv;
    const size_t at = (size_t)row * kHeadDim + 2 * lane;
    if (prm.out_is_bf16)
        static_cast<unsigned *>(prm.out)[at >> 1] =
            (unsigned)bf16_bits(o0) | ((unsigned)bf16_bits(o1) << 16);
    else
        *reinterpret_cast<float2 *>(static_cast<float *>(prm.out) + at) = make_float2(o0, o1);
    if (lane == 0 && prm.lse)
        prm.lse[row] = m + logf(wp + wn);
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
    int resident_wgs;            // persistent grid: two work-groups per compute unit
    char err[256];
};

namespace {

thread_local char g_create_err[256] = "";

int round_up(int x, int m) { return (x + m - 1) / m * m; }

struct Plan {
    int num_splits;
    int split_tokens;
};

// Most work items any call may produce: every resident work-group keeps a table of at most
// kTableSlots items, and the grid has at least kMinGrid work-groups.
constexpr long long kMinGrid = 256;
constexpr long long kMaxItems = kTableSlots * kMinGrid;

// Partitioning.  Explicit num_splits is honoured exactly.  Otherwise: batches that already hold
// one item per resident work-group with contexts of at most 4096 tokens stay unsplit (no
// partial results at all); everything else gets a BASE partition of 512 KiB of K+V per kv head
// (1024 bf16 tokens, 2048 fp8 tokens; more if the item budget requires), which the kernel
// itself doubles up to four times per call depending on how much work seq_lens holds.
// (Measured: items of 512 tokens lose 10-20 % to per-item costs on small batches; items of
// 1024 tokens cost a 64-head layer 11 % against 4096-token items once the batch is large.)
Plan make_plan(const lamina_attn_config &c)
{
    Plan pl;
    const long long pairs = (long long)c.max_batch * c.num_kv_heads;
    int P;
    if (c.num_splits >= 1) {
        P = c.num_splits;
    } else if (c.max_seq_len <= 4096 && pairs >= 256) {
        P = 1;
    } else {
        int target = c.kv_dtype == LAMINA_FP8_E4M3 ? 2048 : 1024;
        while (pairs * ((c.max_seq_len + target - 1) / target) > kMaxItems)
            target *= 2;
        P = (c.max_seq_len + target - 1) / target;
    }
    if (P < 1)
        P = 1;
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
    if (c->num_splits > 1) {
        if (c->max_batch > kMaxSplitBatch)
            return "a partitioned handle supports max_batch up to 1024";
        if ((long long)c->max_batch * c->num_kv_heads * c->num_splits > kMaxItems)
            return "max_batch * num_kv_heads * num_splits above 65536";
    }
    *code = LAMINA_OK;
    return nullptr;
}

size_t workspace_bytes_for(const lamina_attn_config &c, const Plan &pl)
{
    if (pl.num_splits <= 1)
        return 0;
    // partial outputs, partial lse, and one int: the partition size the last call settled on
    return (size_t)c.max_batch * c.num_q_heads * pl.num_splits * (kHeadDim + 1) * sizeof(float) + 16;
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
    {
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, cfg->device);
        if (e != hipSuccess || cus <= 0) {
            snprintf(g_create_err, sizeof g_create_err, "cannot query compute units: %s",
                     hipGetErrorString(e));
            delete h;
            return LAMINA_ERR_HIP;
        }
        h->resident_wgs = 2 * cus;
        if (pl.num_splits > 1 && (h->resident_wgs < kMinGrid || cfg->max_batch > kMaxSplitBatch)) {
            snprintf(g_create_err, sizeof g_create_err,
                     "partitioned handles need max_batch <= %d and a device with >= %lld compute units",
                     kMaxSplitBatch, kMinGrid / 2);
            delete h;
            return LAMINA_ERR_UNSUPPORTED;
        }
    }
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
        e = hipMemset(reinterpret_cast<char *>(h->workspace) + h->workspace_bytes - 16, 0, 16);
        if (e == hipSuccess)
            e = hipDeviceSynchronize();
        if (e != hipSuccess) {
            snprintf(g_create_err, sizeof g_create_err, "clearing the workspace: %s",
                     hipGetErrorString(e));
            (void)hipFree(h->workspace);
            delete h;
            return LAMINA_ERR_HIP;
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

int lamina_attn_used_split_tokens(lamina_attn_t h)
{
    if (!h)
        return 0;
    if (h->num_splits <= 1)
        return h->split_tokens;
    int used = 0;
    DeviceGuard guard(h->cfg.device);
    const char *at = reinterpret_cast<const char *>(h->workspace) + h->workspace_bytes - 16;
    if (!guard.ok() || hipMemcpy(&used, at, sizeof used, hipMemcpyDeviceToHost) != hipSuccess)
        return LAMINA_ERR_HIP;
    return used;
}

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

    if (!paged && (long long)c.max_seq_len * p->kv_stride_tok * esz >= (1LL << 32))
        return fail(h, LAMINA_ERR_UNSUPPORTED,
                    "max_seq_len * kv_stride_tok must stay below 4 GiB per (request, kv head)");
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
    mp.batch = p->batch;
    mp.out_is_bf16 = c.out_dtype == LAMINA_BF16;
    mp.scale_log2 = h->scale * kLog2e;
    if (h->num_splits > 1) {
        mp.part_out = h->workspace;
        mp.part_lse = h->workspace + (size_t)c.max_batch * c.num_q_heads * h->num_splits * kHeadDim;
        mp.chunk_used = reinterpret_cast<int *>(
            mp.part_lse + (size_t)c.max_batch * c.num_q_heads * h->num_splits);
        mp.adapt = c.num_splits == 0;                     // an explicit partition count is kept
    }

    DeviceGuard guard(c.device);
    if (!guard.ok())
        return fail(h, LAMINA_ERR_HIP, "cannot select the handle's device");
    hipStream_t stream = static_cast<hipStream_t>(p->stream);
    // Persistent grid: never more work-groups than can be resident, never more than items.
    long long wgs = (long long)p->batch * c.num_kv_heads * h->num_splits;
    if (wgs > h->resident_wgs)
        wgs = h->resident_wgs;
    if (h->num_splits == 1 &&
        ((long long)p->batch * c.num_kv_heads + wgs - 1) / wgs > 0x3fffffffLL / kThreads)
        return fail(h, LAMINA_ERR_UNSUPPORTED, "batch too large");
    const dim3 grid((unsigned)wgs), block(kThreads);
    // Kernel variant: cache dtype x layout x number of four-head Q row groups.
    const int gq = h->group <= 4 ? 1 : (h->group <= 8 ? 2 : 4);
#define LAMINA_LAUNCH(F8, PG)                                                                  \
    do {                                                                                       \
        if (gq == 1)                                                                           \
            hipLaunchKernelGGL((decode_mfma_kernel<F8, PG, 1>), grid, block, 0, stream, mp);   \
        else if (gq == 2)                                                                      \
            hipLaunchKernelGGL((decode_mfma_kernel<F8, PG, 2>), grid, block, 0, stream, mp);   \
        else                                                                                   \
            hipLaunchKernelGGL((decode_mfma_kernel<F8, PG, 4>), grid, block, 0, stream, mp);   \
    } while (0)
    if (fp8 && paged)
        LAMINA_LAUNCH(true, true);
    else if (fp8)
        LAMINA_LAUNCH(true, false);
    else if (paged)
        LAMINA_LAUNCH(false, true);
    else
        LAMINA_LAUNCH(false, false);
#undef LAMINA_LAUNCH
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
        gp.chunk_used = mp.chunk_used;
        gp.out_is_bf16 = mp.out_is_bf16;
        gp.rows = p->batch * c.num_q_heads;
        hipLaunchKernelGGL(merge_partials_kernel,
                           dim3((unsigned)((gp.rows + kMergeRowsPerBlock - 1) / kMergeRowsPerBlock)),
                           dim3(64 * kMergeRowsPerBlock), 0, stream, gp);
        e = hipGetLastError();
        if (e != hipSuccess)
            return fail_hip(h, "merge kernel launch", e);
    }
    return LAMINA_OK;
}

}  // extern "C"

namespace {

// Shared argument checks of the two new-token entry points.  Returns nullptr if fine.
const char *check_new_token_args(const lamina_attn *h, const lamina_call_params *p, bool need_layout,
                                 const void *block_table)
{
    const lamina_attn_config &c = h->cfg;
    if (!p)
        return "call params are NULL";
    if (p->batch < 0 || p->batch > c.max_batch)
        return "batch is negative or exceeds max_batch";
    if (c.kv_dtype == LAMINA_FP8_E4M3 && (!p->k_scale || !p->v_scale))
        return "fp8 cache needs k_scale and v_scale";
    if (!need_layout)
        return nullptr;
    const int esz = c.kv_dtype == LAMINA_FP8_E4M3 ? 1 : 2;
    if (c.block_size != 0) {
        if (!block_table)
            return "paged cache needs a block_table";
        if (p->pool_stride_head < (long long)c.block_size * kHeadDim || p->pool_stride_block <= 0 ||
            p->block_table_stride <= 0 || (p->pool_stride_head * esz) % 16 != 0 ||
            (p->pool_stride_block * esz) % 16 != 0)
            return "bad pool strides or block_table_stride";
    } else if (p->kv_stride_tok < kHeadDim || p->kv_stride_req < 0 || p->kv_stride_head < 0 ||
               (p->kv_stride_tok * esz) % 16 != 0 || (p->kv_stride_req * esz) % 16 != 0 ||
               (p->kv_stride_head * esz) % 16 != 0) {
        return "bad contiguous-cache strides";
    }
    return nullptr;
}

void fill_new_token_params(const lamina_attn *h, const lamina_call_params *p, NewTokenParams &np)
{
    const lamina_attn_config &c = h->cfg;
    const int esz = c.kv_dtype == LAMINA_FP8_E4M3 ? 1 : 2;
    memset(&np, 0, sizeof np);
    np.k_scale = p->k_scale;
    np.v_scale = p->v_scale;
    np.stride_req_b = p->kv_stride_req * esz;
    np.stride_head_b = p->kv_stride_head * esz;
    np.stride_tok_b = p->kv_stride_tok * esz;
    np.pool_stride_block_b = p->pool_stride_block * esz;
    np.pool_stride_head_b = p->pool_stride_head * esz;
    np.bt_stride = p->block_table_stride;
    np.Hq = c.num_q_heads;
    np.Hkv = c.num_kv_heads;
    np.G = h->group;
    np.fp8 = c.kv_dtype == LAMINA_FP8_E4M3;
    np.paged = c.block_size != 0;
    np.out_is_bf16 = c.out_dtype == LAMINA_BF16;
    np.scale = h->scale;
}

}  // namespace

extern "C" {

int lamina_append_kv(lamina_attn_t h, const void *k_new, const void *v_new, void *k_cache,
                     void *v_cache, const int32_t *positions, const int32_t *block_table,
                     const lamina_call_params *p)
{
    if (!h)
        return LAMINA_ERR_INVALID_ARG;
    h->err[0] = 0;
    if (const char *msg = check_new_token_args(h, p, true, block_table))
        return fail(h, LAMINA_ERR_INVALID_ARG, msg);
    if (p->batch == 0)
        return LAMINA_OK;
    if (!k_new || !v_new || !k_cache || !v_cache || !positions)
        return fail(h, LAMINA_ERR_INVALID_ARG,
                    "k_new, v_new, k_cache, v_cache and positions must be non-NULL");
    if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)k_cache | (uintptr_t)v_cache) % 16 != 0)
        return fail(h, LAMINA_ERR_INVALID_ARG, "k_new, v_new and the caches must be 16-byte aligned");
    NewTokenParams np;
    fill_new_token_params(h, p, np);
    np.k_new = static_cast<const unsigned short *>(k_new);
    np.v_new = static_cast<const unsigned short *>(v_new);
    np.k_cache = static_cast<unsigned char *>(k_cache);
    np.v_cache = static_cast<unsigned char *>(v_cache);
    np.positions = positions;
    np.block_table = block_table;
    np.rows = p->batch * h->cfg.num_kv_heads;
    DeviceGuard guard(h->cfg.device);
    if (!guard.ok())
        return fail(h, LAMINA_ERR_HIP, "cannot select the handle's device");
    hipLaunchKernelGGL(append_kv_kernel, dim3((unsigned)((np.rows + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(p->stream), np);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(h, "append kernel launch", e);
    return LAMINA_OK;
}

int lamina_fold_new_token(lamina_attn_t h, const void *q, const void *k_new, const void *v_new,
                          const float *out_prev, const float *lse_prev, void *out, float *lse,
                          const lamina_call_params *p)
{
    if (!h)
        return LAMINA_ERR_INVALID_ARG;
    h->err[0] = 0;
    if (const char *msg = check_new_token_args(h, p, false, nullptr))
        return fail(h, LAMINA_ERR_INVALID_ARG, msg);
    if (p->batch == 0)
        return LAMINA_OK;
    if (!q || !k_new || !v_new || !out_prev || !lse_prev || !out)
        return fail(h, LAMINA_ERR_INVALID_ARG,
                    "q, k_new, v_new, out_prev, lse_prev and out must be non-NULL");
    if (((uintptr_t)q | (uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)out_prev | (uintptr_t)out) % 8 != 0)
        return fail(h, LAMINA_ERR_INVALID_ARG, "tensors must be 8-byte aligned");
    if ((const void *)out_prev == (const void *)out && h->cfg.out_dtype != LAMINA_F32)
        return fail(h, LAMINA_ERR_INVALID_ARG, "out may alias out_prev only for fp32 output");
    NewTokenParams np;
    fill_new_token_params(h, p, np);
    np.q = static_cast<const unsigned short *>(q);
    np.k_new = static_cast<const unsigned short *>(k_new);
    np.v_new = static_cast<const unsigned short *>(v_new);
    np.out_prev = out_prev;
    np.lse_prev = lse_prev;
    np.out = out;
    np.lse = lse;
    np.rows = p->batch * h->cfg.num_q_heads;
    DeviceGuard guard(h->cfg.device);
    if (!guard.ok())
        return fail(h, LAMINA_ERR_HIP, "cannot select the handle's device");
    hipLaunchKernelGGL(fold_new_token_kernel, dim3((unsigned)((np.rows + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(p->stream), np);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(h, "fold kernel launch", e);
    return LAMINA_OK;
}

}  // extern "C"
