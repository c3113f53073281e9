// Decode attention for gfx950 (MI355X): kernels and the C ABI declared in lamina_attn.h.
//
// The operator (paper Sec. 2.1, starred equation, per head; GQA per Sec. 2.2.2): for each
// request r and query head h, out = sum_j softmax_j(scale * q.K_j) V_j over the request's
// own KV cache.  It is a batched matrix-vector product whose arithmetic intensity does not
// grow with the batch (Sec. 2.2.2), so the kernel is organised around streaming K and V
// from HBM exactly once:
//
//   * a persistent grid of 4-wavefront work-groups shares out the (request, kv head) rows --
//     whole, in fixed partitions, or in equal token shares cut from seq_lens on the device;
//     the G query heads of a group share every K/V tile that is loaded;
//   * every wavefront streams its own 32-token tiles (64 for fp8 caches) with non-temporal
//     128-bit loads of whole rows, one tile ahead of the arithmetic, and never synchronises
//     with its neighbours until an item ends;
//   * q.K^T and p.V run on the matrix cores (16x16x32 bf16 MFMA, the G heads padded to 16
//     columns; e4m3 operands for fp8 caches) so that the vector ALU only does the softmax; K
//     and V tiles are staged through LDS into the operand layouts (V transposed);
//   * pieces of a cut row keep (A_q(I), ln S_q(I)) of Sec. 4.2.2 and a second kernel combines
//     them with the divide-and-conquer identity of that section.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "lamina_attn.h"
#include "lamina_shares.h"

// Partial results of lamina_decode_attention_static, the entry point that allocates nothing:
// one copy of this array per GPU the library runs on, held until the process ends.  In host
// code this name is only a stand-in for the symbol; the device address comes from
// hipGetSymbolAddress (static_scratch_for below) and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[LAMINA_STATIC_SCRATCH_BYTES];

// -------------------------------------------------------------------------------------------
// Timeline build (-DLAMINA_TRACE, see `bench.py --timeline`): every wavefront of the main pass
// and every work-group of the merge passes stamps the device's constant 100 MHz clock at a
// few points -- entry, work range known, first loads issued, first data there, every loop
// iteration early on and every fourth later, end of its tiles, exit -- and leaves the stamps in
// a device array that lamina_trace_read copies out.  Without the macro none of it exists.
// -------------------------------------------------------------------------------------------
#ifdef LAMINA_TRACE
constexpr int kTraceWaves = 4096;                      // main pass: kMaxGrid x 4 wavefronts
constexpr int kTraceWaveWords = 64;
constexpr int kTraceMergeGroups = 4096;
constexpr int kTraceMergeWords = 4;
constexpr int kTraceStamps = 40;                       // loop stamps kept per wavefront
__device__ unsigned long long g_trace[kTraceWaves * kTraceWaveWords + kTraceMergeGroups * kTraceMergeWords];
extern "C" int lamina_trace_read(unsigned long long *host, size_t words)
{
    const size_t have = sizeof(g_trace) / sizeof(g_trace[0]);
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace), sizeof(g_trace[0]) * (words < have ? words : have));
}
#define LAMINA_TRACE_ONLY(...) __VA_ARGS__
#else
#define LAMINA_TRACE_ONLY(...)
#endif

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// Read-only index arrays are read through the constant address space so that uniform reads
// stay on the scalar unit (and off the in-order vector-memory counter) inside the tile loop.
typedef const __attribute__((address_space(4))) int32_t *const_i32_ptr;

constexpr int kHeadDim = 128;
constexpr int kWaves = 4;              // wavefronts per work-group
constexpr int kThreads = kWaves * 64;
constexpr int kChunkAlign = 256;       // partition sizes are multiples of 4 wavefronts x 64 tokens
constexpr int kMaxGroup = 16;          // query heads per kv head the MFMA tile can hold
constexpr int kMaxSplitBatch = 1024;   // requests per call when the KV range is partitioned
// How the KV range of a (request, kv head) row is cut into the pieces work-groups process.
enum : int {
    kModeRows = 0,                     // never cut: a piece is a whole row
    kModeFixed = 1,                    // fixed partitions of `unit` tokens, each its own piece
    kModeBalanced = 2                  // equal shares of the call's tokens per work-group
};
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
    float *part_out;                   // [piece][G][128], normalised partial outputs
    float *part_lse;                   // [piece][G], natural-log partial denominators
    int *cum;                          // [R + 1]: units before request r, written by the main pass
                                       // (fixed partitions: the merge pass reads it back)
    int *tails;                        // balanced shares: per work-group, the row whose last piece
                                       // is that work-group's first item (4 ints each, see below)
    const float *k_scale;
    const float *v_scale;
    long long stride_req_b, stride_head_b, stride_tok_b;     // bytes (contiguous mode)
    long long pool_stride_block_b, pool_stride_head_b;       // bytes (paged mode)
    int bt_stride;
    int Hq, Hkv, G;
    int mode;                          // kModeRows / kModeFixed / kModeBalanced
    int P;                             // kModeFixed: partitions per row at most
    int unit;                          // tokens per unit (split modes)
    int row_cost;                      // balanced mode: units a row weighs beyond its tokens
    int len_cap;                       // seq_lens values are clamped to this (memory safety)
    int batch;
    int out_is_bf16;
    float scale_log2;                  // softmax scale times log2(e)
};

struct MergeParams {
    const float *part_out;
    const float *part_lse;
    void *out;
    float *lse;
    const int *cum;                    // [R + 1], units before request r (from the main pass)
    int Hq, Hkv, G;
    int rows;                          // R * Hq
    int out_is_bf16;
};

// Fixed partitions: with at least kWaveItemParts partitions per wavefront of the grid the
// WAVEFRONTS take shares of their own (4 x nwg workers) and each works through its partitions
// alone -- consecutive tiles, no combining with its neighbours, a third of the cost per item;
// with fewer, the four wavefronts of a work-group share every item (tiles w, w+4, ...), which
// keeps all of them busy.  (Tried for balanced shares too: rows get cut four times as often,
// and workloads 5, 7 and uniform batches lost 0-3 %.)
constexpr unsigned kWaveItemParts = 2;
__host__ __device__ inline bool wave_items_rule(int mode, unsigned U, unsigned nwg)
{
    return mode == kModeFixed && U >= kWaveItemParts * kWaves * nwg;
}

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

__device__ __forceinline__ bf16x8 join_bf16x4(bf16x4 a, bf16x4 b)
{
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

// x = hi + lo with hi and lo both e4m3fn (round to nearest even): four values -> one dword of
// hi bytes and one of lo bytes, value i in byte i.  |x| must stay below 448 (the convert does
// not saturate).  hi keeps 4 significant bits and lo the next 4, so a value with at most 8
// significant bits (any bf16) splits exactly unless lo falls below 2^-9.
__device__ __forceinline__ void split_fp8x4(float x0, float x1, float x2, float x3, int &hi, int &lo)
{
    int h = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, 0, false);
    h = __builtin_amdgcn_cvt_pk_fp8_f32(x2, x3, h, true);
    const f32x2 b01 = __builtin_amdgcn_cvt_pk_f32_fp8(h, false);
    const f32x2 b23 = __builtin_amdgcn_cvt_pk_f32_fp8(h, true);
    int l = __builtin_amdgcn_cvt_pk_fp8_f32(x0 - b01[0], x1 - b01[1], 0, false);
    l = __builtin_amdgcn_cvt_pk_fp8_f32(x2 - b23[0], x3 - b23[1], l, true);
    hi = h;
    lo = l;
}

// Reductions over the four lanes {c, c+16, c+32, c+48} that hold one head's statistics.  The
// gfx950 row-swap instructions exchange 16- and 32-lane halves inside the vector ALU, so the
// running-max update of every tile neither passes through the LDS crossbar (ds_bpermute) nor
// shares its wait counter with the LDS traffic of the tile.
// v_permlane16_swap(x, x) leaves {rows 0,0,2,2 of x} and {rows 1,1,3,3 of x}; v_permlane32_swap(x, x)
// leaves {lower half, lower half} and {upper half, upper half}: combining the two results is the
// butterfly step with distance 16 resp. 32.  (The element reads go through scalars: a bit_cast
// applied directly to a vector element reads element 0 on this compiler.)
__device__ __forceinline__ void swap16(float x, float &a, float &b)
{
    const unsigned xi = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
    const unsigned ra = r[0], rb = r[1];
    a = __builtin_bit_cast(float, ra);
    b = __builtin_bit_cast(float, rb);
}
__device__ __forceinline__ void swap32(float x, float &a, float &b)
{
    const unsigned xi = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    const unsigned ra = r[0], rb = r[1];
    a = __builtin_bit_cast(float, ra);
    b = __builtin_bit_cast(float, rb);
}
__device__ __forceinline__ float quad_max(float x)
{
    float a, b;
    swap16(x, a, b);
    x = fmaxf(a, b);
    swap32(x, a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ float quad_sum(float x)
{
    float a, b;
    swap16(x, a, b);
    x = a + b;
    swap32(x, a, b);
    return a + b;
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

// -------------------------------------------------------------------------------------------
// Main pass: a persistent kernel.  The grid is a fixed number of work-groups (two per compute
// unit; one for balanced shares) that stay resident and share out the call's work among
// themselves.
//
// Work.  The rows (request r, kv head g), g fastest, are laid end to end as a stream of UNITS:
// row (r, g) holds n(r) units, where
//   rows mode       n = 1 (the row is never cut),
//   fixed mode      n = number of `unit`-token partitions of seq_lens[r] (at least one),
//   balanced mode   n = number of 128-token (bf16) / 256-token (fp8) blocks (at least one).
// Work-group j takes a contiguous range of units: all ranges equal to within one unit, except
// that large balanced calls weight the ranges by the parity of j (share_skew: work-groups go
// round-robin to the eight dies, and the odd dies stream several per cent slower).  In
// rows and fixed mode every unit is one ITEM; in balanced mode an item is the part of one row
// that falls into the work-group's range, however long -- so every work-group streams its
// share of the tokens whatever the mix of lengths, and a row is cut only where a range ends
// (at most one extra partial result per work-group).  Every work-group derives its range
// itself from seq_lens (a prefix sum in LDS), so the host never reads seq_lens and no
// planning kernel runs.
//
// Inside an item the four wavefronts take 32-token (bf16) or 64-token (fp8) tiles
// w, w+4, w+8, ... and never synchronise until the item ends, where they combine their
// (max, denominator, output) triples through LDS -- the same identity as the cross-partition
// merge.  An item that covers its whole row is written straight to out/lse; otherwise the
// item writes the partial pair (A_q(I), ln S_q(I)) of Sec. 4.2.2 to the workspace, at piece
// index `unit number` (fixed mode), or in balanced mode at one of the work-group's own two
// slots: 2j for the piece that continues a row begun by an earlier work-group, 2j+1 for the
// piece that begins a row which a later work-group continues.  A 16-byte record per
// work-group says where its range starts, so the merge finds a row's pieces without a search.
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
    // fp8 caches: probabilities are carried as 2^kPShift * p so that their fp8 halves stay
    // normal numbers down to p = 2^-13; numerator and denominator share the factor.
    constexpr float kPShift = FP8 ? 7.0f : 0.0f;
    // Keep the next item's Q rows in registers for a whole item?  Only where the register
    // file has room: contiguous caches spend more registers on per-lane offsets than paged
    // ones, the fp8 tile more than the bf16 one, 16 head rows more than 8.  Otherwise the rows
    // are fetched when the item starts, which costs that wavefront one exposed cache latency
    // behind its prefetched tiles.
    constexpr bool Q_AHEAD = FP8 ? (PAGED && GQ <= 2) : (PAGED || GQ <= 2);
    constexpr int kGroupStep = kWaves * TILE;             // token stride between a wave's tiles when
                                                          // the four wavefronts share an item
    constexpr int TRIP = kMaxGroup * kHeadDim + 2 * kMaxGroup;   // floats: O, then max, then sum
    static_assert(VR * RPI == TILE && KR == VR && KSTRIDE <= VSTRIDE, "tile geometry");
    __shared__ __attribute__((aligned(16))) unsigned char smem[kWaves * VBUF];
    __shared__ __attribute__((aligned(16))) float s_trip[kWaves * TRIP];   // end-of-item triples
    __shared__ int s_busy[kWaves];                        // 1 while s_trip[w] awaits the combine
    __shared__ int s_count;                               // wavefronts that finished the item
    __shared__ int s_cum[kMaxSplitBatch + 1];             // units before request r (split modes)
    __shared__ int s_len[kMaxSplitBatch];                 // seq_lens, capped (split modes)
    __shared__ float s_wgt[kWaves * kMaxGroup];           // combine weights of the four triples
    __shared__ int s_wsum[kWaves];

    LAMINA_TRACE_ONLY(
        __shared__ unsigned long long s_stamp[kWaves][kTraceStamps];
        const unsigned long long tr_enter = __builtin_amdgcn_s_memrealtime();
        unsigned long long tr_range = 0, tr_issued = 0, tr_data = 0, tr_tiles_end = 0, tr_first_item = 0;
        int tr_items = 0, tr_slots = 0, tr_iters = 0;)
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15;
    const int quad = lane >> 4;
    const int G = prm.G;
    const int R = prm.batch;
    const int Hkv = prm.Hkv;
    const int mode = prm.mode;
    const int unit = prm.unit;
    const int j = blockIdx.x;
    const int nwg = gridDim.x;
    const const_i32_ptr lens = (const_i32_ptr)prm.seq_lens;

    // Units of one row of a request with `len` tokens (split modes).  In balanced mode a row
    // weighs rc units more than its tokens: starting and finishing an item costs a wavefront
    // about as long as a 128-token unit, and shares that are equal in tokens alone leave the
    // work-groups that hold many short rows far behind the others.
    const int rc = (mode == kModeBalanced) ? prm.row_cost : 0;
    auto units_of = [&](int len) {
        const int n = max(1, (min(len, prm.len_cap) + unit - 1) / unit);
        return mode == kModeFixed ? min(prm.P, n) : n + rc;
    };
    unsigned char *vbuf = smem + w * VBUF;                // this wavefront's staging area
    // The lane number as a value the compiler cannot see through.  Code at item boundaries
    // derives its lane-dependent offsets from it, so that they are recomputed there instead of
    // being carried (and, with the register file full, spilled) across the tile loop: a spill
    // reload is a vector-memory access and would wait behind the two prefetched tiles.
    auto fresh_lane = [&]() {
        int l = lane;
        asm volatile("" : "+v"(l));
        return l;
    };

    if (tid < kWaves)
        s_busy[tid] = 0;
    if (tid == 0)
        s_count = 0;
    __syncthreads();

    // ---- this work-group's range of units --------------------------------------------------
    long long U;                                          // units in the call
    if (mode != kModeRows) {
        const int per = (R + kThreads - 1) / kThreads;
        const int b = tid * per;
        const int e = min(R, b + per);
        constexpr int kPer = kMaxSplitBatch / kThreads;   // requests per thread at most
        int un[kPer];                                     // their unit counts, read once
        int sum = 0;
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            un[k] = 0;
            if (b + k < e) {
                const int len = min(prm.seq_lens[b + k], prm.len_cap);
                s_len[b + k] = len;                       // the row walk reads lengths from here
                un[k] = units_of(len);
            }
            sum += un[k];
        }
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
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            if (b + k < e) {
                s_cum[b + k] = run;
                if (j == 0 && mode == kModeFixed)
                    prm.cum[b + k] = run;                 // the merge pass reads it back
            }
            run += un[k];
        }
        if (tid == 0) {
            s_cum[R] = tot;
            if (j == 0 && mode == kModeFixed)
                prm.cum[R] = tot;
        }
        __syncthreads();
        U = (long long)__builtin_amdgcn_readfirstlane(tot) * Hkv;
    } else {
        U = (long long)R * Hkv;
    }
    LAMINA_TRACE_ONLY(tr_range = __builtin_amdgcn_s_memrealtime();)
    // Workers: the work-groups, or (fixed partitions, enough of them) the wavefronts on their own.
    const bool wave_items = wave_items_rule(mode, (unsigned)U, (unsigned)nwg);
    const int worker = wave_items ? j * kWaves + w : j;
    const int nworkers = wave_items ? nwg * kWaves : nwg;
    const int step = wave_items ? TILE : kGroupStep;      // token stride between this wave's tiles
    const int step_log2 = wave_items ? (FP8 ? 6 : 5) : (FP8 ? 8 : 7);
    const int skew = share_skew(mode == kModeBalanced, (unsigned)U, (unsigned)nworkers);
    const int u0 = (int)share_begin((unsigned)U, nworkers, worker, skew);
    const int u1 = (int)share_begin((unsigned)U, nworkers, worker + 1, skew);
    if (u0 >= u1) {
        if (mode == kModeBalanced && tid == 0) {
            const i32x4 none = {-1, 0, 0, 0};             // no item here, so no row ends here
            *reinterpret_cast<i32x4 *>(prm.tails + 4 * j) = none;
        }
        LAMINA_TRACE_ONLY(if (lane == 0 && j * kWaves + w < kTraceWaves)
                              g_trace[(size_t)(j * kWaves + w) * kTraceWaveWords + 6] = 0;)
        return;
    }

    // Walking the stream: the next unit to hand out and the row it lies in (all wave-uniform).
    struct Walk {
        int u;                        // next unit
        int r, g;                     // its row
        int S, n;                     // the row's first unit and number of units
        int len;                      // seq_lens[r]
    };
    auto load_row = [&](Walk &s) {
        if (mode == kModeRows) {
            s.len = min(lens[s.r], prm.len_cap);
            s.n = 1;
            s.S = s.r * Hkv + s.g;
        } else {
            s.len = __builtin_amdgcn_readfirstlane(s_len[s.r]);
            const int c0 = __builtin_amdgcn_readfirstlane(s_cum[s.r]);
            const int c1 = __builtin_amdgcn_readfirstlane(s_cum[s.r + 1]);
            s.n = c1 - c0;
            s.S = Hkv * c0 + s.g * s.n;
        }
    };
    struct Piece {
        int r, g;
        int t0, t1;                   // token range
        int whole;                    // covers its whole row: result goes straight to out/lse
        int dest;                     // piece index in the workspace otherwise
    };
    // Hand out the part of the stream that starts at unit s.u (the caller has checked
    // s.u < u1) and say whether it is an item: the first rc units of a row stand for its fixed
    // cost and hold no tokens, so a part that ends inside them is nothing to do.
    auto next_piece = [&](Walk &s, Piece &p) {
        const int E = s.S + s.n;
        const int pe = (mode == kModeBalanced) ? min(E, u1) : s.u + 1;
        const int T0 = s.S + rc;                          // where the row's tokens start
        const int a = max(s.u, T0) - T0;                  // token units [a, b) of the row
        const int b = pe - T0;
        p.r = s.r;
        p.g = s.g;
        p.t0 = a * unit;
        p.t1 = (mode == kModeRows) ? s.len : min(s.len, b * unit);
        p.whole = (s.u <= T0) && (pe == E);
        // Balanced shares: a work-group holds at most one piece that continues a row begun in an
        // earlier share (its first item) and at most one that begins a row it does not finish
        // (its last item); they go to slots 2j and 2j + 1.
        p.dest = (mode == kModeBalanced) ? 2 * worker + (s.u <= T0 ? 1 : 0) : s.u;
        s.u = pe;
        if (pe == E) {
            if (++s.g == Hkv) {
                s.g = 0;
                ++s.r;
            }
            if (pe < u1)
                load_row(s);
        }
        return b > 0;
    };
    Walk start;
    start.u = u0;
    if (mode == kModeRows) {
        start.r = u0 / Hkv;
        start.g = u0 % Hkv;
    } else {
        int lo = 0, hi = R;                               // largest r with Hkv * cum[r] <= u0
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((long long)Hkv * s_cum[mid] <= u0)
                lo = mid;
            else
                hi = mid;
        }
        start.r = __builtin_amdgcn_readfirstlane(lo);
        const int c0 = __builtin_amdgcn_readfirstlane(s_cum[start.r]);
        const int c1 = __builtin_amdgcn_readfirstlane(s_cum[start.r + 1]);
        start.g = (u0 - Hkv * c0) / (c1 - c0);
    }
    load_row(start);
    // Wave-uniform description of the tiles one wavefront owns in one item.
    struct Desc {
        int slot;                     // ordinal of the item in this work-group; -1: none
        int r, g;
        int t0w;                      // first token of this wavefront's first tile
        int t1;                       // end of the item's token range
        int n_even;                   // tile slots this wavefront runs here (tiles rounded up to even)
        const unsigned char *kbase;
        const unsigned char *vbase;
        const int32_t *bt;            // the request's row of the block table (paged caches)
    };
    auto describe = [&](const Piece &p, int slot, Desc &d) {
        d.slot = slot;
        d.r = p.r;
        d.g = p.g;
        d.t0w = p.t0 + (wave_items ? 0 : w * TILE);
        d.t1 = p.t1;
        const int nt = (d.t0w < d.t1) ? (d.t1 - d.t0w + step - 1) >> step_log2 : 0;
        d.n_even = (nt + 1) & ~1;
        if (PAGED) {
            d.kbase = prm.k + (long long)p.g * prm.pool_stride_head_b;
            d.vbase = prm.v + (long long)p.g * prm.pool_stride_head_b;
            d.bt = prm.block_table + (size_t)p.r * prm.bt_stride;
        } else {
            const long long off =
                (long long)p.r * prm.stride_req_b + (long long)p.g * prm.stride_head_b;
            d.kbase = prm.k + off;
            d.vbase = prm.v + off;
            d.bt = nullptr;
        }
    };
    // Next item, from the look-ahead position on, in which this wavefront has at least one tile.
    Walk look = start;
    int look_slot = 0;
    auto find_next = [&](Desc &d) {
        d.slot = -1;
        while (look.u < u1) {
            Piece p;
            if (!next_piece(look, p))
                continue;
            Desc t;
            describe(p, look_slot++, t);
            if (t.n_even > 0) {
                d = t;
                return;
            }
        }
    };

    // Pool blocks of the 16-token pages of the tile starting at ts: lane `sub` (mod NSUB) of the
    // returned register holds the block of page ts/16 + sub.  It is a VECTOR load on purpose.
    // Scalar loads return out of order and share their wait counter with the LDS, so with one
    // in flight every LDS wait of the tile's arithmetic becomes a wait for the block table
    // too; a vector load instead queues in order with the K/V loads, and because the pages of
    // a tile slot are requested one whole generation of its register set ahead (just before
    // the K/V loads of the slot two earlier), they have always arrived by the time the data
    // consumed before their use has.
    // (The fp8 paged variants have no register to spare for it -- the compiler would spill the
    // prefetched Q rows around the tile loop -- and keep scalar loads, one refill ahead.)
    constexpr bool VPAGES = PAGED && !FP8;
    auto load_pages = [&](const int32_t *bt, int ts, int last) -> int {
        if (!VPAGES)
            return 0;
        const int tok = min(ts + (lane & (NSUB - 1)) * 16, last);
        return bt[tok >> 4];
    };
    auto pages_of = [&](int pv, int(&pg)[NSUB]) {
        if (VPAGES) {
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub)
                pg[sub] = __builtin_amdgcn_readlane(pv, sub);
        }
    };
    auto fetch_pages = [&](const int32_t *bt, int ts, int last, int(&pg)[NSUB]) {
        if (PAGED && !VPAGES) {
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub)
                pg[sub] = ((const_i32_ptr)bt)[min(ts + sub * 16, last) >> 4];
        }
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
    //
    // bf16 caches: four k-steps of 8 bf16 dims.  fp8 caches: the matrix cores multiply fp8 by
    // fp8, so Q is split per head into q * 2^a = hi + lo with both halves e4m3fn (exact, see
    // split_fp8x4; a puts the row's largest magnitude into [128, 256)), K needs no conversion
    // at all, and one 16x16x128 MFMA per half covers the whole head dimension: the lane holds
    // dims quad*32 .. quad*32+31 of its row, for Q and for K alike.
    bf16x8 qop[4];
    i32x8 q8hi, q8lo;
    float q_unscale = 1.0f;         // 2^-a of the head in this lane's column (fp8 caches)
    auto request_q = [&](int r, int g, u32x4(&raw)[GQ]) {
        const int lane = fresh_lane();
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
        const int lane = fresh_lane();
        const int col = lane & 15;
        const int quad = lane >> 4;
#pragma unroll
        for (int i = 0; i < GQ; ++i)
            *reinterpret_cast<u32x4 *>(vbuf + (i * 4 + (lane >> 4)) * 256 + (lane & 15) * 16) = raw[i];
        if (FP8) {
            float f[32];
            float amax = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                u32x4 t = {0u, 0u, 0u, 0u};
                if (col < GQ * 4)                         // rows at or above G hold zeros
                    t = *reinterpret_cast<const u32x4 *>(vbuf + col * 256 + quad * 64 + i * 16);
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    f[i * 8 + d * 2] = __builtin_bit_cast(float, t[d] << 16);
                    f[i * 8 + d * 2 + 1] = __builtin_bit_cast(float, t[d] & 0xffff0000u);
                    amax = fmaxf(amax, fmaxf(fabsf(f[i * 8 + d * 2]), fabsf(f[i * 8 + d * 2 + 1])));
                }
            }
            amax = quad_max(amax);
            const int e = (int)((__builtin_bit_cast(unsigned, amax) >> 23) & 255u);
            int a = (amax > 0.0f) ? 134 - e : 0;          // amax * 2^a in [128, 256)
            a = max(-100, min(100, a));
            const float up = __builtin_bit_cast(float, (unsigned)(127 + a) << 23);
            q_unscale = __builtin_bit_cast(float, (unsigned)(127 - a) << 23);
#pragma unroll
            for (int d = 0; d < 8; ++d) {
                int h, l;
                split_fp8x4(f[d * 4] * up, f[d * 4 + 1] * up, f[d * 4 + 2] * up, f[d * 4 + 3] * up, h, l);
                q8hi[d] = h;
                q8lo[d] = l;
            }
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                // The dims a lane holds in step s must be the dims its K operand holds there.
                const int chunk8 = s * 4 + quad;
                bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
                qop[s] = z;
                if (col < GQ * 4)                         // rows at or above G hold zeros
                    qop[s] = *reinterpret_cast<const bf16x8 *>(vbuf + col * 256 + chunk8 * 16);
            }
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
        // K rows -> LDS (pitch KSTRIDE) -> MFMA A-operand layout (row = token col; bf16: the
        // lane holds the 16-byte piece s*4 + quad of that row in k-step s; fp8: its 32-byte
        // piece quad, untouched -- the matrix cores take e4m3 as it is).  The staging area is
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
            if (FP8) {
                const unsigned char *krow = vbuf + (sub * 16 + col) * KSTRIDE + quad * 32;
                const u32x4 k0 = *reinterpret_cast<const u32x4 *>(krow);
                const u32x4 k1 = *reinterpret_cast<const u32x4 *>(krow + 16);
                i32x8 kop;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    kop[d] = (int)k0[d];
                    kop[4 + d] = (int)k1[d];
                }
                // e4m3 x e4m3, no block scales (scale operands 0)
                acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(kop, q8hi, acc, 0, 0, 0, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(kop, q8lo, acc, 0, 0, 0, 0, 0, 0);
            } else {
                const unsigned char *krow = vbuf + (sub * 16 + col) * KSTRIDE + quad * 16;
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
        tmax = quad_max(tmax);
        const float m_new = fmaxf(m_run, tmax);           // finite from the first tile on
        const float alpha = fast_exp2(m_run - m_new);     // exp2(-inf) = 0 on the first tile
        m_run = m_new;
        float psum = 0.0f;
        bf16x8 p_hi[NPAIR], p_lo[NPAIR];                  // bf16 caches: p = hi + lo, both bf16
        long p8_hi[NPAIR], p8_lo[NPAIR];                  // fp8 caches: 2^7 p = hi + lo, both e4m3
        float pj[NSUB * 4];
#pragma unroll
        for (int jj = 0; jj < NSUB * 4; ++jj) {
            pj[jj] = fast_exp2(x[jj] - (m_new - kPShift));
            psum += pj[jj];
        }
        if (FP8) {
#pragma unroll
            for (int pp = 0; pp < NPAIR; ++pp) {
                int h0, l0, h1, l1;
                split_fp8x4(pj[pp * 8], pj[pp * 8 + 1], pj[pp * 8 + 2], pj[pp * 8 + 3], h0, l0);
                split_fp8x4(pj[pp * 8 + 4], pj[pp * 8 + 5], pj[pp * 8 + 6], pj[pp * 8 + 7], h1, l1);
                i32x2 h = {h0, h1}, l = {l0, l1};
                p8_hi[pp] = __builtin_bit_cast(long, h);
                p8_lo[pp] = __builtin_bit_cast(long, l);
            }
        } else {
#pragma unroll
            for (int jj = 0; jj < NSUB * 4; ++jj) {
                // p = hi + lo with both halves bf16: keeps ~16 significant bits through the MFMA
                const __bf16 h = static_cast<__bf16>(pj[jj]);
                p_hi[jj >> 3][jj & 7] = h;
                p_lo[jj >> 3][jj & 7] = static_cast<__bf16>(pj[jj] - static_cast<float>(h));
            }
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
                if (FP8) {
                    // 8 rows x 16 byte-columns per 16-lane block; lane supplies row col/2.
                    // The transposed bytes are the MFMA operand as they are.
                    const int rr = col >> 1;
                    const int trow =
                        pp * 32 + ((rr < 4) ? (quad * 4 + rr) : (16 + quad * 4 + rr - 4));
                    const unsigned char *a = vbuf + trow * VSTRIDE + db * 16 + (col & 1) * 8;
                    const i32x2 raw = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                        (i32x2 __attribute__((address_space(3))) *)(a));
                    const long vop = __builtin_bit_cast(long, raw);
                    o_acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(vop, p8_hi[pp],
                                                                          o_acc[db], 0, 0, 0);
                    o_acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(vop, p8_lo[pp],
                                                                          o_acc[db], 0, 0, 0);
                } else {
                    // 4 rows x 16 columns per 16-lane block; lane supplies row col/4, 4 columns
                    const unsigned char *a = vbuf + (pp * 32 + quad * 4 + (col >> 2)) * VSTRIDE +
                                             db * 32 + (col & 3) * 8;
                    const s16x4 ra = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3))) *)(a));
                    const s16x4 rb = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3))) *)(a + 16 * VSTRIDE));
                    const bf16x8 vop = join_bf16x4(__builtin_bit_cast(bf16x4, ra),
                                                   __builtin_bit_cast(bf16x4, rb));
                    o_acc[db] =
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, p_hi[pp], o_acc[db], 0, 0, 0);
                    o_acc[db] =
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, p_lo[pp], o_acc[db], 0, 0, 0);
                }
            }
        }
    };

    // End of an item for ONE wavefront.  Nobody waits at a barrier: the wavefront parks its
    // (output, max, denominator) triple in LDS, counts itself in, and moves on to its next
    // item; whichever of the four arrives last combines the triples (same identity as the
    // cross-partition merge) and writes the item's result.  A wavefront can be at most one
    // item ahead: it may not overwrite its parked triple before that item was combined.
    // End of an item a wavefront worked through alone: normalise and store, straight from the
    // accumulator layout (lane = head col; 4 consecutive dims per 16-byte store).
    auto finalize_alone = [&](const Piece &id) {
        const int lane = fresh_lane();
        const int col = lane & 15;
        const int quad = lane >> 4;
        l_run = quad_sum(l_run);
        const bool empty = !(l_run > 0.0f);               // a request with no tokens at all
        float vs = 1.0f;
        if (FP8)
            vs = ((const __attribute__((address_space(4))) float *)prm.v_scale)[(size_t)id.r * Hkv + id.g];
        const float inv = empty ? 0.0f : vs * __builtin_amdgcn_rcpf(l_run);
        const float lse_nat =
            empty ? -INFINITY : (m_run + __builtin_amdgcn_logf(l_run) - kPShift) * kLn2;
        if (col < G) {
            const size_t row = (size_t)id.r * prm.Hq + id.g * G + col;
            if (id.whole) {
                if (quad == 0 && prm.lse)
                    prm.lse[row] = lse_nat;
#pragma unroll
                for (int db = 0; db < 8; ++db) {
                    const f32x4 o = o_acc[db] * inv;
                    const size_t at = row * kHeadDim + db * 16 + quad * 4;
                    if (prm.out_is_bf16) {
                        u32x2 pk;
                        pk[0] = (unsigned)bf16_bits(o[0]) | ((unsigned)bf16_bits(o[1]) << 16);
                        pk[1] = (unsigned)bf16_bits(o[2]) | ((unsigned)bf16_bits(o[3]) << 16);
                        *reinterpret_cast<u32x2 *>(static_cast<unsigned short *>(prm.out) + at) = pk;
                    } else {
                        *reinterpret_cast<f32x4 *>(static_cast<float *>(prm.out) + at) = o;
                    }
                }
            } else {
                const size_t slot = (size_t)id.dest * G + col;
                if (quad == 0)
                    prm.part_lse[slot] = lse_nat;
#pragma unroll
                for (int db = 0; db < 8; ++db)
                    *reinterpret_cast<f32x4 *>(prm.part_out + slot * kHeadDim + db * 16 + quad * 4) =
                        o_acc[db] * inv;
            }
        }
        m_run = -INFINITY;
        l_run = 0.0f;
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            f32x4 z = {0.f, 0.f, 0.f, 0.f};
            o_acc[db] = z;
        }
    };

    auto finalize = [&](const Piece &id) {
        if (wave_items) {
            finalize_alone(id);
            return;
        }
        const int lane = fresh_lane();
        const int col = lane & 15;
        const int quad = lane >> 4;
        l_run = quad_sum(l_run);
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
        const int r = id.r, g = id.g;
        const bool whole = id.whole != 0;                 // the row has no other piece
        float vs = 1.0f;
        if (FP8)
            vs = ((const __attribute__((address_space(4))) float *)prm.v_scale)[(size_t)r * Hkv + g];
        {
            // weights: lane = (head col, wavefront quad)
            const float mw = s_trip[quad * TRIP + kMaxGroup * kHeadDim + col];
            const float lw = s_trip[quad * TRIP + kMaxGroup * kHeadDim + kMaxGroup + col];
            const float M = quad_max(mw);
            const float e = (mw == -INFINITY) ? 0.0f : fast_exp2(mw - M);   // idle wavefront
            float L = e * lw;
            L = quad_sum(L);
            const bool empty = !(L > 0.0f);               // a request with no tokens at all
            s_wgt[quad * kMaxGroup + col] = empty ? 0.0f : e * vs * __builtin_amdgcn_rcpf(L);
            if (quad == 0 && col < G) {
                const float lse_nat =
                    empty ? -INFINITY : (M + __builtin_amdgcn_logf(L) - kPShift) * kLn2;
                const size_t row = (size_t)r * prm.Hq + g * G + col;
                if (whole) {
                    if (prm.lse)
                        prm.lse[row] = lse_nat;
                } else {
                    prm.part_lse[(size_t)id.dest * G + col] = lse_nat;
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
                    *reinterpret_cast<f32x4 *>(prm.part_out + ((size_t)id.dest * G + h) * kHeadDim + d4) = o;
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
    find_next(nxt);
    int pvA = 0, pvB = 0;           // pages of the next refill of set A / set B (paged caches)
    if (nxt.slot >= 0) {
        // prologue: the Q rows of this wavefront's first item and its first two tile slots; the
        // pages of slots 2 and 3 as if they lay in the same item (put right at the item's
        // start if they do not).  Q goes first: loads return in order, so the first item can
        // start on its first tile as soon as that has arrived, without waiting for the second
        // (a call of 20 requests x 1024 tokens, all start-up: 20.0 -> 18.6 us).
        if (Q_AHEAD)
            request_q(nxt.r, nxt.g, qn);
        const int pv0 = load_pages(nxt.bt, nxt.t0w, nxt.t1 - 1);
        const int pv1 = load_pages(nxt.bt, nxt.t0w + step, nxt.t1 - 1);
        pvA = load_pages(nxt.bt, nxt.t0w + 2 * step, nxt.t1 - 1);
        pvB = load_pages(nxt.bt, nxt.t0w + 3 * step, nxt.t1 - 1);
        pages_of(pv0, pg);
        fetch_pages(nxt.bt, nxt.t0w, nxt.t1 - 1, pg);
        issue_loads(nxt.kbase, nxt.vbase, nxt.t0w, nxt.t1 - 1, pg, kA, vA);
        __builtin_amdgcn_sched_barrier(0);                // A must be the older set
        pages_of(pv1, pg);
        fetch_pages(nxt.bt, nxt.t0w + step, nxt.t1 - 1, pg);
        issue_loads(nxt.kbase, nxt.vbase, nxt.t0w + step, nxt.t1 - 1, pg, kB, vB);
        __builtin_amdgcn_sched_barrier(0);
        cn = score_scale(nxt.r, nxt.g);
        LAMINA_TRACE_ONLY(tr_issued = __builtin_amdgcn_s_memrealtime();)
    }
    if (mode == kModeBalanced && tid == 0) {
        // Does a row that began in an earlier share end in this one?  Then this work-group's
        // first item is the row's last piece, and the merge pass combines the row from here:
        // the pieces lie in slot 2a + 1 (a = the share holding the row's first tokens) and in
        // slots 2k for the shares k = a + 1 .. j.  One record per work-group, every launch.
        const int T0 = start.S + rc;
        const bool ends_here = u0 > T0 && start.S + start.n <= u1;
        const i32x4 rec = {ends_here ? 1 : -1, start.r, start.g,
                           share_owner((unsigned)U, (unsigned)nworkers, (unsigned)T0, skew)};
        *reinterpret_cast<i32x4 *>(prm.tails + 4 * j) = rec;
    }
    Walk at = start;                // the item every wavefront of the work-group is on
    for (int slot = 0; at.u < u1;) {
        Piece id;
        if (!next_piece(at, id))
            continue;
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
            if (FP8)
                c_log2 *= q_unscale;                      // per head: undo the 2^a of the Q split
            find_next(nxt);
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
            const int32_t *n_bt = more ? nxt.bt : cur.bt;
            const int n_t0w = more ? nxt.t0w : cur.t1;
            const int n_last = (more ? nxt.t1 : cur.t1) - 1;
            const int c_last = cur.t1 - 1;
            const int n_even = cur.n_even;
            // refill number idx (2, 3, ...) of this item -> its addressing, by scalar selects
            auto target = [&](int idx, const unsigned char *&kb, const unsigned char *&vb,
                              const int32_t *&bt, int &ts, int &last) {
                const bool in_item = idx < n_even;
                kb = in_item ? cur.kbase : n_kbase;
                vb = in_item ? cur.vbase : n_vbase;
                bt = in_item ? cur.bt : n_bt;
                ts = in_item ? cur.t0w + idx * step : n_t0w + (idx - n_even) * step;
                last = in_item ? c_last : n_last;
            };
            const unsigned char *kb, *vb, *kb2, *vb2;
            const int32_t *bt, *bt2;
            int rts, rlast, rts2, rlast2;
            // pvA / pvB hold the pages of refills 2 and 3 as seen from the item before (or the
            // prologue), which took them to lie in this item.  With only two tile slots here
            // they lie in the next item, known only now: fetch them again.
            if (VPAGES && n_even == 2) {
                target(2, kb, vb, bt, rts, rlast);
                pvA = load_pages(bt, rts, rlast);
                target(3, kb, vb, bt, rts, rlast);
                pvB = load_pages(bt, rts, rlast);
            }
            target(2, kb, vb, bt, rts, rlast);
            fetch_pages(bt, rts, rlast, pg);
            int ts = cur.t0w;
            for (int k = 0; k < n_even; k += 2) {
                LAMINA_TRACE_ONLY({
                    // iterations 0..7 each, then every fourth
                    const int at_ = tr_iters < 8 ? tr_iters : 8 + ((tr_iters - 8) >> 2);
                    if ((tr_iters < 8 || ((tr_iters - 8) & 3) == 0) && at_ < kTraceStamps && lane == 0)
                        s_stamp[w][at_] = __builtin_amdgcn_s_memrealtime();
                    if (tr_iters == 1)
                        tr_data = s_stamp[w][1];          // first pair of tiles consumed
                    ++tr_iters;
                })
                consume(kA, vA, sc);
                __builtin_amdgcn_sched_barrier(0);
                target(k + 2, kb, vb, bt, rts, rlast);
                pages_of(pvA, pg);
                if (VPAGES) {
                    target(k + 4, kb2, vb2, bt2, rts2, rlast2);
                    pvA = load_pages(bt2, rts2, rlast2);  // older than the loads it rides with
                }
                __builtin_amdgcn_sched_barrier(0);
                issue_loads(kb, vb, rts, rlast, pg, kA, vA);
                target(k + 3, kb, vb, bt, rts, rlast);
                fetch_pages(bt, rts, rlast, pg);
                __builtin_amdgcn_sched_barrier(0);
                finish(ts, sc);
                __builtin_amdgcn_sched_barrier(0);
                consume(kB, vB, sc);
                __builtin_amdgcn_sched_barrier(0);
                pages_of(pvB, pg);
                if (VPAGES) {
                    target(k + 5, kb2, vb2, bt2, rts2, rlast2);
                    pvB = load_pages(bt2, rts2, rlast2);
                }
                __builtin_amdgcn_sched_barrier(0);
                issue_loads(kb, vb, rts, rlast, pg, kB, vB);
                target(k + 4, kb, vb, bt, rts, rlast);
                fetch_pages(bt, rts, rlast, pg);
                __builtin_amdgcn_sched_barrier(0);
                finish(ts + step, sc);
                __builtin_amdgcn_sched_barrier(0);
                ts += 2 * step;
            }
            LAMINA_TRACE_ONLY(++tr_items; tr_slots += n_even; tr_tiles_end = __builtin_amdgcn_s_memrealtime();)
        }
        finalize(id);
        LAMINA_TRACE_ONLY(if (tr_first_item == 0) tr_first_item = __builtin_amdgcn_s_memrealtime();)
        ++slot;
    }
    LAMINA_TRACE_ONLY(
        if (lane == 0 && j * kWaves + w < kTraceWaves) {
            unsigned long long *o = g_trace + (size_t)(j * kWaves + w) * kTraceWaveWords;
            o[0] = tr_enter;
            o[1] = tr_range;
            o[2] = tr_issued;
            o[3] = tr_data;
            o[4] = tr_tiles_end;
            o[6] = tr_items;
            o[7] = tr_slots;
            o[8] = tr_first_item;
            o[9] = tr_iters;
            for (int q = 0; q < kTraceStamps && (q < 8 ? q : 8 + (q - 8) * 4) < tr_iters; ++q)
                o[16 + q] = s_stamp[w][q];
            o[5] = __builtin_amdgcn_s_memrealtime();      // exit
        })
}

// -------------------------------------------------------------------------------------------
// Cross-partition merge (Sec. 4.2.2 identity, any number of parts, log-sum-exp form):
//   lse = ln sum_p e^{lse_p},  out = sum_p e^{lse_p - lse} out_p.
// This kernel serves fixed partitions: one wavefront per (request, query head) row, four rows
// per work-group; the row's pieces are its partitions, found from the unit prefix sums the main
// pass left in the workspace; a row with a single partition was already written to out/lse by
// the main pass.  (Balanced shares have their own pass, merge_balanced_kernel below.)
// Lane p first holds piece p's weight (the log-sum-exp reduction is two wave reductions);
// then the two half-waves take alternate pieces, each lane four output columns, sixteen
// pieces' loads in flight per step.
// -------------------------------------------------------------------------------------------
constexpr int kMergeRowsPerBlock = 4;

__global__ __launch_bounds__(64 * kMergeRowsPerBlock) void merge_partials_kernel(const MergeParams prm)
{
    LAMINA_TRACE_ONLY(
        struct Stamp {
            unsigned long long t0;
            __device__ ~Stamp()
            {
                if ((threadIdx.x & 63) == 0 && blockIdx.x < kTraceMergeGroups) {
                    unsigned long long *o = g_trace + (size_t)kTraceWaves * kTraceWaveWords +
                                            (size_t)blockIdx.x * kTraceMergeWords;
                    o[0] = t0;
                    o[1] = __builtin_amdgcn_s_memrealtime();
                }
            }
        } stamp{__builtin_amdgcn_s_memrealtime()};)
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * kMergeRowsPerBlock + (threadIdx.x >> 6);   // r * Hq + h
    if (row >= prm.rows)
        return;
    const int r = row / prm.Hq;
    const int hq = row - r * prm.Hq;
    const int g = hq / prm.G;
    const int hl = hq - g * prm.G;
    const int c0 = prm.cum[r];
    const int n = prm.cum[r + 1] - c0;
    const long long first = (long long)prm.Hkv * c0 + (long long)g * n;   // the row's first unit
    const int np = n;                                                     // one piece per partition
    if (np == 1)
        return;                                           // the main pass wrote this row itself
    const size_t pstride = (size_t)prm.G;
    const float *pl = prm.part_lse + (size_t)first * prm.G + hl;
    const float *po = prm.part_out + ((size_t)first * prm.G + hl) * kHeadDim;
    float M = -INFINITY;
    for (int p0 = 0; p0 < np; p0 += 64) {
        const float v = (p0 + lane < np) ? pl[(size_t)(p0 + lane) * pstride] : -INFINITY;
        M = fmaxf(M, v);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        M = fmaxf(M, __shfl_xor(M, off));
    const int half = lane >> 5;
    const int c4 = (lane & 31) * 4;
    float W = 0.0f;
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    for (int p0 = 0; p0 < np; p0 += 64) {
        const float e = (p0 + lane < np) ? __expf(pl[(size_t)(p0 + lane) * pstride] - M) : 0.0f;
        W += e;
        const int cnt = min(64, np - p0);
        // Eight pieces per half-wave at a time, all loads issued before the first use.  (A
        // loop with a run-time trip count is not unrolled around the cross-lane read, and the
        // loads would go out one round trip after the other.)  Pieces beyond cnt re-read the
        // last one with weight zero.
        for (int i0 = 0; i0 < (cnt + 1) / 2; i0 += 8) {
            f32x4 t[8];
            float wgt[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int p = 2 * (i0 + k) + half;
                const int pc = min(p, cnt - 1);
                wgt[k] = __shfl(e, pc);
                wgt[k] = (p < cnt) ? wgt[k] : 0.0f;
                t[k] = *reinterpret_cast<const f32x4 *>(
                    po + (size_t)(p0 + pc) * pstride * kHeadDim + c4);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k)
                o += wgt[k] * t[k];
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        W += __shfl_xor(W, off);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        o[i] += __shfl_xor(o[i], 32);
    const float inv = 1.0f / W;
    if (half == 0) {
        const size_t at = (size_t)row * kHeadDim + c4;
        if (prm.out_is_bf16) {
            u32x2 pk;
            pk[0] = (unsigned)bf16_bits(o[0] * inv) | ((unsigned)bf16_bits(o[1] * inv) << 16);
            pk[1] = (unsigned)bf16_bits(o[2] * inv) | ((unsigned)bf16_bits(o[3] * inv) << 16);
            *reinterpret_cast<u32x2 *>(static_cast<unsigned short *>(prm.out) + at) = pk;
        } else {
            *reinterpret_cast<f32x4 *>(static_cast<float *>(prm.out) + at) = o * inv;
        }
    }
    if (lane == 0 && prm.lse)
        prm.lse[row] = M + logf(W);
}

// -------------------------------------------------------------------------------------------
// The same combination for balanced shares.  Work-group j of this pass belongs to work-group j
// of the main pass: if a row that began in an earlier share ended in share j, the main pass
// left a record (row, first share a) and the row's pieces lie in slot 2a + 1 and in slots 2k,
// k = a + 1 .. j.  Nearly every cut row has exactly two pieces (a = j - 1), so the two slots
// that case needs are requested together with the record, before it is known whether they
// will be used: the common case costs one memory round trip, not three (record, weights,
// outputs one after the other), and this launch is pure latency on the call's critical path.
// One wavefront per head of the group (the work-group has G of them), so no wavefront works
// through heads one after the other; within a wavefront the two half-waves each hold one
// piece, every lane four output columns.
// -------------------------------------------------------------------------------------------
struct BalancedMergeParams {
    const float *part_out;             // [slot][G][128]
    const float *part_lse;             // [slot][G]
    const int *tails;                  // [work-group][4]: flag (1 / -1), request, kv head, first share
    void *out;
    float *lse;
    int Hq, G;
    int out_is_bf16;
};

__device__ __forceinline__ void store_merged_row(const BalancedMergeParams &prm, size_t row, int c4,
                                                 f32x4 o)
{
    const size_t at = row * kHeadDim + c4;
    if (prm.out_is_bf16) {
        u32x2 pk;
        pk[0] = (unsigned)bf16_bits(o[0]) | ((unsigned)bf16_bits(o[1]) << 16);
        pk[1] = (unsigned)bf16_bits(o[2]) | ((unsigned)bf16_bits(o[3]) << 16);
        *reinterpret_cast<u32x2 *>(static_cast<unsigned short *>(prm.out) + at) = pk;
    } else {
        *reinterpret_cast<f32x4 *>(static_cast<float *>(prm.out) + at) = o;
    }
}

__global__ __launch_bounds__(64 * kMaxGroup) void merge_balanced_kernel(const BalancedMergeParams prm)
{
    LAMINA_TRACE_ONLY(
        struct Stamp {
            unsigned long long t0;
            __device__ ~Stamp()
            {
                if ((threadIdx.x & 63) == 0 && blockIdx.x < kTraceMergeGroups) {
                    unsigned long long *o = g_trace + (size_t)kTraceWaves * kTraceWaveWords +
                                            (size_t)blockIdx.x * kTraceMergeWords;
                    o[0] = t0;
                    o[1] = __builtin_amdgcn_s_memrealtime();
                }
            }
        } stamp{__builtin_amdgcn_s_memrealtime()};)
    const int j = blockIdx.x + 1;                         // share 0 cannot hold the end of an earlier row
    const int lane = threadIdx.x & 63;
    const int hl = threadIdx.x >> 6;                      // one wavefront per head of the group
    const int half = lane >> 5;
    const int c4 = (lane & 31) * 4;
    const int G = prm.G;
    const i32x4 rec = *reinterpret_cast<const i32x4 *>(prm.tails + 4 * j);
    // the two-piece case, requested before the record is known: the tail piece (slot 2j) in
    // the lower half-wave, the head piece of the share before (slot 2j - 1) in the upper one
    const size_t slot2 = (size_t)(2 * j - half);
    const f32x4 t2 = *reinterpret_cast<const f32x4 *>(prm.part_out + (slot2 * G + hl) * kHeadDim + c4);
    const float l2 = prm.part_lse[slot2 * G + hl];
    if (rec[0] < 0)
        return;                                           // no row ends in this share
    const int r = rec[1], g = rec[2], a = rec[3];
    const size_t row = (size_t)r * prm.Hq + g * G + hl;
    if (a == j - 1) {
        const float lo = __shfl_xor(l2, 32);
        const float M = fmaxf(l2, lo);
        const float w = __expf(l2 - M);
        const float W = w + __expf(lo - M);
        f32x4 o = w * t2;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            o[c] += __shfl_xor(o[c], 32);
        if (half == 0)
            store_merged_row(prm, row, c4, o * (1.0f / W));
        if (lane == 0 && prm.lse)
            prm.lse[row] = M + logf(W);
        return;
    }
    // a row spread over three or more shares: piece p of it (p = 0 .. np - 1) lies in slot
    // 2a + 1 for p = 0 and in slot 2 (a + p) otherwise.  The weights (lane p holds piece p's)
    // and the first sixteen pieces' outputs are requested together: one more round trip.
    const int np = j - a + 1;
    auto slot_of = [&](int p) { return (size_t)(p == 0 ? 2 * a + 1 : 2 * (a + p)); };
    const float *pl = prm.part_lse + hl;
    const float *po = prm.part_out + (size_t)hl * kHeadDim + c4;
    float W = 0.0f, M = -INFINITY;
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    for (int p0 = 0; p0 < np; p0 += 64) {
        const int cnt = min(64, np - p0);
        const float l = (lane < cnt) ? pl[slot_of(p0 + lane) * G] : -INFINITY;
        f32x4 t[8];
#pragma unroll
        for (int k = 0; k < 8; ++k)                       // pieces beyond cnt re-read the last one
            t[k] = *reinterpret_cast<const f32x4 *>(
                po + slot_of(p0 + min(2 * k + half, cnt - 1)) * G * kHeadDim);
        float Mc = l;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1)
            Mc = fmaxf(Mc, __shfl_xor(Mc, off));
        const float Mn = fmaxf(M, Mc);                    // running maximum over chunks of 64 pieces
        const float rescale = __expf(M - Mn);             // 0 for the first chunk
        M = Mn;
        const float e = (lane < cnt) ? __expf(l - M) : 0.0f;
        W = W * rescale + e;
        o *= rescale;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int p = 2 * k + half;
            const float wgt = __shfl(e, min(p, cnt - 1));
            o += ((p < cnt) ? wgt : 0.0f) * t[k];
        }
        for (int i0 = 8; i0 < (cnt + 1) / 2; i0 += 8) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int p = 2 * (i0 + k) + half;
                t[k] = *reinterpret_cast<const f32x4 *>(
                    po + slot_of(p0 + min(p, cnt - 1)) * G * kHeadDim);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int p = 2 * (i0 + k) + half;
                const float wgt = __shfl(e, min(p, cnt - 1));
                o += ((p < cnt) ? wgt : 0.0f) * t[k];
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        W += __shfl_xor(W, off);
#pragma unroll
    for (int c = 0; c < 4; ++c)
        o[c] += __shfl_xor(o[c], 32);
    if (half == 0)
        store_merged_row(prm, row, c4, o * (1.0f / W));
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
    int pos_cap;                       // append: positions at or beyond this are skipped
    int fp8, paged, out_is_bf16;
    float scale;
};

__device__ __forceinline__ float bf16_bits_to_float(unsigned short b)
{
    return __builtin_bit_cast(float, (unsigned)b << 16);
}

// x -> the byte an fp8 cache holds for it: the quotient x / scale formed in fp32 (IEEE division,
// correctly rounded -- not a multiplication by a rounded reciprocal, which can land on the other
// side of an e4m3 tie), clamped to +-448, then rounded to nearest even on the e4m3fn grid.
__device__ __forceinline__ unsigned char quantise_e4m3fn(float x, float scale)
{
    const float y = fminf(fmaxf(x / scale, -448.0f), 448.0f);
    return (unsigned char)(__builtin_amdgcn_cvt_pk_fp8_f32(y, 0.0f, 0, false) & 0xFF);
}

__device__ __forceinline__ float dequantise_e4m3fn(unsigned char b, float scale)
{
    const bf16x2 v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)b, 1.0f, false);
    return static_cast<float>(v[0]) * scale;
}

// Write the new token's K and V rows of one (request, kv head) into the cache: lane i moves
// elements 2i and 2i+1 (kk, vv: two bf16 each).  Skips positions outside the cache.
__device__ __forceinline__ void append_row(const NewTokenParams &prm, int r, int g, int lane,
                                           unsigned kk, unsigned vv)
{
    const int row = r * prm.Hkv + g;
    const int pos = prm.positions[r];
    if (pos < 0 || pos >= prm.pos_cap)
        return;
    const int esz = prm.fp8 ? 1 : 2;
    long long off;
    if (prm.paged) {
        const long long blk = prm.block_table[(size_t)r * prm.bt_stride + (pos >> 4)];
        if (blk < 0)
            return;                                       // no block assigned: nothing to write to
        off = blk * prm.pool_stride_block_b + (long long)g * prm.pool_stride_head_b +
              (long long)(pos & 15) * kHeadDim * esz;
    } else {
        off = (long long)r * prm.stride_req_b + (long long)g * prm.stride_head_b +
              (long long)pos * prm.stride_tok_b;
    }
    if (!prm.fp8) {
        reinterpret_cast<unsigned *>(prm.k_cache + off)[lane] = kk;
        reinterpret_cast<unsigned *>(prm.v_cache + off)[lane] = vv;
    } else {
        const float ks = prm.k_scale[row];
        const float vs = prm.v_scale[row];
        const unsigned short kq =
            (unsigned short)quantise_e4m3fn(bf16_bits_to_float(kk & 0xFFFF), ks) |
            ((unsigned short)quantise_e4m3fn(bf16_bits_to_float(kk >> 16), ks) << 8);
        const unsigned short vq =
            (unsigned short)quantise_e4m3fn(bf16_bits_to_float(vv & 0xFFFF), vs) |
            ((unsigned short)quantise_e4m3fn(bf16_bits_to_float(vv >> 16), vs) << 8);
        reinterpret_cast<unsigned short *>(prm.k_cache + off)[lane] = kq;
        reinterpret_cast<unsigned short *>(prm.v_cache + off)[lane] = vq;
    }
}

// One wavefront per (request, kv head).
__global__ __launch_bounds__(256) void append_kv_kernel(const NewTokenParams prm)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);   // r * Hkv + g
    if (row >= prm.rows)
        return;
    const unsigned kk = reinterpret_cast<const unsigned *>(prm.k_new)[(size_t)row * 64 + lane];
    const unsigned vv = reinterpret_cast<const unsigned *>(prm.v_new)[(size_t)row * 64 + lane];
    append_row(prm, row / prm.Hkv, row % prm.Hkv, lane, kk, vv);
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
    // fold and append in one launch: the wavefront of a group's first head also moves the rows
    // it has just read into the cache
    if (prm.k_cache && (row % prm.Hq) % prm.G == 0)
        append_row(prm, r, g, lane, kk, vv);
    float k0 = bf16_bits_to_float(kk & 0xFFFF), k1 = bf16_bits_to_float(kk >> 16);
    float v0 = bf16_bits_to_float(vv & 0xFFFF), v1 = bf16_bits_to_float(vv >> 16);
    if (prm.fp8) {
        const float ks = prm.k_scale[kvrow], vs = prm.v_scale[kvrow];
        k0 = dequantise_e4m3fn(quantise_e4m3fn(k0, ks), ks);
        k1 = dequantise_e4m3fn(quantise_e4m3fn(k1, ks), ks);
        v0 = dequantise_e4m3fn(quantise_e4m3fn(v0, vs), vs);
        v1 = dequantise_e4m3fn(quantise_e4m3fn(v1, vs), vs);
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
    int mode;                    // kModeRows / kModeFixed / kModeBalanced
    int parts;                   // kModeFixed: partitions per row
    int unit;                    // tokens per unit (split modes), else 0
    long long max_pieces;        // partial results the workspace holds
    int row_cost;                // balanced mode: units a row weighs beyond its tokens
    float scale;
    float *workspace;            // part_out, part_lse, unit prefix sums; nullptr in rows mode
    size_t workspace_bytes;
    int resident_wgs;            // two work-groups per compute unit (see grid_for)
    char err[256];
};

namespace {

thread_local char g_create_err[256] = "";

int round_up(int x, int m) { return (x + m - 1) / m * m; }

struct Plan {
    int mode;
    int parts;
    int unit;
};

// Upper bound on the persistent grid (two work-groups per compute unit, capped), so that the
// workspace size does not depend on the device.
constexpr int kMaxGrid = 1024;

// Balanced mode: what a row weighs beyond its tokens when the shares are cut, in units
// (measured with 0..3: one unit is best -- workload 3: 65.4 / 67.6 / 66.9 / 66.5 % of peak).
constexpr int kRowCostUnits = 1;

// Partitioning.  num_splits == 1 never cuts a row; num_splits == N > 1 cuts every row into
// partitions of ceil(max_seq_len / N) tokens (rounded up to a multiple of 256).  Otherwise
// (0) rows are not cut when that cannot pay for the partial results and the merge launch:
// contexts up to 512 tokens; contexts up to 1024 unless the batch is tiny (one work-group
// streams such a row in ~15 us; with at most 32 rows the second launch is still the cheaper:
// 8 rows of 1024 tokens take 14.8 us uncut, 12.6 us balanced); batches that hold a row per
// quarter (contexts up to 2048) or per third (up to 4096) of the work-groups that can be
// resident (measured, us uncut / balanced: 128 rows x 2048 tokens 27.7 / 32.3, 64 rows 25.5 /
// 22.3; 160 rows x 4096 tokens 56.9 / 58.9, 128 rows 49.7 / 48.3) -- nor for batches beyond
// what the prefix sum in LDS holds; everything else runs balanced: every work-group streams
// the same share of the call's tokens.
Plan make_plan(const lamina_attn_config &c)
{
    Plan pl;
    pl.parts = 1;
    pl.unit = 0;
    const long long pairs = (long long)c.max_batch * c.num_kv_heads;
    if (c.num_splits == 1 ||
        (c.num_splits == 0 && (c.max_batch > kMaxSplitBatch || c.max_seq_len <= 512 ||
                               (c.max_seq_len <= 1024 && pairs > 32) ||
                               (c.max_seq_len <= 2048 && pairs >= 128) ||
                               (c.max_seq_len <= 4096 && pairs >= 160)))) {
        pl.mode = kModeRows;
    } else if (c.num_splits > 1) {
        pl.mode = kModeFixed;
        pl.parts = c.num_splits;
        pl.unit = round_up((c.max_seq_len + c.num_splits - 1) / c.num_splits, kChunkAlign);
    } else {
        pl.mode = kModeBalanced;
        pl.unit = c.kv_dtype == LAMINA_FP8_E4M3 ? 256 : 128;   // four wavefronts x one tile
    }
    return pl;
}

// Units per row at most, and partial results the workspace must hold.
long long max_units_per_row(const lamina_attn_config &c, const Plan &pl)
{
    if (pl.mode == kModeRows)
        return 1;
    if (pl.mode == kModeFixed)
        return pl.parts;
    return ((long long)c.max_seq_len + pl.unit - 1) / pl.unit + kRowCostUnits;
}

long long max_pieces_for(const lamina_attn_config &c, const Plan &pl)
{
    const long long rows = (long long)c.max_batch * c.num_kv_heads;
    if (pl.mode == kModeRows)
        return 0;
    if (pl.mode == kModeFixed)
        return rows * pl.parts;                           // piece index = unit number
    return 2LL * kMaxGrid;                                // two slots per work-group
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
    if (c->num_splits > 1 && c->max_batch > kMaxSplitBatch)
        return "a partitioned handle supports max_batch up to 1024";
    {
        const Plan pl = make_plan(*c);
        if ((long long)c->max_batch * c->num_kv_heads * max_units_per_row(*c, pl) > (1LL << 30))
            return "max_batch * num_kv_heads * partitions per row above 2^30";
    }
    *code = LAMINA_OK;
    return nullptr;
}

size_t workspace_bytes_for(const lamina_attn_config &c, const Plan &pl)
{
    if (pl.mode == kModeRows)
        return 0;
    // partial outputs and lse per (piece, head of the group); then the unit prefix sums (fixed
    // partitions) or one 16-byte record per work-group (balanced shares)
    const size_t G = (size_t)(c.num_q_heads / c.num_kv_heads);
    const size_t index_bytes = pl.mode == kModeFixed
                                   ? (size_t)round_up((c.max_batch + 1) * (int)sizeof(int), 16)
                                   : (size_t)kMaxGrid * 16;
    return (size_t)max_pieces_for(c, pl) * G * (kHeadDim + 1) * sizeof(float) + index_bytes;
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

// Work-groups of the main pass for a call with `batch` requests: never more than can be
// resident, never more than there can be units.  Balanced shares run ONE work-group per
// compute unit: four wavefronts with two tiles in flight each already draw a compute unit's
// share of the memory system (every workload streams as fast with 256 work-groups as with 512),
// and half as many shares are half as many cut rows, partial results and merge work-groups.
// Same box, 512 -> 256 work-groups: workload 3 83.4 -> 82.7 us, workload 7 373.5 -> 369.7 us,
// 16 x 8 x 131072 tokens 1208 -> 1199 us, 20 requests x 4096 tokens 62.7 -> 61.3 us, 4 x 32768
// 89.9 -> 87.0 us, 1 x 8192 19.9 -> 17.4 us.  Whole rows and caller-fixed partitions keep two
// per compute unit (512 rows of workload 2 are one row each; 0.2-0.9 % slower with one).
int grid_for(const lamina_attn *h, int batch)
{
    const Plan pl = {h->mode, h->parts, h->unit};
    long long wgs = (long long)batch * h->cfg.num_kv_heads * max_units_per_row(h->cfg, pl);
    const long long cap = h->mode == kModeBalanced ? (h->resident_wgs + 1) / 2 : h->resident_wgs;
    if (wgs > cap)
        wgs = cap;
    return (int)wgs;
}

int enqueue_decode(lamina_attn *h, const void *q, const void *k_cache, const void *v_cache,
                   const int32_t *seq_lens, const int32_t *block_table, void *out, float *lse,
                   const lamina_call_params *p);

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
    h->mode = pl.mode;
    h->parts = pl.parts;
    h->unit = pl.unit;
    h->max_pieces = max_pieces_for(*cfg, pl);
    h->row_cost = pl.mode == kModeBalanced ? kRowCostUnits : 0;
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
        h->resident_wgs = 2 * cus < kMaxGrid ? 2 * cus : kMaxGrid;
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

int lamina_attn_num_splits(lamina_attn_t h)
{
    if (!h)
        return 0;
    return h->mode == kModeRows ? 1 : (h->mode == kModeFixed ? h->parts : 0);
}

int lamina_attn_split_tokens(lamina_attn_t h) { return h ? h->unit : 0; }

int64_t lamina_attn_count_partials(lamina_attn_t h, const int32_t *host_seq_lens, int32_t batch)
{
    if (!h || !host_seq_lens || batch < 0 || batch > h->cfg.max_batch)
        return LAMINA_ERR_INVALID_ARG;
    if (h->mode == kModeRows)
        return 0;
    const int Hkv = h->cfg.num_kv_heads;
    auto units_of = [&](int len) {
        if (len > h->cfg.max_seq_len)
            len = h->cfg.max_seq_len;                     // as the kernel clamps it
        long long n = ((long long)len + h->unit - 1) / h->unit;
        if (n < 1)
            n = 1;
        if (h->mode == kModeFixed)
            return n > h->parts ? (long long)h->parts : n;
        return n + h->row_cost;
    };
    long long total = 0;
    for (int r = 0; r < batch; ++r)
        total += units_of(host_seq_lens[r]);
    const long long U = total * Hkv;
    const int nwg = grid_for(h, batch);
    const int skew = share_skew(h->mode == kModeBalanced, (unsigned)U, (unsigned)nwg);
    long long pieces = 0, before = 0;
    for (int r = 0; r < batch; ++r) {
        const long long n = units_of(host_seq_lens[r]);
        for (int g = 0; g < Hkv; ++g) {
            const long long S = Hkv * before + g * n;
            const long long np = h->mode == kModeFixed
                                     ? n
                                     : share_owner((unsigned)U, nwg, (unsigned)(S + n - 1), skew) -
                                           share_owner((unsigned)U, nwg, (unsigned)(S + h->row_cost), skew) + 1;
            if (np > 1)
                pieces += np;
        }
        before += n;
    }
    return pieces * h->group;
}

int lamina_decode_attention(lamina_attn_t h, const void *q, const void *k_cache,
                            const void *v_cache, const int32_t *seq_lens,
                            const int32_t *block_table, void *out, float *lse,
                            const lamina_call_params *p)
{
    if (!h)
        return LAMINA_ERR_INVALID_ARG;
    return enqueue_decode(h, q, k_cache, v_cache, seq_lens, block_table, out, lse, p);
}

}  // extern "C"

namespace {

// Validate one call and enqueue its kernels.  `h` may be a handle made by lamina_attn_create
// or a description on the caller's stack whose workspace is the static scratch area; nothing
// here allocates.
int enqueue_decode(lamina_attn *h, const void *q, const void *k_cache, const void *v_cache,
                   const int32_t *seq_lens, const int32_t *block_table, void *out, float *lse,
                   const lamina_call_params *p)
{
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
    mp.mode = h->mode;
    mp.P = h->parts;
    mp.unit = h->unit > 0 ? h->unit : 1;
    mp.row_cost = h->row_cost;
    // a length beyond what the handle (or the block table) was made for must not become an
    // out-of-bounds read: it is treated as the largest valid one
    mp.len_cap = c.max_seq_len;
    if (paged && (long long)p->block_table_stride * c.block_size < mp.len_cap)
        mp.len_cap = p->block_table_stride * c.block_size;
    mp.batch = p->batch;
    mp.out_is_bf16 = c.out_dtype == LAMINA_BF16;
    mp.scale_log2 = h->scale * kLog2e;
    if (h->mode != kModeRows) {
        mp.part_out = h->workspace;
        mp.part_lse = h->workspace + (size_t)h->max_pieces * h->group * kHeadDim;
        // the index area behind the pieces starts 16-byte aligned: max_pieces is even and a
        // piece holds G x 129 floats
        mp.cum = reinterpret_cast<int *>(mp.part_lse + (size_t)h->max_pieces * h->group);
        mp.tails = mp.cum;
    }

    DeviceGuard guard(c.device);
    if (!guard.ok())
        return fail(h, LAMINA_ERR_HIP, "cannot select the handle's device");
    hipStream_t stream = static_cast<hipStream_t>(p->stream);
    if ((long long)p->batch * c.num_kv_heads > (1LL << 30))
        return fail(h, LAMINA_ERR_UNSUPPORTED, "batch too large");
    const int wgs = grid_for(h, p->batch);
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
    if (h->mode == kModeBalanced) {
        if (wgs > 1) {
            BalancedMergeParams bp;
            bp.part_out = mp.part_out;
            bp.part_lse = mp.part_lse;
            bp.tails = mp.tails;
            bp.out = out;
            bp.lse = lse;
            bp.Hq = c.num_q_heads;
            bp.G = h->group;
            bp.out_is_bf16 = mp.out_is_bf16;
            hipLaunchKernelGGL(merge_balanced_kernel, dim3((unsigned)(wgs - 1)),
                               dim3((unsigned)(64 * h->group)), 0, stream, bp);
            e = hipGetLastError();
            if (e != hipSuccess)
                return fail_hip(h, "merge kernel launch", e);
        }
    } else if (h->mode == kModeFixed) {
        MergeParams gp;
        gp.part_out = mp.part_out;
        gp.part_lse = mp.part_lse;
        gp.cum = mp.cum;
        gp.out = out;
        gp.lse = lse;
        gp.Hq = c.num_q_heads;
        gp.Hkv = c.num_kv_heads;
        gp.G = h->group;
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
    np.pos_cap = c.max_seq_len;
    if (np.paged && (long long)p->block_table_stride * c.block_size < np.pos_cap)
        np.pos_cap = p->block_table_stride * c.block_size;
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

int lamina_fold_new_token_and_append(lamina_attn_t h, const void *q, const void *k_new,
                                     const void *v_new, const float *out_prev,
                                     const float *lse_prev, void *out, float *lse, void *k_cache,
                                     void *v_cache, const int32_t *positions,
                                     const int32_t *block_table, const lamina_call_params *p)
{
    if (!h)
        return LAMINA_ERR_INVALID_ARG;
    h->err[0] = 0;
    if (const char *msg = check_new_token_args(h, p, true, block_table))
        return fail(h, LAMINA_ERR_INVALID_ARG, msg);
    if (p->batch == 0)
        return LAMINA_OK;
    if (!q || !k_new || !v_new || !out_prev || !lse_prev || !out || !k_cache || !v_cache || !positions)
        return fail(h, LAMINA_ERR_INVALID_ARG,
                    "q, k_new, v_new, out_prev, lse_prev, out, k_cache, v_cache and positions must be "
                    "non-NULL");
    if (((uintptr_t)q | (uintptr_t)out_prev | (uintptr_t)out) % 8 != 0 ||
        ((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)k_cache | (uintptr_t)v_cache) % 16 != 0)
        return fail(h, LAMINA_ERR_INVALID_ARG,
                    "k_new, v_new and the caches must be 16-byte aligned, the other tensors 8-byte");
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
    np.k_cache = static_cast<unsigned char *>(k_cache);
    np.v_cache = static_cast<unsigned char *>(v_cache);
    np.positions = positions;
    np.block_table = block_table;
    np.rows = p->batch * h->cfg.num_q_heads;
    DeviceGuard guard(h->cfg.device);
    if (!guard.ok())
        return fail(h, LAMINA_ERR_HIP, "cannot select the handle's device");
    hipLaunchKernelGGL(fold_new_token_kernel, dim3((unsigned)((np.rows + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(p->stream), np);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(h, "fold-and-append kernel launch", e);
    return LAMINA_OK;
}

}  // extern "C"

// ============================================================================================
// The entry point for callers that cannot allocate: no handle, no hipMalloc; partial results
// go to the file-scope `scratch` array.
// ============================================================================================
namespace {

constexpr int kMaxStaticDevices = 64;

struct StaticDevice {
    bool ready;
    float *ptr;                  // device address of this GPU's copy of `scratch`
    int resident_wgs;
};
StaticDevice g_static_dev[kMaxStaticDevices];
std::mutex g_static_mu;

// Address of `dev`'s copy of the scratch array and the size of its persistent grid, resolved
// once per device with that device current.  Returns nullptr and sets *err on failure.
const StaticDevice *static_scratch_for(int dev, hipError_t *err)
{
    *err = hipSuccess;
    if (dev < 0 || dev >= kMaxStaticDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_static_mu);
    StaticDevice &sd = g_static_dev[dev];
    if (sd.ready)
        return &sd;
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e == hipSuccess && dev >= ndev)
        e = hipErrorInvalidDevice;
    if (e != hipSuccess) {
        *err = e;
        return nullptr;
    }
    DeviceGuard guard(dev);
    if (!guard.ok()) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
        *err = e != hipSuccess ? e : hipErrorInvalidSymbol;
        (void)hipGetLastError();
        return nullptr;
    }
    int cus = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess || cus <= 0) {
        *err = e != hipSuccess ? e : hipErrorInvalidDevice;
        return nullptr;
    }
    sd.ptr = static_cast<float *>(p);
    sd.resident_wgs = 2 * cus < kMaxGrid ? 2 * cus : kMaxGrid;
    sd.ready = true;
    return &sd;
}

}  // namespace

extern "C" {

int lamina_decode_attention_static(const lamina_attn_config *cfg, const void *q,
                                   const void *k_cache, const void *v_cache,
                                   const int32_t *seq_lens, const int32_t *block_table, void *out,
                                   float *lse, const lamina_call_params *p)
{
    int code;
    if (const char *msg = check_config(cfg, &code)) {
        snprintf(g_create_err, sizeof g_create_err, "%s", msg);
        return code;
    }
    lamina_attn h;                                        // on the stack: nothing is allocated
    h.cfg = *cfg;
    h.group = cfg->num_q_heads / cfg->num_kv_heads;
    const Plan pl = make_plan(*cfg);
    h.mode = pl.mode;
    h.parts = pl.parts;
    h.unit = pl.unit;
    h.max_pieces = max_pieces_for(*cfg, pl);
    h.row_cost = pl.mode == kModeBalanced ? kRowCostUnits : 0;
    h.scale = cfg->softmax_scale > 0.0f ? cfg->softmax_scale : 1.0f / sqrtf((float)cfg->head_dim);
    h.workspace_bytes = workspace_bytes_for(*cfg, pl);
    h.err[0] = 0;
    if (h.workspace_bytes > (size_t)LAMINA_STATIC_SCRATCH_BYTES) {
        snprintf(g_create_err, sizeof g_create_err,
                 "this configuration needs %zu bytes of partial results, the static scratch area "
                 "holds %zu: use a handle (lamina_attn_create), fewer partitions or a smaller "
                 "max_batch",
                 h.workspace_bytes, (size_t)LAMINA_STATIC_SCRATCH_BYTES);
        return LAMINA_ERR_WORKSPACE;
    }
    hipError_t e;
    const StaticDevice *sd = static_scratch_for(cfg->device, &e);
    if (!sd) {
        snprintf(g_create_err, sizeof g_create_err, "static scratch area on device %d: %s",
                 cfg->device, hipGetErrorString(e));
        return LAMINA_ERR_HIP;
    }
    h.workspace = sd->ptr;
    h.resident_wgs = sd->resident_wgs;
    const int rc = enqueue_decode(&h, q, k_cache, v_cache, seq_lens, block_table, out, lse, p);
    if (rc != LAMINA_OK)
        snprintf(g_create_err, sizeof g_create_err, "%s", h.err);
    return rc;
}

}  // extern "C"
