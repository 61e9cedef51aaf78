// GQA decode attention over the compressed, ragged per-layer cache (paper Sec. 2.1, decoding
// phase: the new key/value is appended, then softmax(q K^T / sqrt d) V over every cached slot).
//
// Bandwidth-bound: every K and V row is read once and serves all g query heads of its KV group.
// Rows are ragged (layer budgets differ by 25x), so the work is cut into block-units of 128 to 1024
// slots listed in device-side work lists that vlc_topk_compact builds; a call launches one block per
// unit of the slice of a list that belongs to its layer range (launches over a layer range are capped
// at one resident round of blocks, which then walk the slice with the grid as stride).  Inside a
// block-unit the tiles of 32 slots are dealt round-robin to the 4 waves:
//   1. K and V rows are loaded 16 bytes per lane (LPR lanes per row, fully coalesced), all
//      issued before any arithmetic;
//   2. logits: packed-bf16 dot products (v_dot2_f32_bf16) against the g query rows held in
//      registers, summed over the LPR lanes of a row with DPP rotations, parked in LDS;
//   3. softmax bookkeeping with one 16-lane row per head (DPP row reductions only), the
//      probabilities parked in LDS as bf16 pairs;
//   4. P.V with the K lane mapping: two slots at a time through v_perm + v_dot2_f32_bf16 with
//      the probability pairs broadcast from LDS (fp32 FMAs for fp32 storage); the 64/LPR row
//      groups of a wave are summed once per block-unit.
// The 4 waves merge through LDS.  A row that spans several block-units leaves unnormalised
// partials in scratch; the unit that finishes last (device-scope counter) merges them.  The
// partials and the counter are only ever touched with device-scope atomic accesses, which
// are coherent across the XCDs' L2 caches by themselves, so no cache-wide release/acquire
// fence is needed (those cost tens of microseconds here).  With g <= 8 query rows per KV head the
// work is a stream, not a contraction; the matrix cores only take over step 2 when g > 4 (bf16,
// d = 128), where the vector unit would otherwise be the bound.
//
// Nothing that changes from step to step is a launch parameter: the number of appends a layer has
// received is read from the cache (dev.appended), and the launch that appends leaves count + 1 behind.
// Every block takes a ticket (dev.readers) right after it has read the count; the block that holds the
// last ticket of the launch knows that every other block has read the count and writes the new one.
// A HIP graph that holds one decode step can therefore be replayed step after step.
#include <stddef.h>
#include <stdlib.h>

#include <type_traits>

#include "common.h"
#include "internal.h"

// Measurement builds only (the library then computes wrong results on purpose; the default, 0, is the product):
// -DVLC_DECODE_ABLATE=<bits> takes phases out of the attention kernel so that their share of a launch can be
// timed.  1: the tiles are loaded and waited for, but no arithmetic is done on them; 2: a block-unit ends after
// its last tile (no merge of the waves, no partials, no output); 4: every block-unit is treated as a whole row
// (the merge of the waves and the output store stay, the partials and the cross-block count go); 8: the appended
// row is not copied into the cache (its position is still recorded and the count advances).  All accesses stay in
// bounds in every combination.
#ifndef VLC_DECODE_ABLATE
#define VLC_DECODE_ABLATE 0
#endif

namespace vlc {
namespace {

struct DecodeParams {
    const void* q;
    const void* k_new;
    const void* v_new;
    void* out;
    const float* sm_scale;
    CacheDev dev;
    WorkList wl;             // the work list this launch walks
    int ub_shift, us_shift;  // log2 of the list's unit sizes
    int B, L, Hq, Hkv, m;
    int layer_begin, n_layers, T_max;
    int append_mode;         // 0: attend only; 1: k_new / v_new are appended by this kernel
    int merge_mode;          // 1: last unit of a row merges in-kernel; 2: separate merge kernel
    int zigzag;              // 1 off; 2: tile order within a unit alternates between steps; 3: also the walk over the whole units
    int kv_fp8;              // the cache rows are E4M3 codes with per-row scales
    float default_scale;
};

template <typename T> __device__ __forceinline__ float dot16(const uint4& a, const uint4& b, float acc);
template <> __device__ __forceinline__ float dot16<bf16_t>(const uint4& a, const uint4& b, float acc) {
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.x), __builtin_bit_cast(bf16x2_t, b.x), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.y), __builtin_bit_cast(bf16x2_t, b.y), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.z), __builtin_bit_cast(bf16x2_t, b.z), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w), __builtin_bit_cast(bf16x2_t, b.w), acc, false);
    return acc;
}
template <> __device__ __forceinline__ float dot16<float>(const uint4& a, const uint4& b, float acc) {
    acc = fmaf(__uint_as_float(a.x), __uint_as_float(b.x), acc);
    acc = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), acc);
    acc = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), acc);
    acc = fmaf(__uint_as_float(a.w), __uint_as_float(b.w), acc);
    return acc;
}

constexpr int pad_pow2(int g) { return g <= 1 ? 1 : (g <= 2 ? 2 : (g <= 4 ? 4 : 8)); }

__device__ __forceinline__ void store_agent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_agent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_agent(int32_t* p, int32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// two neighbouring floats (8-byte aligned) as one device-scope store
__device__ __forceinline__ void store_agent2(float* p, float a, float b) {
    const unsigned long long v = ((unsigned long long)__float_as_uint(b) << 32) | __float_as_uint(a);
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// two neighbouring output elements as one store
__device__ __forceinline__ void store_pair(float* p, float a, float b) { *reinterpret_cast<float2*>(p) = make_float2(a, b); }
__device__ __forceinline__ void store_pair(bf16_t* p, float a, float b) {
    *reinterpret_cast<uint32_t*>(p) = (uint32_t)f32_to_bf16_bits(a) | ((uint32_t)f32_to_bf16_bits(b) << 16);
}
__device__ __forceinline__ int32_t add_agent(int32_t* p, int32_t v) {
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Merge the nu partials (unnormalised output, running max, running sum) of one row; partials
// of consecutive units of a row are consecutive.  COHERENT: read with device-scope loads.
// The loads of up to eight partials are all issued before the first is used: a row's merge then
// costs one round trip to memory per eight units instead of one per unit.
template <typename T, int D, int G, bool COHERENT, int THREADS>
__device__ __forceinline__ void merge_partials(const float* part, T* outp, int nu, int tid) {
    constexpr int DP = D + 2;
    constexpr int UNIT = G * DP;
    constexpr int BATCH = 8;
    for (int x = tid; x < G * D; x += THREADS) {
        const int h = x / D, e = x % D;
        const float* ph = part + h * DP;
        float mt = -INFINITY, o = 0.f, lt = 0.f;
        for (int s0 = 0; s0 < nu; s0 += BATCH) {
            float ms[BATCH], ls[BATCH], os[BATCH];
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const float* p = ph + (size_t)min(s0 + j, nu - 1) * UNIT;      // past the end: the last partial again, ignored below
                ms[j] = COHERENT ? load_agent(p + D) : p[D];
                ls[j] = COHERENT ? load_agent(p + D + 1) : p[D + 1];
                os[j] = COHERENT ? load_agent(p + e) : p[e];
            }
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                if (s0 + j < nu) {
                    const float mn = fmaxf(mt, ms[j]);
                    const float wo = (mt > -INFINITY) ? exp2_fast(mt - mn) : 0.f;
                    const float wn = (ms[j] > -INFINITY) ? exp2_fast(ms[j] - mn) : 0.f;
                    o = o * wo + os[j] * wn;
                    lt = lt * wo + ls[j] * wn;
                    mt = mn;
                }
            }
        }
        Elem<T>::store(outp + x, o / lt);
    }
}

// Sum of G values over the 16 lanes of a DPP row, scattered: lane c ends up with the total of
// head (c >> 2) & 3 (for G <= 4) -- 11 operations instead of 16 for four separate all-reduces.
template <int G>
__device__ __forceinline__ float row16_reduce_scatter(const float (&v)[G], int c) {
    static_assert(G <= 4, "scatter form covers up to four heads");
    const bool hi8 = (c & 8) != 0, hi4 = (c & 4) != 0;
    // distance 8: lanes with bit 3 clear keep heads {0,1}, the others heads {2,3}
    const float v0 = v[0], v1 = G > 1 ? v[1] : 0.f, v2 = G > 2 ? v[2] : 0.f, v3 = G > 3 ? v[3] : 0.f;
    const float keepA = hi8 ? v2 : v0, sendA = hi8 ? v0 : v2;
    const float keepB = hi8 ? v3 : v1, sendB = hi8 ? v1 : v3;
    const float a = keepA + dpp_mov<kDppRowRor(8)>(sendA);
    const float b = keepB + dpp_mov<kDppRowRor(8)>(sendB);
    // bit 2 picks between the two heads still held; the half-row mirror pairs lane c with c^7
    const float keep = hi4 ? b : a, send = hi4 ? a : b;
    float r = keep + dpp_mov<kDppRowHalfMirror>(send);  // partner c^7: other value of bit 2, same bit 3
    // the two quads of a half-row now hold complementary lanes: finish with sums inside the quad
    r += dpp_mov<kDppQuadPerm(2, 3, 0, 1)>(r);
    r += dpp_mov<kDppQuadPerm(1, 0, 3, 2)>(r);
    return r;                                           // total of head 2*bit3 + bit2
}

// The same for up to eight heads: three halving levels (lane bits 3, 2, 1 choose the heads a lane keeps,
// the partner at c^8, c^7, c^2 supplies its share of them) and one plain add with c^1.  The partners'
// offsets {8} x {7} x {2} x {1} reach all sixteen lanes.  Lane c ends with the total of head
// 4 bit3 + 2 bit2 + bit1: 22 operations instead of 40 for eight separate all-reduces.
template <int G>
__device__ __forceinline__ float row16_reduce_scatter8(const float (&v)[G], int c) {
    static_assert(G > 4 && G <= 8, "scatter form for five to eight heads");
    const bool b3 = (c & 8) != 0, b2 = (c & 4) != 0, b1 = (c & 2) != 0;
    float x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = j < G ? v[j] : 0.f;
    float a[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {                           // bit 3 clear keeps heads 0..3, set keeps 4..7
        const float keep = b3 ? x[4 + j] : x[j], send = b3 ? x[j] : x[4 + j];
        a[j] = keep + dpp_mov<kDppRowRor(8)>(send);
    }
    float b[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {                           // bit 2 picks the pair; partner c^7 has the other value of bit 2
        const float keep = b2 ? a[2 + j] : a[j], send = b2 ? a[j] : a[2 + j];
        b[j] = keep + dpp_mov<kDppRowHalfMirror>(send);
    }
    const float keep = b1 ? b[1] : b[0], send = b1 ? b[0] : b[1];
    float r = keep + dpp_mov<kDppQuadPerm(2, 3, 0, 1)>(send);   // partner c^2: other value of bit 1
    r += dpp_mov<kDppQuadPerm(1, 0, 3, 2)>(r);                  // partner c^1
    return r;
}

// Max / sum over the 64 lanes of a wave from a DPP row all-reduce plus four lane reads.
__device__ __forceinline__ float lane_value(float x, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}
__device__ __forceinline__ float wave_max_dpp(float x) {
    x = fmaxf(x, dpp_mov<kDppRowRor(8)>(x));
    x = fmaxf(x, dpp_mov<kDppRowRor(4)>(x));
    x = fmaxf(x, dpp_mov<kDppRowRor(2)>(x));
    x = fmaxf(x, dpp_mov<kDppRowRor(1)>(x));
    return fmaxf(fmaxf(lane_value(x, 0), lane_value(x, 16)), fmaxf(lane_value(x, 32), lane_value(x, 48)));
}
__device__ __forceinline__ float wave_sum_dpp(float x) {
    x = group_allreduce_sum<16>(x);
    return (lane_value(x, 0) + lane_value(x, 16)) + (lane_value(x, 32) + lane_value(x, 48));
}

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t uniform64(int64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

template <typename T> struct IsBf16 { static constexpr bool value = false; };
template <> struct IsBf16<bf16_t> { static constexpr bool value = true; };

// Q8: the cache rows are E4M3 codes with one fp32 scale per row (8 bytes per lane instead of 16); codes are
// expanded to bf16 (exactly) where they are consumed, the K scale multiplies the finished logit, the
// V scale the probability before it is rounded to bf16.  The row being appended is quantised by the wave whose tile
// holds its slot, which attends over the quantised row and stores it.
// Blocks of four waves, three per CU for up to four query heads per KV head (two where the accumulators need the
// registers): the blocks of a CU overlap each other's start-up and merge phases.  One wide block per row (12 waves,
// no merge across blocks) measured no faster: the row's loads then queue at a single CU's address path.
template <typename T, int D, int G, bool Q8>
__global__ __launch_bounds__(256, (G <= 4 && (IsBf16<T>::value || D == 64) ? 3 : 2)) void decode_kernel(DecodeParams P) {
    constexpr int NW = 4;                       // waves per block
    constexpr int THREADS = NW * 64;
    constexpr bool BF = IsBf16<T>::value;
    static_assert(!Q8 || BF, "FP8 caches hold bf16 models");
    constexpr int EP = Elem<T>::kPer16B;        // elements in a 16-byte chunk
    constexpr int LPR = D / EP;                 // lanes per K/V row
    constexpr int KPI = 64 / LPR;               // rows per wave load
    constexpr int TK = 32;                      // slots per tile
    constexpr int NIT = TK / KPI;               // loads per tile and operand
    constexpr int GP = pad_pow2(G);
    constexpr int HR = (GP + 3) / 4;            // heads per 16-lane row in the softmax step
    constexpr int KK = TK / 16;                 // slots per lane in the softmax step
    constexpr int DP = D + 2;
    constexpr bool SCATTER = (LPR == 16 && G <= 4);
    // More than four query heads per KV head (bf16, d = 128): the logits of a tile come from the matrix cores,
    // S = K Q^T with the query heads padded into the 32 columns of v_mfma_f32_32x32x16_bf16 (8 instructions per
    // 32-slot tile instead of 7 x 32 packed dot products and their lane reductions; most columns are padding, but
    // the matrix pipe is otherwise idle and the vector unit is what bounds these shapes).  A lane then fetches
    // the K fragment it feeds to the instruction: row lane % 32 of the tile, 16 bytes at k-step 2 s + lane / 32.
    constexpr bool MF = BF && !Q8 && D == 128 && G > 4;
    static_assert(G <= LPR, "one lane per head needed when parking logits");
    static_assert(NIT % 2 == 0, "P.V pairs consecutive loads");

    __shared__ __align__(16) float sL[NW][TK][GP];        // logits, then fp32 probabilities (fp32 path)
    __shared__ __align__(16) uint32_t sPk[NW][TK / 2][GP]; // bf16 probability pairs of loads (2i, 2i+1)
    constexpr int DL = D + 4;                   // LDS row of the wave merge: D outputs, max, sum; a multiple of 16 bytes
    __shared__ __align__(16) float sMerge[NW][G][DL];
    __shared__ int sLast;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int sub = lane / LPR, c = lane % LPR;
    const int srow = lane >> 4, scol = lane & 15;
    // The work list and its layer index were written by the compaction, in an earlier launch: they are constant
    // while this kernel runs and are read as such, which puts their (block-uniform) loads on the scalar unit.
    typedef const __attribute__((address_space(4))) int32_t* IndexPtr;
    // ---- what the whole launch shares: the slice of the list, and the append count of its layers
    const IndexPtr layer_start = (IndexPtr)P.wl.layer_start;
    const int begin = P.layer_begin ? layer_start[P.layer_begin] : 0;
    const int end = layer_start[P.layer_begin + P.n_layers];
    const int appended = P.dev.appended[P.layer_begin];
    int mode = P.append_mode;
    // more steps than slots were reserved (only a replayed graph gets here): attend over what the cache holds,
    // append nothing, count nothing, and report it (after the block's first unit: a store in front of the unit
    // record's load would keep that load off the scalar unit)
    const bool over = mode && appended >= P.T_max;
    if (over) mode = 0;
    const bool appending = mode == 1;
    const int step = appended + (mode ? 1 : 0); // appends the cache holds once this launch is done
    // A block takes its ticket only after it has read the append count: the operand of the ticket's atomic add
    // is produced by a statement that consumes the count.
    int one = 1;
    asm volatile("" : "+s"(one) : "s"(appended));
    // One block-unit per block while the grid covers the slice (the hardware dispatcher then balances the ragged
    // units); a capped grid walks the rest of the slice with the grid as stride (below).  The grid is a host-side
    // upper bound on the units of the layer range, surplus blocks leave at once.  Returns false past the slice.
    // A is the parameter struct: the kernel's own copy for a block's first unit, a view of the kernel-argument
    // memory that the compiler cannot see through for further units (see below).
    auto process_unit = [&](auto firstc, const auto& A, int w0) -> bool {
        constexpr bool FIRST = decltype(firstc)::value;
        // The block that holds the last ticket of its layer, and then of the launch, publishes the new count.
        auto finish = [&](int ticket, int il, int n_layer) {
            if (ticket != n_layer - 1) return;
            store_agent(A.dev.readers + il * kReaderStride, 0);
            if (A.n_layers > 1) {
                if (add_agent(A.dev.readers + A.L * kReaderStride, 1) != A.n_layers - 1) return;
                store_agent(A.dev.readers + A.L * kReaderStride, 0);
            }
            for (int l = A.layer_begin; l < A.layer_begin + A.n_layers; ++l) store_agent(A.dev.appended + l, step);
        };
        int w = w0;
        if (A.wl.by_size && A.zigzag > 2 && (step & 1)) {   // size-class order, odd step: the whole units are walked backwards, so that
            const int nf = min(((IndexPtr)A.wl.layer_start)[A.L + 1], (int)gridDim.x);   // what the memory-side cache kept of the last step comes first
            const int nf8 = nf & ~7;            // whole groups of 8 change places, so a unit stays on its XCD (and its L2)
            if (w < nf8) w = nf8 - 8 - (w & ~7) + (w & 7);
        }
        w += begin;
        if (!FIRST && w >= end) return false;
        if (w >= A.wl.cap) return false;
        // the unit record, word by word (a block's first unit: requested together with the bounds of the slice)
        static_assert(offsetof(WorkItem, row_abs) == 0 && offsetof(WorkItem, key0) == 4 && offsetof(WorkItem, kept) == 8 &&
                      offsetof(WorkItem, unit) == 12 && offsetof(WorkItem, kbase) == 16 && offsetof(WorkItem, idx_base) == 24 &&
                      offsetof(WorkItem, b) == 32 && offsetof(WorkItem, l) == 36 && offsetof(WorkItem, canon) == 40 &&
                      offsetof(WorkItem, ucap) == 44 && offsetof(WorkItem, hkv) == 48 && offsetof(WorkItem, layer_units) == 52,
                      "the record is read as 16 words");
        const IndexPtr rec = (IndexPtr)(A.wl.items + w);
        const int row_abs = rec[0], key0 = rec[1], kept = rec[2], unit = rec[3];
        const int64_t kbase = (int64_t)(((uint64_t)(uint32_t)rec[5] << 32) | (uint32_t)rec[4]);
        const int64_t idx_base = (int64_t)(((uint64_t)(uint32_t)rec[7] << 32) | (uint32_t)rec[6]);
        const int ib = rec[8], il = rec[9], canon = rec[10], ucap = rec[11], hkv = rec[12], n_layer = rec[13];
        if (w >= end) return false;
        const int lr = il - A.layer_begin;
        // The ticket: taken at once by a unit that has nothing to read, else behind the loads of the unit's first
        // tile (returns come back in issue order: in front of them it would hold up the first tile).
        auto take_ticket = [&]() { return (mode && tid == 0) ? add_agent(A.dev.readers + il * kReaderStride, one) : -1; };
        T* outp = reinterpret_cast<T*>(A.out) + ((size_t)(lr * A.B + ib) * A.Hq + (size_t)hkv * G) * D;
        if (kept == 0) {                        // request rejected at compaction: defined output, no reads
            const int ticket = take_ticket();
            for (int x = tid; x < G * D; x += THREADS) Elem<T>::store(outp + x, 0.f);
            if (mode && tid == 0) finish(ticket, il, n_layer);
            return true;
        }
        const int len = kept + step;
        if (key0 >= len) {                      // unit reserved for later appends
            const int ticket = take_ticket();
            if (mode && tid == 0) finish(ticket, il, n_layer);
            return true;
        }
        const int nbig = kept >> A.ub_shift;    // units of this row that hold slots now: the whole ones, and the small ones up to len
#if VLC_DECODE_ABLATE & 4
        const int nu = 1;
#else
        const int nu = nbig + ((len - (nbig << A.ub_shift) + (1 << A.us_shift) - 1) >> A.us_shift);
#endif
        const int cap = kept + A.T_max;
        const int new_slot = appending ? len - 1 : -1;
        const T* Kbase = reinterpret_cast<const T*>(A.dev.kv) + kbase;
        const T* Vbase = Kbase + (int64_t)A.Hkv * cap * D;
        const uint8_t* K8 = reinterpret_cast<const uint8_t*>(A.dev.kv) + kbase;      // FP8 cache: one byte per element
        const uint8_t* V8 = K8 + (int64_t)A.Hkv * cap * D;
        const float* Ksc = A.dev.scales + kbase / D;
        const float* Vsc = Ksc + (int64_t)A.Hkv * cap;
        const T* knew = reinterpret_cast<const T*>(A.k_new) + ((size_t)(lr * A.B + ib) * A.Hkv + hkv) * D;
        const T* vnew = reinterpret_cast<const T*>(A.v_new) + ((size_t)(lr * A.B + ib) * A.Hkv + hkv) * D;
        const float scale2 = (A.sm_scale ? A.sm_scale[il] : A.default_scale) * kLog2e;

        uint4 qv[MF ? 1 : G];                       // vector path: the 16 bytes of each query row that match this lane's K bytes
        uint4 qf[MF ? D / 16 : 1];                  // matrix path: B fragments, column lane % 32 = query head (zero beyond G)
        const T* qrow = reinterpret_cast<const T*>(A.q) + ((size_t)(lr * A.B + ib) * A.Hq + (size_t)hkv * G) * D;
        if constexpr (MF) {
            const int n = lane & 31, half = lane >> 5;
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks)
                qf[ks] = n < G ? *reinterpret_cast<const uint4*>(qrow + (size_t)n * D + ks * 16 + half * 8) : make_uint4(0, 0, 0, 0);
        } else {
#pragma unroll
            for (int h = 0; h < G; ++h) qv[h] = *reinterpret_cast<const uint4*>(qrow + (size_t)h * D + c * EP);
        }

        // running max / sum live per 16-lane row: row r owns heads r*HR .. r*HR + HR - 1
        float m_run[HR], l_run[HR], acc[G][EP];
#pragma unroll
        for (int hh = 0; hh < HR; ++hh) { m_run[hh] = -INFINITY; l_run[hh] = 0.f; }
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
            for (int e = 0; e < EP; ++e) acc[h][e] = 0.f;

        // K and V of a tile sit in separate register buffers; all 16 KB of a tile are requested before any
        // arithmetic on it.
        uint4 kb[Q8 ? 1 : NIT], vb[Q8 ? 1 : NIT];
        uint2 kb8[Q8 ? NIT : 1], vb8[Q8 ? NIT : 1];
        float ksc[Q8 ? NIT : 1], vsc[Q8 ? KK : 1];
        auto load_row8 = [&](const uint8_t* base, int t0, int i) -> uint2 {
            const int key = t0 + i * KPI + sub;
            return (key < len) ? *reinterpret_cast<const uint2*>(base + (int64_t)key * D + c * 8) : make_uint2(0, 0);
        };
        auto load_row = [&](auto fullc, const T* base, const T* fresh, int t0, int i) -> uint4 {
            constexpr bool FULL = decltype(fullc)::value;
            if constexpr (FULL && MF) {
                // one 32-bit lane offset per tile and the load's place in the tile as a constant: the addressing
                // form that takes no address registers per load (a row is far shorter than 4 GiB).  Measured: 4 %
                // on the matrix path, where registers are short; nothing, or a slight loss, on the others.
                const uint32_t off = ((uint32_t)(t0 + sub) * D + c * EP) * (uint32_t)sizeof(T);
                return *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(base) + off + (size_t)i * KPI * D * sizeof(T));
            } else if constexpr (FULL) {
                return *reinterpret_cast<const uint4*>(base + (int64_t)(t0 + i * KPI + sub) * D + c * EP);
            } else {
                const int key = t0 + i * KPI + sub;
                const T* src = (key == new_slot) ? fresh : base + (int64_t)key * D;
                return (key < len) ? *reinterpret_cast<const uint4*>(src + c * EP) : make_uint4(0, 0, 0, 0);
            }
        };
        auto issue_k = [&](int t0) {
            if constexpr (Q8) {
                if (t0 + TK <= len) {           // whole tile (wave-uniform): no per-row tests, one lane offset, constant displacements
                    const uint32_t off = (uint32_t)(t0 + sub) * D + c * 8;
                    const uint32_t so = (uint32_t)(t0 + sub) * (uint32_t)sizeof(float);
#pragma unroll
                    for (int i = 0; i < NIT; ++i) {
                        kb8[i] = *reinterpret_cast<const uint2*>(K8 + off + (size_t)i * KPI * D);
                        ksc[i] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(Ksc) + so + (size_t)i * KPI * sizeof(float));
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < NIT; ++i) {
                        kb8[i] = load_row8(K8, t0, i);
                        const int key = t0 + i * KPI + sub;
                        ksc[i] = key < len ? Ksc[key] : 0.f;
                    }
                }
            } else if constexpr (MF) {
                const bool full = (t0 + TK <= len) && !(new_slot >= t0 && new_slot < t0 + TK);   // wave-uniform
                const int key = t0 + (lane & 31);
                if (full) {
                    const uint32_t off = ((uint32_t)key * D + (lane >> 5) * 8) * (uint32_t)sizeof(T);
#pragma unroll
                    for (int ks = 0; ks < NIT; ++ks)
                        kb[ks] = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(Kbase) + off + (size_t)ks * 16 * sizeof(T));
                } else {
                    const T* src = (key == new_slot ? knew : Kbase + (int64_t)key * D) + (lane >> 5) * 8;
                    const bool live = key < len;
#pragma unroll
                    for (int ks = 0; ks < NIT; ++ks) kb[ks] = live ? *reinterpret_cast<const uint4*>(src + ks * 16) : make_uint4(0, 0, 0, 0);
                }
            } else {
                const bool full = (t0 + TK <= len) && !(new_slot >= t0 && new_slot < t0 + TK);   // wave-uniform
#pragma unroll
                for (int i = 0; i < NIT; ++i)
                    kb[i] = full ? load_row(std::true_type{}, Kbase, knew, t0, i) : load_row(std::false_type{}, Kbase, knew, t0, i);
            }
        };
        auto issue_v = [&](int t0) {
            if constexpr (Q8) {
                if (t0 + TK <= len) {
                    const uint32_t off = (uint32_t)(t0 + sub) * D + c * 8;
                    const uint32_t so = (uint32_t)(t0 + scol) * (uint32_t)sizeof(float);
#pragma unroll
                    for (int i = 0; i < NIT; ++i) vb8[i] = *reinterpret_cast<const uint2*>(V8 + off + (size_t)i * KPI * D);
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk)
                        vsc[kk] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(Vsc) + so + (size_t)kk * 16 * sizeof(float));
                } else {
#pragma unroll
                    for (int i = 0; i < NIT; ++i) vb8[i] = load_row8(V8, t0, i);
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) {
                        const int key = t0 + scol + 16 * kk;      // the slots this lane owns in the softmax step
                        vsc[kk] = key < len ? Vsc[key] : 0.f;
                    }
                }
            } else {
                const bool full = (t0 + TK <= len) && !(new_slot >= t0 && new_slot < t0 + TK);
                if constexpr (MF) {             // the whole tile and the ragged one as two instruction streams
                    if (full) {
#pragma unroll
                        for (int i = 0; i < NIT; ++i) vb[i] = load_row(std::true_type{}, Vbase, vnew, t0, i);
                    } else {
#pragma unroll
                        for (int i = 0; i < NIT; ++i) vb[i] = load_row(std::false_type{}, Vbase, vnew, t0, i);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < NIT; ++i)
                        vb[i] = full ? load_row(std::true_type{}, Vbase, vnew, t0, i) : load_row(std::false_type{}, Vbase, vnew, t0, i);
                }
            }
        };
        auto tile_body = [&](auto fullc, int t0) {
            constexpr bool FULL = decltype(fullc)::value;
#if VLC_DECODE_ABLATE & 1
            if constexpr (!Q8) {                // every loaded word is used once, so the loads and their waits stay
                uint32_t x = 0;
#pragma unroll
                for (int i = 0; i < NIT; ++i) x ^= kb[i].x ^ kb[i].y ^ kb[i].z ^ kb[i].w ^ vb[i].x ^ vb[i].y ^ vb[i].z ^ vb[i].w;
                acc[0][0] += __uint_as_float(x & 0x3fffffu);
                return;
            }
#endif
            // ---- logits of 32 slots -> LDS
            if constexpr (MF) {
                f32x16_t sacc = {0};
#pragma unroll
                for (int ks = 0; ks < NIT; ++ks)
                    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kb[ks]), __builtin_bit_cast(bf16x8_t, qf[ks]), sacc, 0, 0, 0);
                // sacc[i] = <k_slot, q_head>: head = lane % 32, slot = 8 (i / 4) + 4 (lane / 32) + i % 4
                const int n = lane & 31;
                if (n < G) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int slot = 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
                        sL[wave][slot][n] = (FULL || t0 + slot < len) ? sacc[i] * scale2 : -INFINITY;
                    }
                }
            } else {
#pragma unroll
            for (int i = 0; i < NIT; ++i) {
                const int key = t0 + i * KPI + sub;
                const bool live = FULL || key < len;
                float part[G];
                uint4 kq;
                float rs = scale2;                                  // logit scale, times the row's K scale for FP8 rows
                if constexpr (Q8) { kq = e4m3x8_to_bf16x8(kb8[i]); rs *= ksc[i]; } else { kq = kb[i]; }
#pragma unroll
                for (int h = 0; h < G; ++h) part[h] = dot16<T>(kq, qv[h], 0.f);
                if constexpr (SCATTER) {
                    const float tot = row16_reduce_scatter<G>(part, c);
                    const int hh = ((c >> 3) << 1) | ((c >> 2) & 1);
                    if ((c & 3) == 0 && hh < G) sL[wave][i * KPI + sub][hh] = live ? tot * rs : -INFINITY;
                } else if constexpr (LPR == 16 && G > 4) {
                    const float tot = row16_reduce_scatter8<G>(part, c);
                    const int hh = ((c >> 3) << 2) | (((c >> 2) & 1) << 1) | ((c >> 1) & 1);
                    if ((c & 1) == 0 && hh < G) sL[wave][i * KPI + sub][hh] = live ? tot * rs : -INFINITY;
                } else {
                    float mine = 0.f;
#pragma unroll
                    for (int h = 0; h < G; ++h) {
                        const float tot = group_allreduce_sum<LPR>(part[h]);
                        mine = (c == h) ? tot : mine;
                    }
                    if (c < G) sL[wave][i * KPI + sub][c] = live ? mine * rs : -INFINITY;
                }
            }
            }
            __builtin_amdgcn_wave_barrier();
            // ---- softmax bookkeeping: 16-lane row r handles heads r*HR.., lane column j slots j, j+16
            float corr_row[HR];
#pragma unroll
            for (int hh = 0; hh < HR; ++hh) {
                const int h = srow * HR + hh;
                float x[KK], mt = -INFINITY;
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) {
                    x[kk] = (h < G) ? sL[wave][scol + 16 * kk][h % GP] : -INFINITY;
                    mt = fmaxf(mt, x[kk]);
                }
                mt = fmaxf(mt, dpp_mov<kDppRowRor(8)>(mt));
                mt = fmaxf(mt, dpp_mov<kDppRowRor(4)>(mt));
                mt = fmaxf(mt, dpp_mov<kDppRowRor(2)>(mt));
                mt = fmaxf(mt, dpp_mov<kDppRowRor(1)>(mt));
                const float m_new = fmaxf(m_run[hh], mt);            // finite for real heads: the tile holds >= 1 slot
                float ps = 0.f;
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) {
                    const float pr = exp2_fast(x[kk] - m_new);
                    ps += pr;
                    if (h < G) {
                        const int slot = scol + 16 * kk, li = slot / KPI, ls = slot % KPI;
                        if constexpr (BF) {
                            // bf16 probability into its half of the pair word of loads (li & ~1, li | 1)
                            const __bf16 pb = Q8 ? (__bf16)(pr * vsc[kk]) : (__bf16)pr;      // FP8 rows: the V scale rides on the probability
                            reinterpret_cast<uint16_t*>(&sPk[wave][(li >> 1) * KPI + ls][h % GP])[li & 1] =
                                __builtin_bit_cast(uint16_t, pb);
                        } else {
                            sL[wave][slot][h % GP] = pr;
                        }
                    }
                }
                ps = group_allreduce_sum<16>(ps);
                corr_row[hh] = exp2_fast(m_run[hh] - m_new);
                l_run[hh] = l_run[hh] * corr_row[hh] + ps;
                m_run[hh] = m_new;
            }
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const float ch = lane_value(corr_row[h % HR], 16 * (h / HR));
#pragma unroll
                for (int e = 0; e < EP; ++e) acc[h][e] *= ch;
            }
            __builtin_amdgcn_wave_barrier();
            // ---- P.V
            if constexpr (BF) {
#pragma unroll
                for (int i = 0; i < NIT; i += 2) {
                    const uint32_t* pp = &sPk[wave][(i >> 1) * KPI + sub][0];
                    uint32_t pk[G];
#pragma unroll
                    for (int h = 0; h < G; ++h) pk[h] = pp[h];
                    uint4 va, vbb;
                    if constexpr (Q8) { va = e4m3x8_to_bf16x8(vb8[i]); vbb = e4m3x8_to_bf16x8(vb8[i + 1]); }
                    else { va = vb[i]; vbb = vb[i + 1]; }
                    const uint32_t a[4] = {va.x, va.y, va.z, va.w};
                    const uint32_t b[4] = {vbb.x, vbb.y, vbb.z, vbb.w};
#pragma unroll
                    for (int d2 = 0; d2 < 4; ++d2) {
                        const uint32_t lo = __builtin_amdgcn_perm(b[d2], a[d2], 0x05040100u);   // (a.even, b.even)
                        const uint32_t hi = __builtin_amdgcn_perm(b[d2], a[d2], 0x07060302u);   // (a.odd,  b.odd)
#pragma unroll
                        for (int h = 0; h < G; ++h) {
                            acc[h][2 * d2] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, lo), __builtin_bit_cast(bf16x2_t, pk[h]), acc[h][2 * d2], false);
                            acc[h][2 * d2 + 1] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, hi), __builtin_bit_cast(bf16x2_t, pk[h]), acc[h][2 * d2 + 1], false);
                        }
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < NIT; ++i) {
                    float f[EP];
                    unpack16(vb[i], f, (const T*)nullptr);
                    const float* pp = &sL[wave][i * KPI + sub][0];
#pragma unroll
                    for (int h = 0; h < G; ++h) {
                        const float ph = pp[h];
#pragma unroll
                        for (int e = 0; e < EP; ++e) acc[h][e] = fmaf(ph, f[e], acc[h][e]);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        };
        // tiles of the unit are dealt round-robin to the 4 waves, so a partly filled unit keeps all of them busy.
        // A wave walks its tiles forwards on even steps and backwards on odd ones: a cache that is a little
        // larger than an L2 then finds the tiles it touched last in the previous step first in this one.
        const int tw0 = key0 + wave * TK;
        const int lim = min(len, key0 + ucap);                                  // end of the unit's live slots
        const int nt_w = tw0 < lim ? (lim - tw0 + NW * TK - 1) / (NW * TK) : 0;    // tiles of this wave that hold slots
        const bool rev = A.zigzag > 1 && (step & 1);
        if (nt_w > 0) { const int t0 = tw0 + (rev ? nt_w - 1 : 0) * NW * TK; issue_k(t0); issue_v(t0); }
        const int ticket = take_ticket();
        // FP8 cache, appending: the wave one of whose tiles holds the new slot quantises the new row (every 16-lane
        // row group the same row, so each lane gets the codes of its 8 elements and the row's scale) while the loads of
        // its first tile are on their way, and stores codes, scales and position into the cache.  In the tile that
        // holds the slot it replaces what the loads brought for it (the loads make no exception for the slot: a test
        // in their fast path cost 40 registers).
        uint2 qk_new = make_uint2(0, 0), qv_new = make_uint2(0, 0);
        float sk_new = 0.f, sv_new = 0.f;
        if constexpr (Q8) {
            if (new_slot >= key0 && new_slot < key0 + ucap && ((new_slot - key0) / TK) % NW == wave) {      // wave-uniform
                qk_new = quantize_row_e4m3<LPR>(*reinterpret_cast<const uint4*>(knew + c * 8), sk_new);
                qv_new = quantize_row_e4m3<LPR>(*reinterpret_cast<const uint4*>(vnew + c * 8), sv_new);
                if (!(VLC_DECODE_ABLATE & 8) && sub == 0) {
                    *reinterpret_cast<uint2*>(const_cast<uint8_t*>(K8) + (int64_t)new_slot * D + c * 8) = qk_new;
                    *reinterpret_cast<uint2*>(const_cast<uint8_t*>(V8) + (int64_t)new_slot * D + c * 8) = qv_new;
                    if (c == 0) {
                        const_cast<float*>(Ksc)[new_slot] = sk_new;
                        const_cast<float*>(Vsc)[new_slot] = sv_new;
                        A.dev.idx[idx_base + new_slot] = A.m + appended;
                    }
                }
            }
        }
#pragma unroll 1
        for (int i = 0; i < nt_w; ++i) {
            const int t0 = tw0 + (rev ? nt_w - 1 - i : i) * NW * TK;
            if (i > 0) { issue_k(t0); issue_v(t0); }
            if constexpr (Q8) {
                if (new_slot >= t0 && new_slot < t0 + TK) {         // wave-uniform: this is the wave that quantised the new row
                    const int rel = new_slot - t0;
#pragma unroll
                    for (int j = 0; j < NIT; ++j)
                        if (rel / KPI == j && rel % KPI == sub) { kb8[j] = qk_new; ksc[j] = sk_new; vb8[j] = qv_new; }
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk)
                        if (t0 + scol + 16 * kk == new_slot) vsc[kk] = sv_new;
                }
            }
            const bool full = (t0 + TK <= len);
            if (full) tile_body(std::true_type{}, t0); else tile_body(std::false_type{}, t0);
        }

        // The unit that holds the new slot also stores the new row into the cache.
        if (!(VLC_DECODE_ABLATE & 8) && !Q8 && appending && new_slot >= key0 && new_slot < key0 + ucap && wave == 0 && sub == 0) {
            T* kdst = const_cast<T*>(Kbase) + (int64_t)new_slot * D;
            T* vdst = const_cast<T*>(Vbase) + (int64_t)new_slot * D;
            *reinterpret_cast<uint4*>(kdst + c * EP) = *reinterpret_cast<const uint4*>(knew + c * EP);
            *reinterpret_cast<uint4*>(vdst + c * EP) = *reinterpret_cast<const uint4*>(vnew + c * EP);
            if (c == 0) A.dev.idx[idx_base + new_slot] = A.m + appended;
        }

#if VLC_DECODE_ABLATE & 2
        if (acc[0][0] == 1.2345f) Elem<T>::store(outp, acc[0][0]);     // keeps the accumulators alive; practically never taken
        if (mode && tid == 0) finish(ticket, il, n_layer);
        return true;
#endif
        // ---- sum the row groups of the wave, then merge the 4 waves through LDS
        if constexpr (LPR == 16) {
            // Four row groups = the four 16-lane rows of the wave.  Reduce-scatter with the lane-swap instructions
            // (v_permlane16_swap, v_permlane32_swap: vector-unit moves, no trip through the LDS queue): of four
            // accumulators x0..x3, row r ends up with the total of x_r, so four registers become one and every
            // lane has something to write.  swap16(a, b) = ([a.r0, b.r0, a.r2, b.r2], [a.r1, b.r1, a.r3, b.r3]),
            // swap32(a, b) = ([a.lo, b.lo], [a.hi, b.hi]).
            auto pair_sum16 = [](float a, float b) {
                const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
                return __uint_as_float(r[0]) + __uint_as_float(r[1]);       // [a.r0 + a.r1, b.r0 + b.r1, a.r2 + a.r3, b.r2 + b.r3]
            };
            auto pair_sum32 = [](float a, float b) {
                const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
                return __uint_as_float(r[0]) + __uint_as_float(r[1]);
            };
#pragma unroll
            for (int h = 0; h < G; ++h)
#pragma unroll
                for (int e = 0; e < EP; e += 4) {
                    const float tot = pair_sum32(pair_sum16(acc[h][e], acc[h][e + 1]), pair_sum16(acc[h][e + 2], acc[h][e + 3]));
                    sMerge[wave][h][c * EP + e + sub] = tot;                  // row `sub` holds the total of element e + sub
                }
        } else {
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
                for (int h = 0; h < G; ++h)
#pragma unroll
                    for (int e = 0; e < EP; ++e) acc[h][e] += __shfl_xor(acc[h][e], off, 64);
            if (sub == 0) {
#pragma unroll
                for (int h = 0; h < G; ++h)
#pragma unroll
                    for (int e = 0; e < EP; e += 4)
                        *reinterpret_cast<float4*>(&sMerge[wave][h][c * EP + e]) = make_float4(acc[h][e], acc[h][e + 1], acc[h][e + 2], acc[h][e + 3]);
            }
        }
        if (scol == 0) {
#pragma unroll
            for (int hh = 0; hh < HR; ++hh)
                if (srow * HR + hh < G) *reinterpret_cast<float2*>(&sMerge[wave][srow * HR + hh][D]) = make_float2(m_run[hh], l_run[hh]);
        }
        __syncthreads();
        // every thread merges two neighbouring output elements of one head: one weight per wave, one store
        float* part = A.dev.partials + (size_t)canon * G * DP;      // partials sit in the layer-major order
        for (int x = tid; x < G * D / 2; x += THREADS) {
            const int h = x / (D / 2), e = (x % (D / 2)) * 2;
            float2 ml[NW];
            float mt = -INFINITY;
#pragma unroll
            for (int wv = 0; wv < NW; ++wv) {
                ml[wv] = *reinterpret_cast<const float2*>(&sMerge[wv][h][D]);
                mt = fmaxf(mt, ml[wv].x);
            }
            float o0 = 0.f, o1 = 0.f, lt = 0.f;
#pragma unroll
            for (int wv = 0; wv < NW; ++wv) {
                const float wgt = (ml[wv].x > -INFINITY) ? exp2_fast(ml[wv].x - mt) : 0.f;
                const float2 ov = *reinterpret_cast<const float2*>(&sMerge[wv][h][e]);
                o0 = fmaf(ov.x, wgt, o0);
                o1 = fmaf(ov.y, wgt, o1);
                lt = fmaf(ml[wv].y, wgt, lt);
            }
            if (nu == 1) {
                const float inv = __builtin_amdgcn_rcpf(lt);        // within an ulp of the quotient: far inside the output's rounding
                store_pair(outp + h * D + e, o0 * inv, o1 * inv);
            } else if (A.merge_mode == 1) {
                store_agent2(part + h * DP + e, o0, o1);
                if (e == 0) store_agent2(part + h * DP + D, mt, lt);
            } else {
                *reinterpret_cast<float2*>(part + h * DP + e) = make_float2(o0, o1);
                if (e == 0) *reinterpret_cast<float2*>(part + h * DP + D) = make_float2(mt, lt);
            }
        }
        if (nu > 1 && A.merge_mode == 1) {
            // Publication of the partials.  They were written with device-scope stores, which go through to the
            // memory side of the XCDs' L2 caches.  Every thread first waits until its own stores have been
            // acknowledged (a workgroup barrier alone does not drain another wave's outstanding stores), then
            // the barrier orders all four waves before thread 0, and only then does thread 0 add to the row's
            // counter.  The unit that counts nu - 1 predecessors therefore finds every partial of the row in
            // memory; it reads them with device-scope loads, which do not hit a stale line of its own L2.
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            int32_t* counter = A.dev.counters + row_abs;
            if (tid == 0) sLast = (add_agent(counter, 1) == nu - 1) ? 1 : 0;
            __syncthreads();
            if (sLast) {
                merge_partials<T, D, G, true, THREADS>(A.dev.partials + (size_t)(canon - unit) * G * DP, outp, nu, tid);
                if (tid == 0) store_agent(counter, 0);
            }
        }
        if (mode && tid == 0) finish(ticket, il, n_layer);
        return true;
    };
    const bool more = process_unit(std::true_type{}, P, (int)blockIdx.x);
    if (over && blockIdx.x == 0 && tid == 0) set_sticky(P.dev.status, VLC_ERR_CAPACITY, -3, P.layer_begin, appended);
    if (!more) return;
    // A launch over a layer range runs at most one resident round of blocks, whatever the budgets turn out to be;
    // units beyond the grid are taken here, with the grid as stride.  Code inside a loop compiles worse (loop
    // invariants are hoisted and held in registers, which spills here), so a block's first unit, which is all
    // there is unless a layer range holds more units than the grid, stays outside the loop, and inside it the
    // parameters are read where they are used, through a copy of the kernel-argument pointer that the compiler
    // cannot see through.
    typedef const __attribute__((address_space(4))) DecodeParams* ParamsPtr;
#pragma unroll 1
    for (int w0 = (int)blockIdx.x + (int)gridDim.x;; w0 += (int)gridDim.x) {
        ParamsPtr Q = (ParamsPtr)__builtin_amdgcn_kernarg_segment_ptr();
        asm volatile("" : "+s"(Q));
        __syncthreads();                        // the previous unit's merge buffers are free again
        if (!process_unit(std::false_type{}, *Q, w0)) break;
    }
}

// Second kernel of merge mode 2: one block per (layer, request, KV head) row.  It runs after the attention
// kernel of the same call, so the append count it reads already includes this call's step.
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void decode_merge_kernel(DecodeParams P) {
    const int row = blockIdx.x;
    const int hkv = row % P.Hkv;
    const int b = (row / P.Hkv) % P.B;
    const int lr = row / (P.Hkv * P.B);
    const int bl = b * P.L + P.layer_begin + lr;
    const int kept = P.dev.kept[bl];
    if (kept == 0) return;
    const int len = kept + P.dev.appended[P.layer_begin];
    const int nbig = kept >> P.ub_shift;
    const int nu = nbig + ((len - (nbig << P.ub_shift) + (1 << P.us_shift) - 1) >> P.us_shift);
    if (nu == 1) return;
    T* outp = reinterpret_cast<T*>(P.out) + ((size_t)(lr * P.B + b) * P.Hq + (size_t)hkv * G) * D;
    const int w0 = P.wl.row_first[(size_t)bl * P.Hkv + hkv];
    merge_partials<T, D, G, false, 256>(P.dev.partials + (size_t)w0 * G * (D + 2), outp, nu, threadIdx.x);
}

template <typename T, int D, int G>
hipError_t launch_one(const DecodeParams& P, int grid, int rows, hipStream_t st) {
    bool done = false;
    if constexpr (IsBf16<T>::value) {
        if (P.kv_fp8) {
            decode_kernel<T, D, G, true><<<grid, 256, 0, st>>>(P);
            done = true;
        }
    }
    if (!done) decode_kernel<T, D, G, false><<<grid, 256, 0, st>>>(P);
    if (P.merge_mode == 2) decode_merge_kernel<T, D, G><<<rows, 256, 0, st>>>(P);
    return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_g(const DecodeParams& P, int g, int grid, int rows, hipStream_t st) {
    switch (g) {
        case 1: return launch_one<T, D, 1>(P, grid, rows, st);
        case 2: return launch_one<T, D, 2>(P, grid, rows, st);
        case 3: return launch_one<T, D, 3>(P, grid, rows, st);
        case 4: return launch_one<T, D, 4>(P, grid, rows, st);
        case 5: return launch_one<T, D, 5>(P, grid, rows, st);
        case 6: return launch_one<T, D, 6>(P, grid, rows, st);
        case 7: return launch_one<T, D, 7>(P, grid, rows, st);
        case 8: return launch_one<T, D, 8>(P, grid, rows, st);
    }
    return hipErrorInvalidValue;
}

int log2i(int v) {
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

}  // namespace

hipError_t launch_decode(const DecodeArgs& a) {
    const vlc_cache& c = *a.c;
    const vlc_shape& s = c.shape;
    DecodeParams P;
    P.q = a.q; P.k_new = a.k_new; P.v_new = a.v_new; P.out = a.out; P.sm_scale = a.sm_scale;
    P.dev = c.dev;
    // A launch over all layers walks list 1 (coarser units; by size class once the cache has more units than
    // fit the chip at once, so that the blocks dispatched last are short), a launch over a layer range list 0
    // (fine units in layer order, so that one layer of the batch still fills the chip).
    const bool all_layers = a.layer_begin == 0 && a.n_layers == s.L;
    P.wl = c.dev.list[all_layers ? 1 : 0];
    P.ub_shift = log2i(P.wl.u_big); P.us_shift = log2i(P.wl.u_small);
    P.B = s.B; P.L = s.L; P.Hq = s.Hq; P.Hkv = s.Hkv; P.m = s.m;
    P.layer_begin = a.layer_begin; P.n_layers = a.n_layers; P.T_max = c.T_max;
    P.append_mode = a.k_new ? 1 : 0;
    P.default_scale = 1.0f / sqrtf((float)s.d);
    P.merge_mode = c.opt.decode_merge;
    P.zigzag = c.opt.decode_zigzag;
    P.kv_fp8 = c.kv_fp8 ? 1 : 0;
    const int rows = a.n_layers * s.B * s.Hkv;
    // Upper bound on the block-units of the layer range: every row at the full prompt length, and never more
    // than the whole work list.  A launch over a layer range is capped at one resident round of blocks (3 per
    // CU); its blocks walk the slice with the grid as stride.  The budgets, and with them the true number of
    // units, are known on the device only.
    int64_t grid = (int64_t)rows * (((int64_t)s.m + c.T_max) / P.wl.u_small + 1);
    if (grid > P.wl.cap) grid = P.wl.cap;
    if (!all_layers && grid > 3 * (int64_t)c.num_cus) grid = 3 * (int64_t)c.num_cus;
    if (grid < 1) grid = 1;
    const int g = s.Hq / s.Hkv;
    if (s.dtype == VLC_F32)
        return s.d == 64 ? launch_g<float, 64>(P, g, (int)grid, rows, a.stream) : launch_g<float, 128>(P, g, (int)grid, rows, a.stream);
    return s.d == 64 ? launch_g<bf16_t, 64>(P, g, (int)grid, rows, a.stream) : launch_g<bf16_t, 128>(P, g, (int)grid, rows, a.stream);
}

}  // namespace vlc
