// Token eviction: per-(request, layer, KV head) TopK of the accumulated post-vision scores
// (paper Sec. 2.2 top-k set, Sec. 4.2) and the copy of the surviving K/V rows into the contiguous,
// ragged per-layer cache (App. A.4).  Three kernels on one stream:
//   layout : validates k[b][l], prefix-sums the slab offsets of a request's layers
//   select : radix-select of the k-th largest score over keys held in registers, then an ordered
//            compaction that emits the kept positions ascending (ties to the lower position)
//   gather : one block per work-list unit streams the kept rows of K and V into the slabs
#include <stdlib.h>

#include "common.h"
#include "internal.h"

namespace vlc {
namespace {

// One block for the whole batch (B*L is a few hundred entries): clears the sticky status, validates
// the budgets, lays the slabs of each request out back to back, and builds the decode work list.
// Everything is staged in LDS so that the serial prefix sums never wait on global memory.
constexpr int kLayoutMaxBL = 2048;     // B*L entries staged in LDS (the shape check admits no larger batch)

struct LayoutArgs {
    const int32_t* k;          // [B, L] budgets as the caller passed them
    const int32_t* lens;       // [B, 2] per-request (m, tau), or null
    int B, L, Hkv, m, tau, d, T_max;
    int64_t slots_per_request;
};

// Units of a row with `kk` kept slots in a list that cuts rows into u_big units followed by u_small units:
// big = whole u_big units, live = small units that hold kept slots, total = all units including those
// that only hold append reserve.  A rejected row (kk == 0) has one unit, which only carries the marker.
struct RowUnits { int big, live, total; };
__device__ __forceinline__ RowUnits row_units(int kk, int T_max, int ub, int us) {
    if (kk == 0) return RowUnits{0, 0, 1};
    const int big = kk / ub, rem = kk - big * ub;
    return RowUnits{big, (rem + us - 1) / us, big + (rem + T_max + us - 1) / us};
}

// Runs in TWO blocks of NT threads (every thread of a block must enter): the lists are independent of each other
// once budgets and slab offsets are known, and those are cheap, so both blocks derive them and part 0 writes them
// out, zeroes the counters and builds the layer-ordered list, while part 1 builds the list of the all-layer launches
// (and the gather's, when that is a list of its own).  Errors are reported by part 0.
template <int NT>
__device__ void layout_body(const LayoutArgs& a, CacheDev dev, int part) {
    const int32_t* __restrict__ k = a.k;
    const int32_t* __restrict__ lens = a.lens;
    const int B = a.B, L = a.L, Hkv = a.Hkv, m = a.m, tau = a.tau, d = a.d, T_max = a.T_max;
    const int64_t slots_per_request = a.slots_per_request;
    __shared__ int32_t sKept[kLayoutMaxBL];
    __shared__ int32_t sFirst[kLayoutMaxBL];        // first unit of (b, l), kv head 0, in canon order
    __shared__ int64_t sSlot[kLayoutMaxBL];
    __shared__ int64_t sScan[NT], sScan2[NT];
    __shared__ int32_t sBigFirst[kLayoutMaxBL], sLiveFirst[kLayoutMaxBL], sResFirst[kLayoutMaxBL];
    __shared__ int sTotals[2];
    __shared__ int sBad;
    __shared__ uint32_t sSort[kLayoutMaxBL];        // (request, layer) entries in the order of the size-class walk's second class
    const int tid = threadIdx.x;
    const int BL = B * L;
    const bool first = part == 0;               // the part that owns everything but the lists of part 1
    if (first && tid < 4) dev.status[tid] = 0;
    __syncthreads();
    // per-request lengths: checked here (the only place with an error channel), kept in the cache
    if (first) {
        for (int b = tid; b < B; b += NT) {
            int mb = m, tb = tau;
            if (lens) {
                mb = lens[2 * b]; tb = lens[2 * b + 1];
                if (mb < 1 || mb > m || tb < 1 || tb > tau || tb > mb) set_sticky(dev.status, VLC_ERR_INVALID_ARG, b, -2, mb);
            }
            const ReqLen rl = request_len(lens, b, m, tau);
            dev.lens[2 * b] = rl.m; dev.lens[2 * b + 1] = rl.tau;
        }
    }
    for (int x = tid; x < BL; x += NT) {
        int kk = k[x];
        if (kk < 1 || kk > request_len(lens, x / L, m, tau).m) {
            if (first) set_sticky(dev.status, VLC_ERR_INVALID_ARG, x / L, x % L, kk);
            kk = 0;
        }
        sKept[x] = kk;
    }
    if (first) {
        for (int x = tid; x < BL * Hkv; x += NT) dev.counters[x] = 0;
        for (int x = tid; x < L; x += NT) dev.appended[x] = 0;          // decode starts at step 0
        for (int x = tid; x <= L; x += NT) dev.readers[x * kReaderStride] = 0;
    }
    __syncthreads();
    // slab offsets, one thread per request; a request whose budgets do not fit keeps nothing
    for (int b = tid; b < B; b += NT) {
        int64_t acc = 0;
        for (int l = 0; l < L; ++l) acc += sKept[b * L + l] + T_max;
        const bool over = acc > slots_per_request;
        if (over && first) set_sticky(dev.status, VLC_ERR_CAPACITY, b, -1, (int)min(acc, (int64_t)INT32_MAX));
        acc = 0;
        for (int l = 0; l < L; ++l) {
            if (over) sKept[b * L + l] = 0;
            sSlot[b * L + l] = (int64_t)b * slots_per_request + acc;
            acc += sKept[b * L + l] + T_max;
        }
    }
    __syncthreads();
    if (first) {
        for (int x = tid; x < BL; x += NT) {
            dev.kept[x] = sKept[x];
            dev.slot_off[x] = sSlot[x];
        }
    }
    // The work lists.  Units per row, exclusive prefix over (layer, request) in that order, for all units
    // and separately for the u_big units and the live small ones (the size-class order).  Each thread sums
    // a run of consecutive entries, the run totals are scanned across the block, then every thread
    // walks its run again from its offset.
    // (one instance of the code per list, so that each list's description stays in scalar registers)
    auto build_list = [&](const WorkList& wl) {
        const int ub = wl.u_big, us = wl.u_small;
        __syncthreads();                        // the staging arrays of the previous list are no longer read
        if (tid == 0) sBad = 0;
        const int per = (BL + NT - 1) / NT;
        const int y0 = tid * per, y1 = min(BL, y0 + per);
        int64_t run = 0, run2 = 0;              // run2 packs (u_big units << 32) | live small units
        for (int y = y0; y < y1; ++y) {
            const RowUnits ru = row_units(sKept[(y % B) * L + y / B], T_max, ub, us);
            run += (int64_t)ru.total * Hkv;
            run2 += ((int64_t)ru.big * Hkv << 32) | (int64_t)(ru.live * Hkv);
        }
        // inclusive scan of the run totals: inside each wave with lane shifts, then across the waves through LDS
        int64_t inc = run, inc2 = run2;
        const int lane = tid & 63, wv = tid >> 6;
        for (int o = 1; o < 64; o <<= 1) {
            const int64_t v = (int64_t)__shfl_up((long long)inc, o, 64), v2 = (int64_t)__shfl_up((long long)inc2, o, 64);
            if (lane >= o) { inc += v; inc2 += v2; }
        }
        if (lane == 63) { sScan[wv] = inc; sScan2[wv] = inc2; }
        __syncthreads();
        int64_t total = 0, total2 = 0;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) {
            const int64_t t = sScan[w], t2 = sScan2[w];
            if (w < wv) { inc += t; inc2 += t2; }
            total += t; total2 += t2;
        }
        if (tid == 0) { sTotals[0] = (int)(total2 >> 32); sTotals[1] = (int)(total2 & 0xffffffff); }
        if (total > wl.cap) {                   // cannot happen for budgets that passed the capacity check
            if (tid == 0) {
                set_sticky(dev.status, VLC_ERR_CAPACITY, -1, -1, -1);
                sBad = 1;
            }
            for (int l = tid; l <= L + 1; l += NT) wl.layer_start[l] = 0;
        } else {
            int64_t acc = inc - run, acc2 = inc2 - run2;
            for (int y = y0; y < y1; ++y) {
                const int l = y / B, b = y % B;
                const RowUnits ru = row_units(sKept[b * L + l], T_max, ub, us);
                if (b == 0) wl.layer_start[l] = (int)acc;
                sFirst[b * L + l] = (int)acc;
                sBigFirst[b * L + l] = (int)(acc2 >> 32);
                sLiveFirst[b * L + l] = (int)(acc2 & 0xffffffff);
                sResFirst[b * L + l] = (int)acc - (int)(acc2 >> 32) - (int)(acc2 & 0xffffffff);    // reserve units listed before this entry's
                acc += (int64_t)ru.total * Hkv;
                acc2 += ((int64_t)ru.big * Hkv << 32) | (int64_t)(ru.live * Hkv);
            }
            if (tid == 0) wl.layer_start[L] = (int)total;
        }
        __syncthreads();
        if (sBad) return;
        // Size-class order, second class (the units that are partly filled): longest first, so that the blocks
        // dispatched last, which decide when the launch ends, are the shortest.  All rows of a (request, layer) entry
        // have the same fill, so the entries are sorted (by the slots their rows hold beyond whole u_big units,
        // descending, ties in list order: a bitonic sort in LDS of one word per entry, u_big - 1 - fill above the
        // entry's list position) and the class's positions are the prefix sums in that order.
        if (wl.by_size) {
            static_assert(kLayoutMaxBL <= 2048 && kMaxUnitSlots <= 2048, "11 bits each for the fill and the entry");
            int n2 = 1;
            while (n2 < BL) n2 <<= 1;
            for (int y = tid; y < n2; y += NT) {
                uint32_t v = 0xffffffffu;                       // padding sorts last
                if (y < BL) {
                    const int kk = sKept[(y % B) * L + y / B];
                    v = ((uint32_t)(ub - 1 - (kk - (kk / ub) * ub)) << 11) | (uint32_t)y;
                }
                sSort[y] = v;
            }
            __syncthreads();
            for (int kb = 2; kb <= n2; kb <<= 1)
                for (int j = kb >> 1; j > 0; j >>= 1) {
                    for (int x = tid; x < n2; x += NT) {
                        const int p = x ^ j;
                        if (p > x) {
                            const uint32_t va = sSort[x], vb = sSort[p];
                            if ((va > vb) == ((x & kb) == 0)) { sSort[x] = vb; sSort[p] = va; }
                        }
                    }
                    __syncthreads();
                }
            const int per2 = (BL + NT - 1) / NT;
            const int r0 = tid * per2, r1 = min(BL, r0 + per2);
            int runl = 0;
            for (int r = r0; r < r1; ++r) {
                const int y = (int)(sSort[r] & 2047u);
                runl += row_units(sKept[(y % B) * L + y / B], T_max, ub, us).live * Hkv;
            }
            int incl = runl;
            for (int o = 1; o < 64; o <<= 1) {
                const int v = __shfl_up(incl, o, 64);
                if (lane >= o) incl += v;
            }
            if (lane == 63) sScan[wv] = incl;
            __syncthreads();
#pragma unroll
            for (int w = 0; w < NT / 64; ++w)
                if (w < wv) incl += (int)sScan[w];
            int accl = incl - runl;
            for (int r = r0; r < r1; ++r) {
                const int y = (int)(sSort[r] & 2047u), bl = (y % B) * L + y / B;
                sLiveFirst[bl] = accl;
                accl += row_units(sKept[bl], T_max, ub, us).live * Hkv;
            }
            __syncthreads();
        }
        const int n_big = sTotals[0], n_live = sTotals[1];
        if (tid == 0) wl.layer_start[L + 1] = n_big;               // decode reverses the walk over the u_big units on odd steps
        for (int x = tid; x < BL * Hkv; x += NT) {
            const int h = x % Hkv, bl = x / Hkv, b = bl / L, l = bl % L;
            const int kk = sKept[bl];
            const RowUnits ru = row_units(kk, T_max, ub, us);
            const int nres = ru.total - ru.big - ru.live;
            const int cap = kk + T_max;
            const int64_t so = sSlot[bl];
            WorkItem it;
            it.row_abs = x; it.kept = kk; it.b = b; it.l = l; it.hkv = h; it.pad[0] = 0; it.pad[1] = 0;
            it.layer_units = (l + 1 < L ? sFirst[l + 1] : (int)total) - sFirst[l];      // request 0 starts each layer
            it.kbase = ((so * 2 * Hkv) + (int64_t)h * cap) * d;
            it.idx_base = so * Hkv + (int64_t)h * cap;
            const int w0 = sFirst[bl] + h * ru.total;
            // units of the third class that precede this row's in the list (all units before it minus big and live)
            const int res0 = n_big + n_live + sResFirst[bl] + h * nres;
            wl.row_first[x] = w0;
            for (int u = 0; u < ru.total; ++u) {
                it.unit = u;
                it.key0 = u < ru.big ? u * ub : ru.big * ub + (u - ru.big) * us;
                it.ucap = u < ru.big ? ub : us;
                it.canon = w0 + u;
                int ws = w0 + u;
                if (wl.by_size) {
                    if (u < ru.big) ws = sBigFirst[bl] + h * ru.big + u;
                    else if (u < ru.big + ru.live) ws = n_big + sLiveFirst[bl] + h * ru.live + (u - ru.big);
                    else ws = res0 + (u - ru.big - ru.live);
                }
                wl.items[ws] = it;
            }
        }
    };
    if (first) {
        build_list(dev.list[0]);
    } else {
        build_list(dev.list[1]);
        if (dev.list[2].items != dev.list[0].items && dev.list[2].items != dev.list[1].items) build_list(dev.list[2]);   // else the gather shares a decode list
    }
    static_assert(kNumLists == 3, "one call per list");
}

__global__ __launch_bounds__(256) void layout_kernel(LayoutArgs a, CacheDev dev) { layout_body<256>(a, dev, (int)blockIdx.x); }   // two blocks

// Order-preserving map float -> uint32 (larger float, larger key).
__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kSelThreads = 512;
constexpr int kSelWaves = kSelThreads / 64;

// Visit the candidates of this wave's segment [j0, j1): f(position, key, inside).  Every lane calls f
// the same number of times, so f may hold wave-wide ballots.  With NK > 0 the keys come from the
// registers filled at the start of the kernel, else they are streamed from memory four at a time.
template <int NK, typename F>
__device__ __forceinline__ void for_keys(const uint32_t (&key)[NK > 0 ? NK : 1], const float* __restrict__ s,
                                         int j0, int j1, int lane, F f) {
    if constexpr (NK > 0) {
#pragma unroll
        for (int i = 0; i < NK; ++i) {
            const int j = j0 + i * 64 + lane;
            f(j, key[i], j < j1);
        }
    } else {
        for (int jb = j0; jb < j1; jb += 4 * 64) {
            float v[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) v[x] = s[min(jb + x * 64 + lane, j1 - 1)];    // unconditional: no wait between loads
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int j = jb + x * 64 + lane;
                f(j, order_key(v[x]), j < j1);
            }
        }
    }
}

// One block per (request, layer, KV head) row.  Each wave owns a contiguous segment of the row and,
// when the segment fits NK values per lane, keeps its keys in registers: the scores are then read
// from memory once for the four digit passes, the count and the ordered emission.
// The digit histogram is kept in SUB interleaved copies: lane l adds into copy l % SUB, so that lanes of a
// wave with equal digits do not all serialise on one LDS word.
// HIT = false: emits the kept positions into the cache (and idx_out).  HIT = true (Def. 3.1): `scores` are the
// decode-query attention, the top-k set S* is found the same way with the cache's own budget and no
// recent window, and instead of emitting it the block counts how many positions the cache already holds
// lie in S*: hits_out[row] = |kept ∩ S*|.
// FOLD = true (small batches, where a one-block kernel and its launch gap show): the grid has one block more
// than there are rows, and block 0 does the layout kernel's work while the others select.  A selecting
// block then cannot read the layout's results: it derives its row's budget and slab offset from the caller's
// budgets by the layout's own rules (a budget outside [1, m_b] keeps nothing; a request whose slabs do not
// fit keeps nothing).
template <int NK, bool HIT, bool FOLD>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ scores, CacheDev dev,
                                                             int L, int Hkv, int m, int ragged, int T_max, int n_recent,
                                                             int recent_num, int recent_den,
                                                             int32_t* __restrict__ idx_out,
                                                             int32_t* __restrict__ hits_out, float* __restrict__ rate_out,
                                                             LayoutArgs la) {
    static_assert(!(HIT && FOLD), "the hit count reads a cache that is already laid out");
    // copies of the histogram: short rows have few adds, so the clear and the sum dominate (4); long rows measured
    // on the 7B shape with m = 10368: 4 copies 47.5 us, 8: 44.1, 16: 68.5, 32: 94.7 (with more copies the bank of an
    // add depends less on its digit, and the lanes of a wave crowd into fewer banks)
    constexpr int kSelSub = NK == 8 ? 4 : 8;
    __shared__ __align__(16) uint32_t hist[256 * kSelSub];
    __shared__ uint32_t sel_bin, sel_above;
    __shared__ uint32_t cnt_gt[kSelWaves], cnt_eq[kSelWaves];
    if constexpr (FOLD) {
        if (blockIdx.x < 2) {                        // first, so that they start with the first rows
            layout_body<kSelThreads>(la, dev, (int)blockIdx.x);
            return;
        }
    }
    const int row = FOLD ? (int)blockIdx.x - 2 : (int)blockIdx.x;
    const int hkv = row % Hkv, bl = row / Hkv;
    int kk, mb;
    int64_t slot_off;
    if constexpr (FOLD) {
        __shared__ long long sSum[2 * kSelWaves];
        const int b = bl / L, l = bl % L;
        kk = la.k[bl];                                 // requested with the loads of the sum, not after its barrier
        mb = request_len(la.lens, b, m, la.tau).m;
        long long tot = 0, before = 0;
        for (int x = threadIdx.x; x < L; x += kSelThreads) {
            int v = la.k[b * L + x];
            if (v < 1 || v > mb) v = 0;
            tot += v + T_max;
            if (x < l) before += v + T_max;
        }
        for (int o = 32; o >= 1; o >>= 1) {
            tot += __shfl_xor(tot, o, 64);
            before += __shfl_xor(before, o, 64);
        }
        if ((threadIdx.x & 63) == 0) { sSum[2 * (threadIdx.x >> 6)] = tot; sSum[2 * (threadIdx.x >> 6) + 1] = before; }
        __syncthreads();
        tot = 0; before = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) { tot += sSum[2 * w]; before += sSum[2 * w + 1]; }
        if (kk < 1 || kk > mb || tot > la.slots_per_request) kk = 0;
        slot_off = (int64_t)b * la.slots_per_request + before;
    } else {
        kk = dev.kept[bl];
        mb = ragged ? dev.lens[2 * (bl / L)] : m;     // this request's prompt length (validated by the layout kernel)
        slot_off = dev.slot_off[bl];
    }
    if (kk == 0) {
        if (HIT && threadIdx.x == 0) {
            hits_out[row] = 0;
            if (rate_out) rate_out[row] = 0.f;
        }
        return;
    }
    // forced recent window: a count, or a fraction of this layer's budget (Sec. 5: 10 % of the budget)
    const int rcnt = HIT ? 0 : recent_den > 0 ? (int)((int64_t)kk * recent_num / recent_den) : min(max(n_recent, 0), kk);
    const int need = kk - rcnt;                // picked by score among positions [0, mc)
    const int mc = mb - rcnt;
    const int cap = kk + T_max;
    const float* s = scores + (size_t)row * m;
    int32_t* out = dev.idx + slot_off * Hkv + (int64_t)hkv * cap;
    int32_t* out2 = idx_out ? idx_out + (size_t)row * m : nullptr;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seg = ((mc + kSelWaves - 1) / kSelWaves + 63) & ~63;
    const int j0 = wave * seg, j1 = min(mc, j0 + seg);

    uint32_t key[NK > 0 ? NK : 1];
    if constexpr (NK > 0) {
#pragma unroll
        for (int i = 0; i < NK; ++i) {
            const int j = j0 + i * 64 + lane;
            // the address is clamped rather than the load predicated, so that the NK loads of a lane
            // are all in flight together (a predicated load is followed by a wait for its value)
            const uint32_t u = order_key(s[max(0, min(j, mc - 1))]);
            key[i] = j < j1 ? u : 0u;
        }
    }

    // The keys of a row usually share their leading bits (positive scores within a few binades), and a
    // digit taken from shared bits would send every lane's LDS atomic to one or two bins.  The digit
    // passes therefore start at the highest bit in which two keys of the row differ.
    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)need;
    if (need > 0) {
        uint32_t all_and = 0xffffffffu, all_or = 0u;
        for_keys<NK>(key, s, j0, j1, lane, [&](int, uint32_t u, bool in) {
            if (in) { all_and &= u; all_or |= u; }
        });
        for (int o = 32; o >= 1; o >>= 1) {
            all_and &= (uint32_t)__shfl_xor((int)all_and, o, 64);
            all_or |= (uint32_t)__shfl_xor((int)all_or, o, 64);
        }
        if (lane == 0) { cnt_gt[wave] = all_and; cnt_eq[wave] = all_or; }
        __syncthreads();
        all_and = 0xffffffffu; all_or = 0u;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) { all_and &= cnt_gt[w]; all_or |= cnt_eq[w]; }
        __syncthreads();
        const uint32_t diff = all_and ^ all_or;
        int bits_left = diff ? 32 - __clz((int)diff) : 0;          // low bits still to be resolved
        mask = bits_left >= 32 ? 0u : ~((1u << bits_left) - 1u);
        prefix = all_or & mask;
        while (bits_left > 0) {
            const int width = min(8, bits_left);
            const int shift = bits_left - width;
            const uint32_t dmask = (1u << width) - 1u;
            for (int x = tid; x < 256 * kSelSub / 4; x += kSelThreads)
                reinterpret_cast<uint4*>(hist)[x] = make_uint4(0, 0, 0, 0);
            __syncthreads();
            for_keys<NK>(key, s, j0, j1, lane, [&](int, uint32_t u, bool in) {
                if (in && (u & mask) == prefix) atomicAdd(&hist[((u >> shift) & dmask) * kSelSub + (lane & (kSelSub - 1))], 1u);
            });
            __syncthreads();
            if (wave == 0) {
                // lane i owns bins 4i..4i+3; find the highest bin whose count, added to everything
                // above it, reaches `remaining`
                uint32_t c[4] = {0, 0, 0, 0};
#pragma unroll
                for (int q = 0; q < kSelSub; ++q) {              // the lane's 4 bins x kSelSub copies are 4 kSelSub consecutive words
                    const uint4 h4 = reinterpret_cast<const uint4*>(hist)[lane * kSelSub + q];
                    const uint32_t w[4] = {h4.x, h4.y, h4.z, h4.w};
#pragma unroll
                    for (int y = 0; y < 4; ++y) c[(q * 4 + y) / kSelSub] += w[y];
                }
                const uint32_t tot = c[0] + c[1] + c[2] + c[3];
                uint32_t suf = tot;             // inclusive suffix sum over lanes >= this one
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t v = __shfl_down(suf, o, 64);
                    if (lane + o < 64) suf += v;
                }
                uint32_t above = suf - tot;
                if (above < remaining && remaining <= above + tot) {
#pragma unroll
                    for (int x = 3; x >= 0; --x) {
                        if (above + c[x] >= remaining) { sel_bin = lane * 4 + x; sel_above = above; break; }
                        above += c[x];
                    }
                }
            }
            __syncthreads();
            prefix |= sel_bin << shift;
            mask |= dmask << shift;
            remaining -= sel_above;            // those above are all kept; keep looking inside the bin
            bits_left = shift;
            __syncthreads();
        }
    }
    // `prefix` is now the key of the need-th largest candidate; `remaining` of the candidates equal
    // to it are kept, lowest positions first.
    uint32_t gt = 0, eq = 0;
    if (need > 0) {
        for_keys<NK>(key, s, j0, j1, lane, [&](int, uint32_t u, bool in) {
            gt += (in && u > prefix) ? 1u : 0u;
            eq += (in && u == prefix) ? 1u : 0u;
        });
        gt = wave_allreduce_sum_u32(gt);
        eq = wave_allreduce_sum_u32(eq);
    }
    if (lane == 0) { cnt_gt[wave] = gt; cnt_eq[wave] = eq; }
    __syncthreads();
    if constexpr (HIT) {
        // position of the last candidate equal to the k-th key that S* still takes (ties go to the
        // lower position); then a kept position is a hit if its key is larger, or equal and not beyond it
        uint32_t eq_run = 0;
        for (int w = 0; w < wave; ++w) eq_run += cnt_eq[w];
        const unsigned long long lt_mask = (1ull << lane) - 1ull;
        for_keys<NK>(key, s, j0, j1, lane, [&](int j, uint32_t u, bool in) {
            const bool is_eq = in && (u == prefix);
            const unsigned long long be = __ballot(is_eq);
            if (is_eq && eq_run + (uint32_t)__popcll(be & lt_mask) == remaining - 1) sel_bin = (uint32_t)j;
            eq_run += (uint32_t)__popcll(be);
        });
        __syncthreads();
        const int eq_cut = (int)sel_bin;
        uint32_t hits = 0;
        for (int r = tid; r < kk; r += kSelThreads) {
            const int j = out[r];
            const uint32_t u = order_key(s[j]);
            hits += (u > prefix || (u == prefix && j <= eq_cut)) ? 1u : 0u;
        }
        hits = wave_allreduce_sum_u32(hits);
        if (lane == 0) cnt_gt[wave] = hits;
        __syncthreads();
        if (tid == 0) {
            uint32_t tot = 0;
            for (int w = 0; w < kSelWaves; ++w) tot += cnt_gt[w];
            hits_out[row] = (int32_t)tot;
            if (rate_out) rate_out[row] = (float)tot / (float)kk;
        }
        return;
    }
    if (need > 0) {
        uint32_t gt_run = 0, eq_run = 0;
        for (int w = 0; w < wave; ++w) { gt_run += cnt_gt[w]; eq_run += cnt_eq[w]; }
        const unsigned long long lt_mask = (1ull << lane) - 1ull;
        for_keys<NK>(key, s, j0, j1, lane, [&](int j, uint32_t u, bool in) {
            const bool is_gt = in && (u > prefix);
            const bool is_eq = in && (u == prefix);
            const unsigned long long bg = __ballot(is_gt), be = __ballot(is_eq);
            const uint32_t eq_rank = eq_run + (uint32_t)__popcll(be & lt_mask);
            const bool take = is_gt || (is_eq && eq_rank < remaining);
            const unsigned long long bs = __ballot(take);
            if (take) {
                const uint32_t pos = gt_run + min(eq_run, remaining) + (uint32_t)__popcll(bs & lt_mask);
                out[pos] = j;
                if (out2) out2[pos] = j;
            }
            gt_run += (uint32_t)__popcll(bg);
            eq_run += (uint32_t)__popcll(be);
        });
    }
    for (int x = tid; x < rcnt; x += kSelThreads) {     // forced recent window
        out[need + x] = mc + x;
        if (out2) out2[need + x] = mc + x;
    }
}

// `parts` blocks per unit of the gather's work list (up to kGatherUnit rows of one (request, layer, KV head) row),
// each moving an equal share of it.  The grid is a multiple of the list's capacity, so it
// follows the budgets that fit the arena rather than rows * m, and surplus blocks leave after two loads.  Each lane moves 16 bytes of one K row and
// one V row per pass; the position of the next row is fetched before the stores are issued.  More
// rows in flight per lane measured slower on every shape (the gathered reads are 256-byte pieces at
// random DRAM pages; eight blocks per CU already keep enough of them outstanding).
template <int ROWBYTES>
__global__ __launch_bounds__(256) void gather_kernel(const char* __restrict__ k_full, const char* __restrict__ v_full,
                                                     CacheDev dev, int L, int Hkv, int m, int T_max,
                                                     int elem_bytes, int parts) {
    constexpr int LPR = ROWBYTES / 16;          // lanes per row
    constexpr int RPB = 256 / LPR;              // rows per block pass
    const WorkList wl = dev.list[2];
    const int w = blockIdx.x / parts, part = blockIdx.x % parts;
    const WorkItem it = wl.items[w];            // the grid never exceeds the list's capacity
    if (w >= wl.layer_start[L]) return;
    const int kk = it.kept, key0 = it.key0;
    if (kk == 0 || key0 >= kk) return;          // rejected row, or a unit reserved for appends
    const int span = it.ucap / parts;           // a block moves one of `parts` equal shares of the unit
    const int r_begin = key0 + part * span;
    const int r_end = min(kk, r_begin + span);
    if (r_begin >= r_end) return;
    const int cap = kk + T_max;
    uint4* kd = reinterpret_cast<uint4*>(dev.kv + it.kbase * elem_bytes);
    uint4* vd = kd + (int64_t)Hkv * cap * LPR;
    const uint4* ks = reinterpret_cast<const uint4*>(k_full + (size_t)it.row_abs * m * ROWBYTES);
    const uint4* vs = reinterpret_cast<const uint4*>(v_full + (size_t)it.row_abs * m * ROWBYTES);
    const int32_t* idx = dev.idx + it.idx_base;
    const int c = threadIdx.x % LPR, sub = threadIdx.x / LPR;
    int r = r_begin + sub;
    int32_t jn = r < r_end ? idx[r] : 0;
    for (; r < r_end; r += RPB) {
        const uint4 a = ks[(int64_t)jn * LPR + c];
        const uint4 b = vs[(int64_t)jn * LPR + c];
        jn = r + RPB < r_end ? idx[r + RPB] : 0;
        kd[(int64_t)r * LPR + c] = a;
        vd[(int64_t)r * LPR + c] = b;
    }
}

// The gather for an FP8 cache (bf16 source rows of D elements): same decomposition, each row is
// quantised on the way (one fp32 scale per row, stored by the row's first lane).
template <int D>
__global__ __launch_bounds__(256) void gather_fp8_kernel(const char* __restrict__ k_full, const char* __restrict__ v_full,
                                                         CacheDev dev, int L, int Hkv, int m, int T_max) {
    constexpr int LPR = D / 8;                  // lanes per row: 8 bf16 values (16 bytes) each
    constexpr int RPB = 256 / LPR;
    const WorkList wl = dev.list[2];
    const int w = blockIdx.x;
    const WorkItem it = wl.items[w];
    if (w >= wl.layer_start[L]) return;
    const int kk = it.kept, key0 = it.key0;
    if (kk == 0 || key0 >= kk) return;
    const int r_end = min(kk, key0 + it.ucap);
    const int cap = kk + T_max;
    uint2* kd = reinterpret_cast<uint2*>(dev.kv + it.kbase);                     // one byte per element
    uint2* vd = kd + (int64_t)Hkv * cap * LPR;
    float* ksc = dev.scales + it.kbase / D;
    float* vsc = ksc + (int64_t)Hkv * cap;
    const uint4* ks = reinterpret_cast<const uint4*>(k_full + (size_t)it.row_abs * m * D * 2);
    const uint4* vs = reinterpret_cast<const uint4*>(v_full + (size_t)it.row_abs * m * D * 2);
    const int32_t* idx = dev.idx + it.idx_base;
    const int c = threadIdx.x % LPR, sub = threadIdx.x / LPR;
    // every lane of a row group runs the same number of passes (the reductions are group-wide)
    for (int r0 = key0; r0 < r_end; r0 += RPB) {
        const int r = r0 + sub;
        const bool live = r < r_end;
        const int64_t j = live ? idx[r] : idx[r_end - 1];
        const uint4 a = ks[j * LPR + c];
        const uint4 b = vs[j * LPR + c];
        float sa, sb;
        const uint2 qa = quantize_row_e4m3<LPR>(a, sa);
        const uint2 qb = quantize_row_e4m3<LPR>(b, sb);
        if (live) {
            kd[(int64_t)r * LPR + c] = qa;
            vd[(int64_t)r * LPR + c] = qb;
            if (c == 0) { ksc[r] = sa; vsc[r] = sb; }
        }
    }
}

}  // namespace

hipError_t launch_topk_compact(const vlc_cache& c, const int32_t* lens, const float* scores, const int32_t* k, int32_t n_recent,
                               int32_t recent_num, int32_t recent_den, const void* k_full, const void* v_full,
                               int32_t* idx_out, hipStream_t st) {
    const vlc_shape& s = c.shape;
    const int rows = s.B * s.L * s.Hkv;
    LayoutArgs la{k, lens, s.B, s.L, s.Hkv, s.m, s.tau, s.d, c.T_max, c.slots_per_request};
    // values per lane of a wave's segment (an eighth of the row, rounded up to whole wave loads)
    const int per_lane = (((s.m + kSelWaves - 1) / kSelWaves + 63) / 64);
    // the layout as one more block of the selection (short rows only), or as a kernel of its own
    const bool fold = c.opt.select_fold == 2 && per_lane <= 8;
    if (!fold) layout_kernel<<<2, 256, 0, st>>>(la, c.dev);
#define VLC_SELECT(NK) select_kernel<NK, false, false><<<rows, kSelThreads, 0, st>>>(scores, c.dev, s.L, s.Hkv, s.m, lens != nullptr, c.T_max, n_recent, recent_num, recent_den, idx_out, nullptr, nullptr, la)
    if (fold) select_kernel<8, false, true><<<rows + 2, kSelThreads, 0, st>>>(scores, c.dev, s.L, s.Hkv, s.m, lens != nullptr, c.T_max, n_recent, recent_num, recent_den, idx_out, nullptr, nullptr, la);
    else if (per_lane <= 8) VLC_SELECT(8);
    else if (per_lane <= 24) VLC_SELECT(24);
    else if (per_lane <= 64) VLC_SELECT(64);
    else VLC_SELECT(0);
#undef VLC_SELECT
    const int rowbytes = s.d * (s.dtype == VLC_F32 ? 4 : 2);
    const int es = s.dtype == VLC_F32 ? 4 : 2;
    const unsigned grid = (unsigned)c.dev.list[2].cap;
    const char* kf = (const char*)k_full;
    const char* vf = (const char*)v_full;
    if (c.kv_fp8) {
        if (s.d == 64) gather_fp8_kernel<64><<<grid, 256, 0, st>>>(kf, vf, c.dev, s.L, s.Hkv, s.m, c.T_max);
        else gather_fp8_kernel<128><<<grid, 256, 0, st>>>(kf, vf, c.dev, s.L, s.Hkv, s.m, c.T_max);
        return hipGetLastError();
    }
    // Several blocks share a unit: more, shorter chains of dependent passes in flight (64 rows per block measured
    // 3-7 % faster on the whole compaction than 512).
    const int parts = kGatherUnit / c.opt.gather_rows;
    const unsigned g2 = grid * (unsigned)parts;
    if (rowbytes == 128) gather_kernel<128><<<g2, 256, 0, st>>>(kf, vf, c.dev, s.L, s.Hkv, s.m, c.T_max, es, parts);
    else if (rowbytes == 256) gather_kernel<256><<<g2, 256, 0, st>>>(kf, vf, c.dev, s.L, s.Hkv, s.m, c.T_max, es, parts);
    else gather_kernel<512><<<g2, 256, 0, st>>>(kf, vf, c.dev, s.L, s.Hkv, s.m, c.T_max, es, parts);
    return hipGetLastError();
}

hipError_t launch_cache_hit_count(const vlc_cache& c, const float* scores_star, int32_t* hits_out, float* rate_out,
                                  hipStream_t st) {
    const vlc_shape& s = c.shape;
    const int rows = s.B * s.L * s.Hkv;
    const int per_lane = (((s.m + kSelWaves - 1) / kSelWaves + 63) / 64);
#define VLC_HITS(NK) select_kernel<NK, true, false><<<rows, kSelThreads, 0, st>>>(scores_star, c.dev, s.L, s.Hkv, s.m, c.ragged, c.T_max, 0, 0, 0, nullptr, hits_out, rate_out, LayoutArgs{})
    if (per_lane <= 8) VLC_HITS(8);
    else if (per_lane <= 24) VLC_HITS(24);
    else if (per_lane <= 64) VLC_HITS(64);
    else VLC_HITS(0);
#undef VLC_HITS
    return hipGetLastError();
}

}  // namespace vlc
