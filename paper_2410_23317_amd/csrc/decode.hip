// GQA decode attention over the compressed, ragged per-layer cache (paper Sec. 2.1, decoding
// phase: the new key/value is appended, then softmax(q K^T / sqrt d) V over every cached slot).
//
// Bandwidth-bound: every K and V row is read once, coalesced (16 bytes per lane, LPR lanes per
// row), and serves all g query heads of its KV group from registers.  Work unit = one wave and
// one tile of 64 slots:
//   1. logits: packed-bf16 dot products (v_dot2_f32_bf16) against the g query rows held in
//      registers, reduced over the LPR lanes of a row with DPP rotations, parked in LDS;
//   2. softmax over the tile with lane = slot (wave-wide max / sum), running max and sum per head;
//   3. P.V with the V rows streamed the same way, probabilities broadcast from LDS.
// Tiles of a row are dealt round-robin to the 4*S waves of its S blocks (split-KV); the block merges
// its waves through LDS and, if S > 1, the last block to finish (device-scope counter) merges the
// S partial results.  Matrix cores are not used: with g <= 8 query rows per KV head the work is a
// stream, not a contraction.
#include "common.h"
#include "internal.h"

namespace vlc {
namespace {

struct DecodeParams {
    const void* q;
    const void* k_new;
    const void* v_new;
    void* out;
    const float* sm_scale;
    CacheDev dev;
    int B, L, Hq, Hkv, m;
    int layer_begin, T_max, S;
    int appended;            // appends before this call
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

template <typename T, int D, int G>
__global__ __launch_bounds__(256) void decode_kernel(DecodeParams P) {
    constexpr int EP = Elem<T>::kPer16B;        // elements in a 16-byte chunk
    constexpr int LPR = D / EP;                 // lanes per K/V row
    constexpr int KPI = 64 / LPR;               // rows per wave load
    constexpr int TK = 64;                      // slots per tile
    constexpr int NIT = TK / KPI;
    constexpr int UB = NIT < 8 ? NIT : 8;       // loads in flight per batch
    constexpr int GP = pad_pow2(G);
    constexpr int DP = D + 2;
    static_assert(G <= LPR, "one lane per head needed when parking logits");

    __shared__ __align__(16) float sP[4][TK][GP];
    __shared__ float sMerge[4][G][DP];
    __shared__ int sLast;

    const int S = P.S;
    const int row = blockIdx.x / S, split = blockIdx.x % S;
    const int hkv = row % P.Hkv;
    const int b = (row / P.Hkv) % P.B;
    const int lr = row / (P.Hkv * P.B);
    const int l = P.layer_begin + lr;
    const int bl = b * P.L + l;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int sub = lane / LPR, c = lane % LPR;

    T* outp = reinterpret_cast<T*>(P.out) + ((size_t)(lr * P.B + b) * P.Hq + (size_t)hkv * G) * D;
    const int kept = P.dev.kept[bl];
    if (kept == 0) {                            // request rejected at compaction: defined output, no reads
        if (split == 0)
            for (int x = tid; x < G * D; x += 256) Elem<T>::store(outp + x, 0.f);
        return;
    }
    const bool appending = P.k_new != nullptr;
    const int len = kept + P.appended + (appending ? 1 : 0);
    const int cap = kept + P.T_max;
    const int new_slot = appending ? len - 1 : -1;
    const T* Kbase = reinterpret_cast<const T*>(P.dev.kv) + ((P.dev.slot_off[bl] * 2 * P.Hkv) + (int64_t)hkv * cap) * D;
    const T* Vbase = Kbase + (int64_t)P.Hkv * cap * D;
    const T* knew = reinterpret_cast<const T*>(P.k_new) + ((size_t)(lr * P.B + b) * P.Hkv + hkv) * D;
    const T* vnew = reinterpret_cast<const T*>(P.v_new) + ((size_t)(lr * P.B + b) * P.Hkv + hkv) * D;
    const float scale2 = (P.sm_scale ? P.sm_scale[l] : P.default_scale) * kLog2e;

    uint4 qv[G];
#pragma unroll
    for (int h = 0; h < G; ++h)
        qv[h] = *reinterpret_cast<const uint4*>(reinterpret_cast<const T*>(P.q) +
                                                ((size_t)(lr * P.B + b) * P.Hq + (size_t)hkv * G + h) * D + c * EP);

    float m_run[G], l_run[G], acc[G][EP];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m_run[h] = -INFINITY;
        l_run[h] = 0.f;
#pragma unroll
        for (int e = 0; e < EP; ++e) acc[h][e] = 0.f;
    }

    const int nW = 4 * S, wid = split * 4 + wave;
    const int ntiles = (len + TK - 1) / TK;
    for (int tile = wid; tile < ntiles; tile += nW) {
        const int t0 = tile * TK;
        // ---- 1. logits of 64 slots -> LDS
#pragma unroll
        for (int ib = 0; ib < NIT; ib += UB) {
            uint4 kb[UB];
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int key = t0 + (ib + u) * KPI + sub;
                const T* src = (key == new_slot) ? knew : Kbase + (int64_t)key * D;
                kb[u] = (key < len) ? *reinterpret_cast<const uint4*>(src + c * EP) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int key = t0 + (ib + u) * KPI + sub;
                float mine = 0.f;
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float tot = group_allreduce_sum<LPR>(dot16<T>(kb[u], qv[h], 0.f));
                    mine = (c == h) ? tot : mine;
                }
                if (c < G) sP[wave][(ib + u) * KPI + sub][c] = (key < len) ? mine * scale2 : -INFINITY;
            }
        }
        __builtin_amdgcn_wave_barrier();
        // ---- 2. softmax bookkeeping, lane = slot
        float corr[G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float x = sP[wave][lane][h];
            const float m_new = fmaxf(m_run[h], wave_allreduce_max(x));     // finite: the tile has >= 1 slot
            const float pr = exp2_fast(x - m_new);
            corr[h] = exp2_fast(m_run[h] - m_new);
            l_run[h] = l_run[h] * corr[h] + wave_allreduce_sum(pr);
            m_run[h] = m_new;
            sP[wave][lane][h] = pr;
        }
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
            for (int e = 0; e < EP; ++e) acc[h][e] *= corr[h];
        __builtin_amdgcn_wave_barrier();
        // ---- 3. P.V
#pragma unroll
        for (int ib = 0; ib < NIT; ib += UB) {
            uint4 vb[UB];
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int key = t0 + (ib + u) * KPI + sub;
                const T* src = (key == new_slot) ? vnew : Vbase + (int64_t)key * D;
                vb[u] = (key < len) ? *reinterpret_cast<const uint4*>(src + c * EP) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                float f[EP];
                unpack16(vb[u], f, (const T*)nullptr);
                const float* pp = &sP[wave][(ib + u) * KPI + sub][0];
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float ph = pp[h];
#pragma unroll
                    for (int e = 0; e < EP; ++e) acc[h][e] = fmaf(ph, f[e], acc[h][e]);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }

    // The wave that owns the tile of the new slot also stores the new row into the cache.
    if (appending && ((new_slot / TK) % nW) == wid && sub == 0) {
        T* kdst = const_cast<T*>(Kbase) + (int64_t)new_slot * D;
        T* vdst = const_cast<T*>(Vbase) + (int64_t)new_slot * D;
        *reinterpret_cast<uint4*>(kdst + c * EP) = *reinterpret_cast<const uint4*>(knew + c * EP);
        *reinterpret_cast<uint4*>(vdst + c * EP) = *reinterpret_cast<const uint4*>(vnew + c * EP);
        if (c == 0) P.dev.idx[P.dev.slot_off[bl] * P.Hkv + (int64_t)hkv * cap + new_slot] = P.m + P.appended;
    }

    // ---- merge the KPI row groups of the wave, then the 4 waves of the block
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
            for (int e = 0; e < EP; ++e) acc[h][e] += __shfl_xor(acc[h][e], off, 64);
    if (sub == 0) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
#pragma unroll
            for (int e = 0; e < EP; ++e) sMerge[wave][h][c * EP + e] = acc[h][e];
            if (c == 0) { sMerge[wave][h][D] = m_run[h]; sMerge[wave][h][D + 1] = l_run[h]; }
        }
    }
    __syncthreads();
    float* part = P.dev.partials + ((size_t)bl * P.Hq + (size_t)hkv * G) * kMaxSplits * DP;
    for (int x = tid; x < G * D; x += 256) {
        const int h = x / D, e = x % D;
        float mt = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mt = fmaxf(mt, sMerge[w][h][D]);
        float o = 0.f, lt = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float mw = sMerge[w][h][D];
            const float wgt = (mw > -INFINITY) ? exp2_fast(mw - mt) : 0.f;
            o = fmaf(sMerge[w][h][e], wgt, o);
            lt = fmaf(sMerge[w][h][D + 1], wgt, lt);
        }
        if (S == 1) {
            Elem<T>::store(outp + x, o / lt);
        } else {
            float* ps = part + ((size_t)h * kMaxSplits + split) * DP;
            ps[e] = o;
            if (e == 0) { ps[D] = mt; ps[D + 1] = lt; }
        }
    }
    if (S == 1) return;

    // ---- split-KV: the last block of the row to arrive merges the S partials
    __threadfence();
    __syncthreads();
    int32_t* counter = P.dev.counters + (size_t)bl * P.Hkv + hkv;
    if (tid == 0) sLast = (atomicAdd(counter, 1) == S - 1) ? 1 : 0;
    __syncthreads();
    if (!sLast) return;
    __threadfence();
    for (int x = tid; x < G * D; x += 256) {
        const int h = x / D, e = x % D;
        const float* ph = part + (size_t)h * kMaxSplits * DP;
        float mt = -INFINITY;
        for (int s2 = 0; s2 < S; ++s2) mt = fmaxf(mt, ph[s2 * DP + D]);
        float o = 0.f, lt = 0.f;
        for (int s2 = 0; s2 < S; ++s2) {
            const float ms = ph[s2 * DP + D];
            const float wgt = (ms > -INFINITY) ? exp2_fast(ms - mt) : 0.f;
            o = fmaf(ph[s2 * DP + e], wgt, o);
            lt = fmaf(ph[s2 * DP + D + 1], wgt, lt);
        }
        Elem<T>::store(outp + x, o / lt);
    }
    if (tid == 0) *counter = 0;                 // ready for the next launch on this stream
}

template <typename T, int D, int G>
hipError_t launch_one(const DecodeParams& P, int rows, hipStream_t st) {
    decode_kernel<T, D, G><<<rows * P.S, 256, 0, st>>>(P);
    return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_g(const DecodeParams& P, int g, int rows, hipStream_t st) {
    switch (g) {
        case 1: return launch_one<T, D, 1>(P, rows, st);
        case 2: return launch_one<T, D, 2>(P, rows, st);
        case 3: return launch_one<T, D, 3>(P, rows, st);
        case 4: return launch_one<T, D, 4>(P, rows, st);
        case 5: return launch_one<T, D, 5>(P, rows, st);
        case 6: return launch_one<T, D, 6>(P, rows, st);
        case 7: return launch_one<T, D, 7>(P, rows, st);
        case 8: return launch_one<T, D, 8>(P, rows, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_decode(const DecodeArgs& a) {
    const vlc_cache& c = *a.c;
    const vlc_shape& s = c.shape;
    DecodeParams P;
    P.q = a.q; P.k_new = a.k_new; P.v_new = a.v_new; P.out = a.out; P.sm_scale = a.sm_scale;
    P.dev = c.dev;
    P.B = s.B; P.L = s.L; P.Hq = s.Hq; P.Hkv = s.Hkv; P.m = s.m;
    P.layer_begin = a.layer_begin; P.T_max = c.T_max;
    P.appended = a.appended;
    P.default_scale = 1.0f / sqrtf((float)s.d);
    const int rows = a.n_layers * s.B * s.Hkv;
    // Split-KV factor from what the host knows: the mean budget bound and the step count.
    const int64_t est_len = c.sum_k_max / s.L + a.appended + 1;
    const int ntiles = (int)((est_len + 63) / 64);
    int waves_per_row = (4096 + rows - 1) / rows;
    if (waves_per_row > ntiles) waves_per_row = ntiles;
    int S = (waves_per_row + 3) / 4;
    if (S < 1) S = 1;
    if (S > kMaxSplits) S = kMaxSplits;
    P.S = S;
    const int g = s.Hq / s.Hkv;
    if (s.dtype == VLC_F32) return s.d == 64 ? launch_g<float, 64>(P, g, rows, a.stream) : launch_g<float, 128>(P, g, rows, a.stream);
    return s.d == 64 ? launch_g<bf16_t, 64>(P, g, rows, a.stream) : launch_g<bf16_t, 128>(P, g, rows, a.stream);
}

}  // namespace vlc
