// Causal attention of the post-vision window rows that also emits its row statistics
// (gfx950, v_mfma_f32_32x32x16_bf16).
//
// The first kernel of the paper's App. A.3 computes, for the window rows, exactly the two
// reductions a fused-softmax attention kernel already carries (running max, running sum).  A
// prefill attention kernel that hands those out for its last tau rows makes that sweep of K
// unnecessary: this file is that kernel for the window rows, O = softmax(Q' K^T) V under the
// causal mask of Alg. 1, with M and Z as by-products; the column sweep then runs from them.
//
// Layout of the work: as in the row-statistics sweep, S^T = K Q'^T per 32-key tile, so the 16
// logits a lane holds belong to ONE query row and the online softmax stays in the lane (the two
// lane halves share their running max once per tile).  The probabilities, rounded to bf16, are
// then already laid out as the B operand of O^T += V^T P^T (lane = query row, 8 keys per lane
// half), provided V^T is read with the keys in the accumulator's order: V is staged transposed in
// LDS ([d][key], keys permuted inside each group of 16, 16-byte granules XOR-swizzled so that both
// the transposing 4-byte writes and the 16-byte fragment reads are free of bank conflicts).
// A lane's 64 output accumulators belong to its query row too, so the rescale when a running
// max moves is a per-lane factor; it is skipped for tiles in which no max of the wave moved.
// The key range is split across blocks as in the scoring sweeps; partial outputs (unnormalised,
// with their max and sum) are merged by a second kernel, or written out directly when a KV group
// has a single split.
#include <type_traits>

#include "common.h"
#include "internal.h"
#include "score_tiles.h"

namespace vlc {
namespace {

using namespace tiles;

constexpr int kVtRowBytes = kChunk * 2;         // one d-row of the transposed V chunk: 128 keys, no padding
constexpr int kMaxRowBlocks = 8;                // 32-row blocks per launch (one per wave)

struct WinArgs {
    const bf16_t* q_win;
    const bf16_t* k;
    const bf16_t* v;
    const float* sm_scale;
    bf16_t* out;             // [B,L,Hq,tau,d]
    float* row_max;          // [B,L,Hq,tau], natural-log domain
    float* row_sum;
    float* part_o;           // [group][split][RP][kD] unnormalised partial outputs
    float2* part_ms;         // [group][split][RP] (max in the exponent domain, sum)
    const int32_t* lens;
    int L, Hq, Hkv, g, m, tau, tauP, RP, keys_per_split, nsplit;
    int rb0;                 // first 32-row block of this launch
};

// Position of chunk-local key kappa inside its d-row of the transposed chunk: inside each group of
// 16 keys the order is the one in which a lane half holds them in a 32x32 accumulator
// (keys {0..3, 8..11} for half 0, {4..7, 12..15} for half 1).
__device__ __forceinline__ int vt_pos(int kappa) {
    const int k16 = kappa & 15;
    return (kappa & ~15) | (((k16 >> 2) & 1) << 3) | ((k16 >> 3) << 2) | (k16 & 3);
}
// Byte offset of the 16-byte granule `gran` of d-row `d`.
__device__ __forceinline__ int vt_granule_offset(int d, int gran) {
    return d * kVtRowBytes + ((gran ^ ((d >> 3) ^ d)) & 15) * 16;
}

// V chunk staging: global -> registers -> LDS, transposed.  A thread holds the same 8 d-values of two
// consecutive keys, so that each LDS write is a 4-byte pair of keys.  Keys at or beyond m are zero.
template <int THREADS>
struct VStage {
    static constexpr int NP = (kChunk / 2) / (THREADS / 16);    // key pairs per thread
    uint4 ra[NP], rb[NP];
    __device__ __forceinline__ void load(const bf16_t* vg, int key0, int m) {
        const int piece = threadIdx.x & 15;
        if (key0 + kChunk <= m) {               // block-uniform: a whole chunk needs no per-key test
#pragma unroll
            for (int u = 0; u < NP; ++u) {
                const int key = key0 + 2 * ((threadIdx.x >> 4) + (THREADS / 16) * u);
                const uint4* src = reinterpret_cast<const uint4*>(vg + (size_t)key * kD + piece * 8);
                ra[u] = src[0];
                rb[u] = src[kD / 8];
            }
            return;
        }
#pragma unroll
        for (int u = 0; u < NP; ++u) {
            const int key = key0 + 2 * ((threadIdx.x >> 4) + (THREADS / 16) * u);
            const uint4* src = reinterpret_cast<const uint4*>(vg + (size_t)key * kD + piece * 8);
            ra[u] = (key < m) ? src[0] : make_uint4(0, 0, 0, 0);
            rb[u] = (key + 1 < m) ? src[kD / 8] : make_uint4(0, 0, 0, 0);
        }
    }
    // The same in 4 instalments: the 2 NP requests of a thread, numbered 2 u + (second key of the pair).
    template <int P>
    __device__ __forceinline__ void load_part(const bf16_t* vg, int key0, int m) {
        static_assert((2 * NP) % 4 == 0, "requests per thread must divide evenly");
        const int piece = threadIdx.x & 15;
        const bool whole = key0 + kChunk <= m;
#pragma unroll
        for (int j = P * (NP / 2); j < (P + 1) * (NP / 2); ++j) {
            const int u = j >> 1, second = j & 1;
            const int key = key0 + 2 * ((threadIdx.x >> 4) + (THREADS / 16) * u) + second;
            const uint4* src = reinterpret_cast<const uint4*>(vg + (size_t)key * kD + piece * 8);
            const uint4 val = (whole || key < m) ? *src : make_uint4(0, 0, 0, 0);
            if (second) rb[u] = val; else ra[u] = val;
        }
    }
    __device__ __forceinline__ void store(uint8_t* sVt) const {
        const int piece = threadIdx.x & 15;
#pragma unroll
        for (int u = 0; u < NP; ++u) {
            const int kappa = 2 * ((threadIdx.x >> 4) + (THREADS / 16) * u);
            const int pos = vt_pos(kappa);                     // even: the pair (kappa, kappa + 1) is one aligned word
            const uint32_t a[4] = {ra[u].x, ra[u].y, ra[u].z, ra[u].w};
            const uint32_t b[4] = {rb[u].x, rb[u].y, rb[u].z, rb[u].w};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t even = __builtin_amdgcn_perm(b[w], a[w], 0x05040100u);   // (a.lo, b.lo): element 2w of both keys
                const uint32_t odd = __builtin_amdgcn_perm(b[w], a[w], 0x07060302u);    // (a.hi, b.hi): element 2w + 1
                const int d0 = piece * 8 + 2 * w;
                *reinterpret_cast<uint32_t*>(sVt + vt_granule_offset(d0, pos >> 3) + (pos & 7) * 2) = even;
                *reinterpret_cast<uint32_t*>(sVt + vt_granule_offset(d0 + 1, pos >> 3) + (pos & 7) * 2) = odd;
            }
        }
    }
};

// A-operand fragment of V^T for d-tile dt, tile t of the chunk, k-step s: lane (l % 32) owns d-row
// 32 dt + l % 32, lane half l / 32 the 8 keys that half holds in accumulator slots [8 s, 8 s + 8).
__device__ __forceinline__ uint4 load_vt_frag(const uint8_t* sVt, int dt, int t, int s, int lane) {
    const int d = dt * 32 + (lane & 31);
    return *reinterpret_cast<const uint4*>(sVt + vt_granule_offset(d, t * 4 + s * 2 + (lane >> 5)));
}

// Maximum over the two lanes l and l ^ 32 (v_permlane32_swap: no trip through the LDS queue).
__device__ __forceinline__ float max_across_halves(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64, 2) void window_attn_kernel(WinArgs a) {   // two waves per SIMD: two 4-wave blocks or one 8-wave block per compute unit
    constexpr int THREADS = WAVES * 64;
    __shared__ __align__(16) bf16_t sK[kChunk * kPitch];
    __shared__ __align__(16) uint8_t sVt[kD * kVtRowBytes];
    const int group = blockIdx.y, split = blockIdx.x;
    const int hkv = group % a.Hkv, bl = group / a.Hkv, l = bl % a.L;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const float c = (a.sm_scale ? a.sm_scale[l] : rsqrtf((float)kD)) * kLog2e;
    const bf16_t* kg = a.k + (size_t)group * a.m * kD;
    const bf16_t* vg = a.v + (size_t)group * a.m * kD;
    const ReqLen rl = request_len(a.lens, bl / a.L, a.m, a.tau);
    const int mb = rl.m, tb = rl.tau;
    const int k_begin = split * a.keys_per_split;
    const int k_end = min(mb, k_begin + a.keys_per_split);
    const bool has_rows = (a.rb0 + wave) * 32 < a.RP;          // wave-uniform

    uint4 qf[1][kKSteps];
    load_q_frags<WAVES, 1>(a, bl, hkv, wave, lane, tb, qf);
    const int r = (a.rb0 + wave) * 32 + (lane & 31);           // this lane's padded window row
    const int jlim = mb - tb + (r % a.tauP);                   // last key it may see
    float m_run = -INFINITY, z_run = 0.f;
    f32x16_t o[kD / 32];
#pragma unroll
    for (int dt = 0; dt < kD / 32; ++dt) o[dt] = f32x16_t{0};

    KStage<THREADS> ks_;
    VStage<THREADS> vs_;
    if (k_begin < k_end) { ks_.load(kg, k_begin, mb); vs_.load(vg, k_begin, mb); }
    for (int kc = k_begin; kc < k_end; kc += kChunk) {
        __syncthreads();                                       // previous chunk fully consumed
        ks_.store(sK);
        vs_.store(sVt);
        __syncthreads();
        const bool next = kc + kChunk < k_end;                 // block-uniform
        const bool masked = kc + kChunk > mb - tb + 1;         // chunk reaches past the first window key
        // In an 8-wave block the next chunk's global requests go out in four instalments, one per tile, so
        // that the waves do not queue up behind the compute unit's one address path at the top of a chunk
        // (measured: 940 cycles per chunk).  The 4-wave block has no registers for the unrolled form.
        constexpr bool SPREAD = WAVES == 8;
        if (next && (!SPREAD || !has_rows)) { ks_.load(kg, kc + kChunk, mb); vs_.load(vg, kc + kChunk, mb); }
        if (!has_rows) continue;
        auto tile = [&](auto partc, int t) {
            constexpr int part = decltype(partc)::value;
            if constexpr (part >= 0) {
                if (next) {
                    ks_.template load_part<part, kChunk / 32>(kg, kc + kChunk, mb);
                    vs_.template load_part<part>(vg, kc + kChunk, mb);
                }
            }
            uint4 kf[kKSteps];
            load_k_frags(sK, t, lane, kf);
            f32x16_t acc = {0};
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(kf[ks]), as_frag(qf[0][ks]), acc, 0, 0, 0);
            // acc[i] = <k_key, q_row>, key = kc + 32 t + acc_row(i), row = this lane's
            float v[16];
            if (masked) {
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = (kc + t * 32 + acc_row(i, lane) <= jlim) ? acc[i] : -INFINITY;
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = acc[i];
            }
            float tmax = v[0];
#pragma unroll
            for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, v[i]);
            tmax = max_across_halves(tmax);                    // both lane halves of a row use one max
            const float m_new = fmaxf(m_run, tmax * c);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;   // a row that has seen no key yet: all p = 0
            float p[16], zs = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) { p[i] = exp2_fast(fmaf(v[i], c, -m_use)); zs += p[i]; }
            const float alpha = exp2_fast(m_run - m_use);      // 1 when the max did not move, 0 for the first keys
            if (__any(m_new > m_run)) {
#pragma unroll
                for (int dt = 0; dt < kD / 32; ++dt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
            }
            z_run = z_run * alpha + zs;
            m_run = m_new;
            // probabilities as bf16: slots [8 s, 8 s + 8) are the 8 keys this lane half supplies to k-step s
            bf16x8_t pf[2];
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[s][e] = (__bf16)p[8 * s + e];
#pragma unroll
            for (int dt = 0; dt < kD / 32; ++dt)
#pragma unroll
                for (int s = 0; s < 2; ++s)
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(load_vt_frag(sVt, dt, t, s, lane)), pf[s], o[dt], 0, 0, 0);
        };
        if constexpr (SPREAD) {
            tile(std::integral_constant<int, 0>{}, 0);
            if (kc + 32 < k_end) tile(std::integral_constant<int, 1>{}, 1);
            if (kc + 64 < k_end) tile(std::integral_constant<int, 2>{}, 2);
            if (kc + 96 < k_end) tile(std::integral_constant<int, 3>{}, 3);
        } else {
#pragma unroll 1
            for (int t = 0; t < kChunk / 32 && kc + t * 32 < k_end; ++t) tile(std::integral_constant<int, -1>{}, t);
        }
    }
    if (!has_rows) return;
    // the two lane halves hold disjoint keys of the same query row under the same max
    const float z = z_run + __shfl_xor(z_run, 32, 64);
    const int hl = r / a.tauP, iw = r % a.tauP;
    const bool real = hl < a.g && iw < tb && r < a.RP;
    if (a.nsplit == 1) {
        if (!real) return;
        const size_t orow = ((size_t)bl * a.Hq + (size_t)hkv * a.g + hl) * a.tau + iw;
        const float inv = 1.f / z;                             // every real row sees key 0 in the only split
        bf16_t* dst = a.out + orow * kD;
#pragma unroll
        for (int dt = 0; dt < kD / 32; ++dt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int d = dt * 32 + acc_row(4 * q4, lane);
                const uint32_t lo = f32_to_bf16_bits(o[dt][4 * q4] * inv) | (f32_to_bf16_bits(o[dt][4 * q4 + 1] * inv) << 16);
                const uint32_t hi = f32_to_bf16_bits(o[dt][4 * q4 + 2] * inv) | (f32_to_bf16_bits(o[dt][4 * q4 + 3] * inv) << 16);
                *reinterpret_cast<uint2*>(dst + d) = make_uint2(lo, hi);
            }
        if (lane < 32) { a.row_max[orow] = m_run * kLn2; a.row_sum[orow] = z; }
        return;
    }
    if (r >= a.RP) return;
    const size_t prow = ((size_t)group * a.nsplit + split) * a.RP + r;
    float* dst = a.part_o + prow * kD;
#pragma unroll
    for (int dt = 0; dt < kD / 32; ++dt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
            *reinterpret_cast<float4*>(dst + dt * 32 + acc_row(4 * q4, lane)) =
                make_float4(o[dt][4 * q4], o[dt][4 * q4 + 1], o[dt][4 * q4 + 2], o[dt][4 * q4 + 3]);
    if (lane < 32) a.part_ms[prow] = make_float2(m_run, z);
}

// Merge of the per-split partials: 32 lanes (4 d-values each) per padded row, 32 rows per block.
__global__ __launch_bounds__(256) void window_attn_merge_kernel(WinArgs a, int groups) {
    const int sub = threadIdx.x >> 5, lane = threadIdx.x & 31;
    for (int it = 0; it < 4; ++it) {
        const size_t x = ((size_t)blockIdx.x * 4 + it) * 8 + sub;      // (group, padded row)
        if (x >= (size_t)groups * a.RP) return;
        const int r = (int)(x % a.RP), group = (int)(x / a.RP);
        const int hl = r / a.tauP, iw = r % a.tauP;
        const int hkv = group % a.Hkv, bl = group / a.Hkv;
        if (hl >= a.g || iw >= request_len(a.lens, bl / a.L, a.m, a.tau).tau) continue;
        float M = -INFINITY;
        for (int s = 0; s < a.nsplit; ++s) M = fmaxf(M, a.part_ms[((size_t)group * a.nsplit + s) * a.RP + r].x);
        float Z = 0.f;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int s = 0; s < a.nsplit; ++s) {
            const size_t prow = ((size_t)group * a.nsplit + s) * a.RP + r;
            const float2 ms = a.part_ms[prow];
            if (!(ms.x > -INFINITY)) continue;                         // this split saw no key of the row
            const float w = exp2_fast(ms.x - M);
            const float4 po = *reinterpret_cast<const float4*>(a.part_o + prow * kD + lane * 4);
            Z += ms.y * w;
            acc.x = fmaf(po.x, w, acc.x); acc.y = fmaf(po.y, w, acc.y); acc.z = fmaf(po.z, w, acc.z); acc.w = fmaf(po.w, w, acc.w);
        }
        const size_t orow = ((size_t)bl * a.Hq + (size_t)hkv * a.g + hl) * a.tau + iw;
        const float inv = 1.f / Z;
        const uint32_t lo = f32_to_bf16_bits(acc.x * inv) | (f32_to_bf16_bits(acc.y * inv) << 16);
        const uint32_t hi = f32_to_bf16_bits(acc.z * inv) | (f32_to_bf16_bits(acc.w * inv) << 16);
        *reinterpret_cast<uint2*>(a.out + orow * kD + lane * 4) = make_uint2(lo, hi);
        if (lane == 0) { a.row_max[orow] = M * kLn2; a.row_sum[orow] = Z; }
    }
}

struct WinPlan { int tauP, RP, nsplit, keys_per_split; };

WinPlan make_plan(const vlc_shape& s) {
    WinPlan p;
    const int g = s.Hq / s.Hkv;
    p.tauP = (s.tau + 31) / 32 * 32;
    p.RP = g * p.tauP;
    const int groups = s.B * s.L * s.Hkv;
    const int chunks = (s.m + kChunk - 1) / kChunk;
    // Two staged chunks (66 KB of LDS) allow two blocks per compute unit: about one resident round
    // of blocks per launch, as for the scoring sweeps; a KV group that has a block of its own
    // anyway is not split (no partial outputs to merge).
    int ns = (512 + groups - 1) / groups;
    if (ns > chunks) ns = chunks;
    if (ns < 1) ns = 1;
    const int cps = (chunks + ns - 1) / ns;
    p.keys_per_split = cps * kChunk;
    p.nsplit = (s.m + p.keys_per_split - 1) / p.keys_per_split;
    return p;
}

}  // namespace

bool window_attn_supported(const vlc_shape& s) {
    return s.dtype == VLC_BF16 && s.d == kD;
}

size_t window_attn_workspace_bytes(const vlc_shape& s) {
    const WinPlan p = make_plan(s);
    if (p.nsplit == 1) return 256;
    const size_t rows = (size_t)s.B * s.L * s.Hkv * p.nsplit * p.RP;
    return (rows * kD * sizeof(float) + 255) / 256 * 256 + (rows * sizeof(float2) + 255) / 256 * 256;
}

hipError_t launch_window_attn(const WindowAttnArgs& w) {
    const vlc_shape& s = w.s;
    const WinPlan p = make_plan(s);
    WinArgs a;
    a.q_win = (const bf16_t*)w.q_win; a.k = (const bf16_t*)w.k; a.v = (const bf16_t*)w.v; a.sm_scale = w.sm_scale;
    a.out = (bf16_t*)w.out; a.row_max = w.row_max; a.row_sum = w.row_sum;
    const int groups = s.B * s.L * s.Hkv;
    const size_t rows = (size_t)groups * p.nsplit * p.RP;
    a.part_o = (float*)w.workspace;
    a.part_ms = (float2*)((char*)w.workspace + (rows * kD * sizeof(float) + 255) / 256 * 256);
    a.lens = s.lens;
    a.L = s.L; a.Hq = s.Hq; a.Hkv = s.Hkv; a.g = s.Hq / s.Hkv; a.m = s.m; a.tau = s.tau;
    a.tauP = p.tauP; a.RP = p.RP; a.keys_per_split = p.keys_per_split; a.nsplit = p.nsplit;
    dim3 grid(p.nsplit, groups);
    const int total_rb = p.RP / 32;
    // Windows beyond 8 row blocks (256 padded rows per KV head) take one launch per 8 row blocks;
    // their rows are independent, K and V are streamed once per launch.
    for (int rb0 = 0; rb0 < total_rb; rb0 += kMaxRowBlocks) {
        const int nrb = total_rb - rb0 < kMaxRowBlocks ? total_rb - rb0 : kMaxRowBlocks;
        a.rb0 = rb0;
        if (nrb <= 4) window_attn_kernel<4><<<grid, 256, 0, w.stream>>>(a);
        else window_attn_kernel<8><<<grid, 512, 0, w.stream>>>(a);
    }
    if (p.nsplit > 1) {
        const size_t n = (size_t)groups * p.RP;
        a.rb0 = 0;
        window_attn_merge_kernel<<<(unsigned)((n + 31) / 32), 256, 0, w.stream>>>(a, groups);
    }
    return hipGetLastError();
}

}  // namespace vlc
