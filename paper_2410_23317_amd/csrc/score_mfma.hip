// Matrix-core scoring sweeps for bf16 storage (gfx950, v_mfma_f32_32x32x16_bf16).
//
// The post-vision window Q' K^T of Alg. 1 is the one dense contraction of the path: per KV head a
// (g * tau) x d x m product.  Following the two-sweep schedule of the paper's App. A.3, neither
// the logits nor the attention matrix reach HBM:
//   sweep 1 (row statistics) computes S^T = K Q'^T tile by tile, so that the 16 values a lane holds
//           belong to ONE query row: running max and sum stay in the lane, with one rescale per
//           32-key tile instead of one per element;
//   sweep 2 (column sums + ThresholdFilter counts) first merges sweep 1's per-split statistics for its own rows,
//           then computes S = Q' K^T, so that a lane holds 16
//           query rows of ONE key: the sum over the window rows of Sec. 3.2 is in-lane too, and the
//           Eq. 1 test is one compare on the exponent argument.
// Q' fragments of a block's rows live in registers for the whole sweep; K streams through LDS in
// chunks of 128 keys (global -> registers -> LDS, the next chunk in flight while the current one is
// multiplied).  Each head's tau window rows are padded to a multiple of 32 so that every 32-row
// block belongs to one query head; padded rows carry a +inf offset and vanish from every sum.
#include "common.h"
#include "internal.h"
#include "score_tiles.h"

namespace vlc {
namespace {

using namespace tiles;

struct MfmaArgs {
    const bf16_t* q_win;
    const bf16_t* k;
    const float* sm_scale;
    float2* part;            // [group][split][RP] partial (max, sum), exponent domain (log2)
    const float* row_max;    // natural-log domain, [B,L,Hq,tau]
    const float2* part_in;   // sweep 2: partials of sweep 1 to merge in the prologue, or null (statistics given)
    float* row_max_out;      // sweep 2 with part_in: where the merged statistics go ([B,L,Hq,tau]; either may be null)
    float* row_sum_out;
    const float* row_sum;
    float* scores;           // may be null
    unsigned long long* nnz; // may be null
    const int32_t* lens;     // per-request (m_b, tau_b), or null
    float log2p;
    int L, Hq, Hkv, g, m, tau, tauP, RP, keys_per_split, nsplit;
    int rb0;                 // first 32-row block of this launch (a launch covers at most 16 of them)
    int accumulate;          // sweep 2: add to scores instead of overwriting (row groups after the first)
};

// ------------------------------------------------------------------------------------------------
// Sweep 1: partial row statistics of one key range of one KV group.
template <int WAVES, int RB>
__global__ __launch_bounds__(WAVES * 64, WAVES == 4 ? 3 : 0) void rowstats_mfma_kernel(MfmaArgs a) {   // 4-wave blocks: registers for 3 blocks per CU, accumulators stay out of the AGPRs
    constexpr int THREADS = WAVES * 64;
    __shared__ __align__(16) bf16_t sK[kChunk * kPitch];
    const int group = blockIdx.x, split = blockIdx.y;       // group-major: see the launch
    const int hkv = group % a.Hkv, bl = group / a.Hkv, l = bl % a.L;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;     // wave index in a scalar register
    const float c = (a.sm_scale ? a.sm_scale[l] : rsqrtf((float)kD)) * kLog2e;
    const bf16_t* kg = a.k + (size_t)group * a.m * kD;
    const ReqLen rl = request_len(a.lens, bl / a.L, a.m, a.tau);
    const int mb = rl.m, tb = rl.tau;                       // this request's prompt and window length
    const int k_begin = split * a.keys_per_split;
    const int k_end = min(mb, k_begin + a.keys_per_split);

    if (a.nnz && split == 0 && a.rb0 == 0 && (int)threadIdx.x < a.g)
        a.nnz[(size_t)bl * a.Hq + (size_t)hkv * a.g + threadIdx.x] = 0;      // sweep 2 adds into these
    uint4 qf[RB][kKSteps];
    load_q_frags<WAVES, RB>(a, bl, hkv, wave, lane, tb, qf);
    // this lane's query row per row block, and the last key it may see (causal mask of Alg. 1)
    int jlim[RB];
    float m_run[RB], z_run[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int r = (a.rb0 + wave * RB + rb) * 32 + (lane & 31);
        jlim[rb] = mb - tb + (r % a.tauP);
        m_run[rb] = -INFINITY;
        z_run[rb] = 0.f;
    }

    KStage<THREADS> st;
    if (k_begin < k_end) st.load(kg, k_begin, mb);
    for (int kc = k_begin; kc < k_end; kc += kChunk) {
        __syncthreads();                                   // previous chunk fully consumed
        st.store(sK);
        __syncthreads();
        if (kc + kChunk < k_end) st.load(kg, kc + kChunk, mb);
        const bool masked = kc + kChunk > mb - tb + 1;     // chunk reaches past the first window key
#pragma unroll 1
        for (int t = 0; t < kChunk / 32; ++t) {
            if (kc + t * 32 >= k_end) break;
            uint4 kf[kKSteps];
            load_k_frags(sK, t, lane, kf);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                if ((a.rb0 + wave * RB + rb) * 32 >= a.RP) continue;       // wave-uniform: no rows here
                f32x16_t acc = {0};
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks)
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(kf[ks]), as_frag(qf[rb][ks]), acc, 0, 0, 0);
                // acc[i] = <k_key, q_row>, key = kc + 32 t + acc_row(i), row = this lane's
                float v[16];
                if (masked) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) v[i] = (kc + t * 32 + acc_row(i, lane) <= jlim[rb]) ? acc[i] : -INFINITY;
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) v[i] = acc[i];
                }
                float tmax = v[0];
#pragma unroll
                for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, v[i]);
                const float m_new = fmaxf(m_run[rb], tmax * c);
                if (m_new > -INFINITY) {
                    float zs = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; ++i) zs += exp2_fast(fmaf(v[i], c, -m_new));
                    z_run[rb] = z_run[rb] * exp2_fast(m_run[rb] - m_new) + zs;
                    m_run[rb] = m_new;
                }
            }
        }
    }
    // the two lane halves hold disjoint keys of the same query row
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const float mo = __shfl_xor(m_run[rb], 32, 64), zo = __shfl_xor(z_run[rb], 32, 64);
        const float mm = fmaxf(m_run[rb], mo);
        float z = 0.f;
        if (m_run[rb] > -INFINITY) z += z_run[rb] * exp2_fast(m_run[rb] - mm);
        if (mo > -INFINITY) z += zo * exp2_fast(mo - mm);
        const int r = (a.rb0 + wave * RB + rb) * 32 + (lane & 31);
        if (lane < 32 && r < a.RP) a.part[((size_t)group * a.nsplit + split) * a.RP + r] = make_float2(mm, z);
    }
}

// ------------------------------------------------------------------------------------------------
// Sweep 2: column sums of the softmax over all window rows of the KV group, and per-head counts.
template <int WAVES, int RB>
__global__ __launch_bounds__(WAVES * 64, WAVES == 4 ? 3 : 4) void colsweep_mfma_kernel(MfmaArgs a) {   // waves per SIMD: 2 blocks of 8 waves, or 3 of 4
    constexpr int THREADS = WAVES * 64;
    __shared__ __align__(16) bf16_t sK[kChunk * kPitch];
    __shared__ float sCol[WAVES][kChunk];
    const int group = blockIdx.x, split = blockIdx.y;       // group-major: see the launch
    const int hkv = group % a.Hkv, bl = group / a.Hkv, l = bl % a.L;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;     // wave index in a scalar register
    const float c = (a.sm_scale ? a.sm_scale[l] : rsqrtf((float)kD)) * kLog2e;
    const bf16_t* kg = a.k + (size_t)group * a.m * kD;
    const ReqLen rl = request_len(a.lens, bl / a.L, a.m, a.tau);
    const int mb = rl.m, tb = rl.tau;                       // this request's prompt and window length
    const int k_begin = split * a.keys_per_split;
    const int k_end = min(mb, k_begin + a.keys_per_split);

    // Order of the first requests: the few bytes of sweep 1's partial statistics go out first (every block of the
    // launch starts at once, and behind 32 KB of K per block they would wait for the whole burst), then the first
    // K chunk, then the Q' fragments; the merge of the statistics and its barrier run while K is on its way.
    constexpr int kSplitRegs = 4;               // splits whose partials a thread holds at once (more are merged in rounds)
    float2 pin[kSplitRegs];
    const int r_mine = a.rb0 * 32 + (int)threadIdx.x;       // the row whose statistics this thread merges (first round)
    const bool mine = a.part_in && (int)threadIdx.x < WAVES * RB * 32 && r_mine < a.RP;
    if (mine) {
#pragma unroll
        for (int sp = 0; sp < kSplitRegs; ++sp)
            pin[sp] = sp < a.nsplit ? a.part_in[((size_t)group * a.nsplit + sp) * a.RP + r_mine] : make_float2(-INFINITY, 0.f);
    }
    KStage<THREADS> st;
    if (k_begin < k_end) st.load(kg, k_begin, mb);
    uint4 qf[RB][kKSteps];
    load_q_frags<WAVES, RB>(a, bl, hkv, wave, lane, tb, qf);
    // per accumulator slot: exponent offset (+inf for padded rows) and 1 / row sum
    float mc[RB][16], iz[RB][16];
    uint32_t cnt[RB];
    __shared__ __align__(16) float2 sStat[WAVES * RB * 32];
    if (a.part_in) {
        // the partial statistics of sweep 1's key splits are merged here, one thread per row of the block; the
        // block of the first split also writes the row maximum and sum the caller asked for
        for (int t = threadIdx.x; t < WAVES * RB * 32; t += THREADS) {
            const int r = a.rb0 * 32 + t;
            float2 st = make_float2(INFINITY, 0.f);
            const int hl = r / a.tauP, iw = r % a.tauP;
            if (r < a.RP && hl < a.g && iw < tb) {
                float M = -INFINITY, Z = 0.f;
                for (int sp0 = 0; sp0 < a.nsplit; sp0 += kSplitRegs) {
                    if (sp0 > 0 || t != (int)threadIdx.x) {          // beyond what was requested at the start
#pragma unroll
                        for (int sp = 0; sp < kSplitRegs; ++sp)
                            pin[sp] = sp0 + sp < a.nsplit ? a.part_in[((size_t)group * a.nsplit + sp0 + sp) * a.RP + r] : make_float2(-INFINITY, 0.f);
                    }
                    float Mn = M;
#pragma unroll
                    for (int sp = 0; sp < kSplitRegs; ++sp) Mn = fmaxf(Mn, pin[sp].x);
                    if (Mn > -INFINITY) {
                        Z *= exp2_fast(M - Mn);                       // 0 on the first round (M = -inf)
#pragma unroll
                        for (int sp = 0; sp < kSplitRegs; ++sp)
                            if (pin[sp].x > -INFINITY) Z += pin[sp].y * exp2_fast(pin[sp].x - Mn);
                        M = Mn;
                    }
                }
                st = make_float2(M, 1.f / Z);
                if (split == 0) {                  // either output may be absent (a count-only sweep keeps no row sums)
                    const size_t o = ((size_t)bl * a.Hq + (size_t)hkv * a.g + hl) * a.tau + iw;
                    if (a.row_max_out) a.row_max_out[o] = M * kLn2;
                    if (a.row_sum_out) a.row_sum_out[o] = Z;
                }
            }
            sStat[t] = st;
        }
        __syncthreads();
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        cnt[rb] = 0;
        if (a.part_in) {
            const float2* sp = sStat + (wave * RB + rb) * 32 + 4 * (lane >> 5);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 lo = *reinterpret_cast<const float4*>(sp + 8 * q);
                const float4 hi = *reinterpret_cast<const float4*>(sp + 8 * q + 2);
                mc[rb][4 * q] = lo.x; iz[rb][4 * q] = lo.y; mc[rb][4 * q + 1] = lo.z; iz[rb][4 * q + 1] = lo.w;
                mc[rb][4 * q + 2] = hi.x; iz[rb][4 * q + 2] = hi.y; mc[rb][4 * q + 3] = hi.z; iz[rb][4 * q + 3] = hi.w;
            }
            continue;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int r = (a.rb0 + wave * RB + rb) * 32 + acc_row(i, lane);
            const int hl = r / a.tauP, iw = r % a.tauP;
            const bool ok = hl < a.g && iw < tb;
            const size_t o = ((size_t)bl * a.Hq + (size_t)hkv * a.g + (ok ? hl : 0)) * a.tau + (ok ? iw : 0);
            mc[rb][i] = ok ? a.row_max[o] * kLog2e : INFINITY;
            iz[rb][i] = (ok && a.row_sum) ? 1.f / a.row_sum[o] : 0.f;
        }
    }

    for (int kc = k_begin; kc < k_end; kc += kChunk) {
        // no barrier in front of the store: the one that follows the tiles of the previous chunk (below) already
        // orders every wave's reads of sK before it, and the readers of sCol pass the barrier after the store
        // before any wave writes sCol again
        st.store(sK);
        __syncthreads();
        if (kc + kChunk < k_end) st.load(kg, kc + kChunk, mb);
        const bool masked = kc + kChunk > mb - tb + 1;
#pragma unroll 1
        for (int t = 0; t < kChunk / 32; ++t) {
            uint4 kf[kKSteps];
            load_k_frags(sK, t, lane, kf);
            const int key = kc + t * 32 + (lane & 31);          // this lane's key (column of the tile)
            float col = 0.f;
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                if ((a.rb0 + wave * RB + rb) * 32 >= a.RP) continue;
                f32x16_t acc = {0};
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks)
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(qf[rb][ks]), as_frag(kf[ks]), acc, 0, 0, 0);
                // acc[i] = <q_row, k_key>, row = row block base + acc_row(i), key = this lane's
                if (masked) {
                    const int base = mb - tb + ((a.rb0 + wave * RB + rb) * 32) % a.tauP;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const bool valid = key <= base + acc_row(i, lane);
                        const float ea = fmaf(acc[i], c, -mc[rb][i]);
                        const float e = valid ? exp2_fast(ea) : 0.f;
                        col = fmaf(e, iz[rb][i], col);
                        cnt[rb] += (uint32_t)__popcll(__ballot(valid && ea >= a.log2p));   // wave-wide count on the scalar unit
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float ea = fmaf(acc[i], c, -mc[rb][i]);
                        col = fmaf(exp2_fast(ea), iz[rb][i], col);
                        cnt[rb] += (uint32_t)__popcll(__ballot(ea >= a.log2p));
                    }
                }
            }
            {   // the lane halves hold different rows of the same key: lane l + lane l ^ 32, with the lane-swap
                // instruction rather than a shuffle through the LDS queue
                const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(col), __float_as_uint(col), false, false);
                col = __uint_as_float(r[0]) + __uint_as_float(r[1]);
            }
            if (lane < 32) sCol[wave][t * 32 + lane] = col;
        }
        __syncthreads();
        if (a.scores && threadIdx.x < kChunk && kc + threadIdx.x < k_end) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) s += sCol[w][threadIdx.x];
            float* dst = a.scores + (size_t)group * a.m + kc + threadIdx.x;
            *dst = a.accumulate ? *dst + s : s;
        }
    }
    // keys of the padded prompt beyond this request's own length score zero
    if (a.scores && a.lens) {
        const int z_end = min(a.m, k_begin + a.keys_per_split);
        for (int j = max(k_begin, mb) + (int)threadIdx.x; j < z_end; j += THREADS) a.scores[(size_t)group * a.m + j] = 0.f;
    }
    if (a.nnz) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int rbase = (a.rb0 + wave * RB + rb) * 32;
            if (rbase >= a.RP) continue;
            const uint32_t tot = cnt[rb];                        // already a wave-wide count
            const int hl = rbase / a.tauP;
            if (lane == 0 && tot && hl < a.g)
                atomicAdd(a.nnz + (size_t)bl * a.Hq + (size_t)hkv * a.g + hl, (unsigned long long)tot);
        }
    }
}

struct Plan { int tauP, RP, nsplit, keys_per_split; };

constexpr int kMaxRowBlocksPerLaunch = 16;      // 512 padded window rows per KV head and launch

Plan make_plan(const vlc_shape& s) {
    Plan p;
    const int g = s.Hq / s.Hkv;
    p.tauP = (s.tau + 31) / 32 * 32;
    p.RP = g * p.tauP;
    const int groups = s.B * s.L * s.Hkv;
    const int chunks = (s.m + kChunk - 1) / kChunk;
    // Splits of the key range per KV group.  Measured on the 7B and 34B shapes: about one resident
    // round of blocks (768 four-wave blocks fit the chip) beats finer splits, whose per-block
    // prologue (Q' fragments, row statistics) is not hidden; with a thousand or more groups two
    // splits even out the last round.
    int ns = (768 + groups - 1) / groups;
    if (ns == 1 && chunks >= 16) ns = 2;
    if (ns > chunks) ns = chunks;
    if (ns < 1) ns = 1;
    const int cps = (chunks + ns - 1) / ns;
    p.keys_per_split = cps * kChunk;
    p.nsplit = (s.m + p.keys_per_split - 1) / p.keys_per_split;
    return p;
}

MfmaArgs make_args(const ScoreArgs& a, const Plan& p) {
    MfmaArgs m;
    const vlc_shape& s = a.s;
    m.q_win = (const bf16_t*)a.q_win; m.k = (const bf16_t*)a.k; m.sm_scale = a.sm_scale;
    m.part = (float2*)a.workspace;
    m.row_max = a.row_max; m.row_sum = a.row_sum;
    m.part_in = nullptr; m.row_max_out = a.row_max; m.row_sum_out = a.row_sum;
    m.scores = a.scores; m.nnz = (unsigned long long*)a.nnz;
    m.log2p = log2f(a.p);
    m.lens = s.lens;
    m.L = s.L; m.Hq = s.Hq; m.Hkv = s.Hkv; m.g = s.Hq / s.Hkv; m.m = s.m; m.tau = s.tau;
    m.tauP = p.tauP; m.RP = p.RP; m.keys_per_split = p.keys_per_split; m.nsplit = p.nsplit;
    m.rb0 = 0; m.accumulate = 0;
    return m;
}

size_t part_bytes(const vlc_shape& s, const Plan& p) {
    return ((size_t)s.B * s.L * s.Hkv * p.nsplit * p.RP * sizeof(float2) + 255) / 256 * 256;
}

}  // namespace

bool score_mfma_supported(const vlc_shape& s) {
    return s.dtype == VLC_BF16 && s.d == kD;
}

size_t score_mfma_workspace_bytes(const vlc_shape& s) {
    if (!score_mfma_supported(s)) return 0;
    return part_bytes(s, make_plan(s));
}

// A launch covers up to 16 row blocks (32 padded window rows each) of every KV group; longer windows
// take several launches over consecutive row-block ranges.  Block shape by row blocks in the launch:
// up to 4 -> 4 waves, up to 8 -> 8 waves, else 8 waves x 2 row blocks (sweep 1) or 16 waves (sweep 2).
hipError_t launch_rowstats_mfma(const ScoreArgs& a) {
    const vlc_shape& s = a.s;
    const Plan p = make_plan(s);
    MfmaArgs m = make_args(a, p);
    const int groups = s.B * s.L * s.Hkv;
    // Group-major grid: blocks go to the 8 XCDs round-robin by linear index, so with a multiple of 8 KV groups the key
    // splits of a group run on one XCD and share its Q' rows in that XCD's L2 (cfg1: 44.7 -> 42.3 us, sweep 2
    // 49.5 -> 45.5 us; no change for shapes whose splits are dispatched rounds apart).
    dim3 grid(groups, p.nsplit);
    const int total_rb = p.RP / 32;
    for (int rb0 = 0; rb0 < total_rb; rb0 += kMaxRowBlocksPerLaunch) {
        const int nrb = total_rb - rb0 < kMaxRowBlocksPerLaunch ? total_rb - rb0 : kMaxRowBlocksPerLaunch;
        m.rb0 = rb0;
        if (nrb <= 4) rowstats_mfma_kernel<4, 1><<<grid, 256, 0, a.stream>>>(m);
        else if (nrb <= 8) rowstats_mfma_kernel<8, 1><<<grid, 512, 0, a.stream>>>(m);
        else rowstats_mfma_kernel<8, 2><<<grid, 512, 0, a.stream>>>(m);        // measured faster than 16 x 1 for this sweep
    }
    return hipGetLastError();
}

hipError_t launch_colsweep_mfma(const ScoreArgs& a, bool merge_partials) {
    const vlc_shape& s = a.s;
    const Plan p = make_plan(s);
    MfmaArgs m = make_args(a, p);
    if (merge_partials) m.part_in = m.part;          // sweep 1 ran just before on the same workspace
    dim3 grid(s.B * s.L * s.Hkv, p.nsplit);       // group-major, as in sweep 1
    const int total_rb = p.RP / 32;
    for (int rb0 = 0; rb0 < total_rb; rb0 += kMaxRowBlocksPerLaunch) {
        const int nrb = total_rb - rb0 < kMaxRowBlocksPerLaunch ? total_rb - rb0 : kMaxRowBlocksPerLaunch;
        m.rb0 = rb0;
        m.accumulate = rb0 > 0;                 // launches of one stream run in order: the column sums add up deterministically
        if (nrb <= 4) colsweep_mfma_kernel<4, 1><<<grid, 256, 0, a.stream>>>(m);
        else if (nrb <= 8) colsweep_mfma_kernel<8, 1><<<grid, 512, 0, a.stream>>>(m);
        else colsweep_mfma_kernel<16, 1><<<grid, 1024, 0, a.stream>>>(m);
    }
    return hipGetLastError();
}

}  // namespace vlc
