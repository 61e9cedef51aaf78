// Window attention with row statistics, generic version (any storage dtype, d = 64 or 128): the
// causal attention of the last tau prompt rows (paper Sec. 2.1, prefill phase) that also hands out
// the row maximum M_i and row sum Z_i of its softmax, which is what the first scoring kernel of the
// paper's App. A.3 would otherwise compute in a sweep of its own.  The matrix-core kernel in
// window_attn.hip takes bf16 storage with d = 128; this one takes everything else (fp32 storage,
// d = 64) and, on request, that shape too, so that the two can be compared on the same inputs.
// It is written for clarity, not for speed: shapes outside the matrix-core path are small.
//
// One wave per query row.  Keys are taken 64 at a time:
//   1. lane j computes the logit of key j0 + j (its own K row against the query row in LDS);
//   2. online softmax over the tile with two wave reductions; the probabilities go to LDS;
//   3. P.V with lane = output element: the V rows of the tile are read one after the other, each
//      by the whole wave (coalesced), and accumulated in fp32 with fp32 probabilities.
#include "common.h"
#include "internal.h"

namespace vlc {
namespace {

constexpr int kRowsPerBlock = 4;    // query rows (waves) per block

template <typename T, int D>
__global__ __launch_bounds__(kRowsPerBlock * 64) void window_attn_simple_kernel(
    const T* __restrict__ q_win, const T* __restrict__ k, const T* __restrict__ v, const float* __restrict__ sm_scale,
    T* __restrict__ out, float* __restrict__ row_max, float* __restrict__ row_sum,
    int L, int Hq, int Hkv, int m, int tau, int row_tiles, const int32_t* __restrict__ lens) {
    constexpr int EPL = D / 64;                             // output elements per lane
    constexpr int EP = Elem<T>::kPer16B;
    __shared__ __align__(16) float sQ[kRowsPerBlock][D];
    __shared__ float sP[kRowsPerBlock][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = blockIdx.x / row_tiles;                   // (b*L + l)*Hq + h
    const int i = (blockIdx.x % row_tiles) * kRowsPerBlock + wave;       // window row of this wave
    const int h = r % Hq, bl = r / Hq, l = bl % L;
    const int g = Hq / Hkv;
    const ReqLen rl = request_len(lens, bl / L, m, tau);
    const int mb = rl.m, tb = rl.tau;                       // this request's prompt and window length
    if (i >= tb) return;                                    // no block-wide barrier below: a wave may leave
    const float c = (sm_scale ? sm_scale[l] : rsqrtf((float)D)) * kLog2e;
    const T* qrow = q_win + ((size_t)r * tau + i) * D;
    const T* kh = k + ((size_t)bl * Hkv + h / g) * m * D;
    const T* vh = v + ((size_t)bl * Hkv + h / g) * m * D;
#pragma unroll
    for (int e = 0; e < EPL; ++e) sQ[wave][lane * EPL + e] = Elem<T>::load(qrow + lane * EPL + e);
    __builtin_amdgcn_wave_barrier();
    const int jlim = mb - tb + i;                           // last key this row may see (causal mask of Alg. 1)
    float m_run = -INFINITY, z_run = 0.f, acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    for (int j0 = 0; j0 <= jlim; j0 += 64) {
        // ---- logits: lane = key
        const int j = j0 + lane;
        const bool valid = j <= jlim;
        const T* krow = kh + (size_t)(valid ? j : 0) * D;
        float s = 0.f;
#pragma unroll
        for (int cidx = 0; cidx < D / EP; ++cidx) {
            const uint4 raw = reinterpret_cast<const uint4*>(krow)[cidx];
            float f[EP];
            unpack16(raw, f, (const T*)nullptr);
#pragma unroll
            for (int e = 0; e < EP; ++e) s = fmaf(sQ[wave][cidx * EP + e], f[e], s);
        }
        s = valid ? s * c : -INFINITY;                       // exponent domain (log2)
        // ---- online softmax over the tile (every tile holds key j0 <= jlim, so the maximum is finite)
        const float m_new = fmaxf(m_run, wave_allreduce_max(s));
        const float p = valid ? exp2_fast(s - m_new) : 0.f;
        const float corr = exp2_fast(m_run - m_new);         // 0 on the first tile (m_run = -inf)
        z_run = z_run * corr + wave_allreduce_sum(p);
        m_run = m_new;
        __builtin_amdgcn_wave_barrier();
        sP[wave][lane] = p;
        __builtin_amdgcn_wave_barrier();
        // ---- P.V: lane = output element
        const int n = min(64, jlim - j0 + 1);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= corr;
        for (int jj = 0; jj < n; ++jj) {
            const float pj = sP[wave][jj];
            const T* vrow = vh + (size_t)(j0 + jj) * D + lane * EPL;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(pj, Elem<T>::load(vrow + e), acc[e]);
        }
    }
    T* orow = out + ((size_t)r * tau + i) * D;
    const float inv = 1.f / z_run;
#pragma unroll
    for (int e = 0; e < EPL; ++e) Elem<T>::store(orow + lane * EPL + e, acc[e] * inv);
    if (lane == 0) {
        row_max[(size_t)r * tau + i] = m_run * kLn2;        // natural-log domain, as vlc_score hands it out
        row_sum[(size_t)r * tau + i] = z_run;
    }
}

template <typename T, int D>
hipError_t launch_t(const WindowAttnArgs& a) {
    const vlc_shape& s = a.s;
    const int row_tiles = (s.tau + kRowsPerBlock - 1) / kRowsPerBlock;
    const size_t blocks = (size_t)s.B * s.L * s.Hq * row_tiles;
    window_attn_simple_kernel<T, D><<<(unsigned)blocks, kRowsPerBlock * 64, 0, a.stream>>>(
        (const T*)a.q_win, (const T*)a.k, (const T*)a.v, a.sm_scale, (T*)a.out, a.row_max, a.row_sum,
        s.L, s.Hq, s.Hkv, s.m, s.tau, row_tiles, s.lens);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_window_attn_simple(const WindowAttnArgs& a) {
    const vlc_shape& s = a.s;
    if ((size_t)s.B * s.L * s.Hq * ((s.tau + kRowsPerBlock - 1) / kRowsPerBlock) > 0x7fffffffull) return hipErrorInvalidValue;
    if (s.dtype == VLC_F32) return s.d == 64 ? launch_t<float, 64>(a) : launch_t<float, 128>(a);
    return s.d == 64 ? launch_t<bf16_t, 64>(a) : launch_t<bf16_t, 128>(a);
}

}  // namespace vlc
