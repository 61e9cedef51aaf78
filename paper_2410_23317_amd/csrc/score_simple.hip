// Generic scoring sweeps (any storage dtype): plain-ALU version of the two-sweep schedule of the
// paper's App. A.3.  Sweep 1 reduces over keys (row max M_i and row sum Z_i of the causal softmax
// of Alg. 1), sweep 2 recomputes the logits and reduces over the window rows (accumulated
// post-vision attention, Sec. 3.2) while counting the entries ThresholdFilter keeps (Eq. 1).
// Neither the logits nor the attention matrix ever reach HBM.
//
// One thread owns one key: its K row sits in registers, the query rows are broadcast from LDS.
// This is the path for fp32 storage and the fallback for shapes the matrix-core path does not
// take; it is arithmetic-bound, not bandwidth-bound.
#include "common.h"
#include "internal.h"

namespace vlc {
namespace {

constexpr int kRT = 32;   // query rows staged in LDS at a time

template <typename T, int D>
__device__ __forceinline__ void load_key_row(const T* row, bool ok, float (&kr)[D]) {
    constexpr int EP = Elem<T>::kPer16B;
#pragma unroll
    for (int c = 0; c < D / EP; ++c) {
        uint4 v = ok ? reinterpret_cast<const uint4*>(row)[c] : make_uint4(0, 0, 0, 0);
        float f[EP];
        unpack16(v, f, (const T*)nullptr);
#pragma unroll
        for (int e = 0; e < EP; ++e) kr[c * EP + e] = f[e];
    }
}

// Stage rows [i0, i0 + n) of one head's query window into LDS as fp32.
template <typename T, int D>
__device__ __forceinline__ void stage_q(const T* qh, int i0, int n, float* qs) {
    for (int x = threadIdx.x; x < n * D; x += blockDim.x) qs[x] = Elem<T>::load(qh + (size_t)i0 * D + x);
}

template <int D>
__device__ __forceinline__ float dot_lds(const float* qrow, const float (&kr)[D]) {
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < D; e += 4) {
        float4 qv = *reinterpret_cast<const float4*>(qrow + e);
        acc = fmaf(qv.x, kr[e], acc);
        acc = fmaf(qv.y, kr[e + 1], acc);
        acc = fmaf(qv.z, kr[e + 2], acc);
        acc = fmaf(qv.w, kr[e + 3], acc);
    }
    return acc;
}

// Sweep 1: partial (max, sum) of every window row over this block's 256 keys.
template <typename T, int D>
__global__ __launch_bounds__(256) void rowstats_simple_kernel(
    const T* __restrict__ q_win, const T* __restrict__ k, const float* __restrict__ sm_scale,
    float2* __restrict__ part, int L, int Hq, int Hkv, int m, int tau, int nchunks,
    const int32_t* __restrict__ lens) {
    __shared__ __align__(16) float qs[kRT * D];
    __shared__ float2 red[kRT][4];
    const int r = blockIdx.x / nchunks, chunk = blockIdx.x % nchunks;      // r = (b*L + l)*Hq + h; 1-D grid: rows * chunks
    const int h = r % Hq, bl = r / Hq, l = bl % L;
    const int g = Hq / Hkv;
    const int j = chunk * kScoreChunk + threadIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const float scale = sm_scale ? sm_scale[l] : rsqrtf((float)D);
    const ReqLen rl = request_len(lens, bl / L, m, tau);
    const int mb = rl.m, tb = rl.tau;                       // this request's prompt and window length
    const T* krow = k + (((size_t)bl * Hkv + h / g) * m + (j < mb ? j : 0)) * D;
    const T* qh = q_win + (size_t)r * tau * D;
    float kr[D];
    load_key_row<T, D>(krow, j < mb, kr);
    for (int i0 = 0; i0 < tb; i0 += kRT) {
        const int n = min(kRT, tb - i0);
        __syncthreads();
        stage_q<T, D>(qh, i0, n, qs);
        __syncthreads();
        for (int ii = 0; ii < n; ++ii) {
            const int i = i0 + ii;
            const float s = dot_lds<D>(qs + ii * D, kr) * scale;
            const bool valid = (j < mb) && (j <= mb - tb + i);
            const float wmax = wave_allreduce_max(valid ? s : -INFINITY);
            const float e = valid ? exp2_fast((s - wmax) * kLog2e) : 0.f;
            const float wsum = wave_allreduce_sum(e);
            if (lane == 0) red[ii][wave] = make_float2(wmax, wsum);
        }
        __syncthreads();
        if (threadIdx.x < n) {                       // combine the four waves for the rows of this stage
            const int ii = threadIdx.x;
            float M = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) M = fmaxf(M, red[ii][w].x);
            float Z = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w)
                if (red[ii][w].x > -INFINITY) Z += red[ii][w].y * exp2_fast((red[ii][w].x - M) * kLog2e);
            part[((size_t)r * tau + i0 + ii) * nchunks + chunk] = make_float2(M, Z);
        }
    }
}

// Merge the per-chunk partials of a window row: thread per (head row r, window row i).  The first
// n_clear threads also zero the per-head counters that the second sweep adds into.
__global__ void rowstats_merge_kernel(const float2* __restrict__ part, float* __restrict__ row_max,
                                      float* __restrict__ row_sum, size_t rows, int nchunks,
                                      uint64_t* __restrict__ nnz_clear, size_t n_clear,
                                      const int32_t* __restrict__ lens, int LHq, int m, int tau) {
    const size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x < n_clear) nnz_clear[x] = 0;
    if (x >= rows) return;
    if ((int)(x % tau) >= request_len(lens, (int)(x / tau / LHq), m, tau).tau) return;      // window row beyond this request's
    const float2* p = part + x * nchunks;
    float M = -INFINITY;
    for (int c = 0; c < nchunks; ++c) M = fmaxf(M, p[c].x);
    float Z = 0.f;
    for (int c = 0; c < nchunks; ++c)
        if (p[c].x > -INFINITY) Z += p[c].y * exp2_fast((p[c].x - M) * kLog2e);
    row_max[x] = M;
    row_sum[x] = Z;
}

// Sweep 2: column sums of the softmax over the window rows of the whole KV group, plus the
// per-query-head count of entries with s_ij - M_i >= ln p.
template <typename T, int D>
__global__ __launch_bounds__(256) void colsweep_simple_kernel(
    const T* __restrict__ q_win, const T* __restrict__ k, const float* __restrict__ sm_scale,
    const float* __restrict__ row_max, const float* __restrict__ row_sum,
    float* __restrict__ scores, unsigned long long* __restrict__ nnz, float lnp,
    int L, int Hq, int Hkv, int m, int tau, const int32_t* __restrict__ lens) {
    __shared__ __align__(16) float qs[kRT * D];
    __shared__ float ms[kRT], izs[kRT];
    const int nchunks = (m + kScoreChunk - 1) / kScoreChunk;
    const int rk = blockIdx.x / nchunks, chunk = blockIdx.x % nchunks;     // rk = (b*L + l)*Hkv + hkv
    const int hkv = rk % Hkv, bl = rk / Hkv, l = bl % L;
    const int g = Hq / Hkv;
    const int j = chunk * kScoreChunk + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const float scale = sm_scale ? sm_scale[l] : rsqrtf((float)D);
    const ReqLen rl = request_len(lens, bl / L, m, tau);
    const int mb = rl.m, tb = rl.tau;
    const T* krow = k + ((size_t)rk * m + (j < mb ? j : 0)) * D;
    float kr[D];
    load_key_row<T, D>(krow, j < mb, kr);
    float psi = 0.f;
    for (int hh = 0; hh < g; ++hh) {
        const size_t r = (size_t)bl * Hq + hkv * g + hh;
        const T* qh = q_win + r * tau * D;
        uint32_t cnt = 0;
        for (int i0 = 0; i0 < tb; i0 += kRT) {
            const int n = min(kRT, tb - i0);
            __syncthreads();
            stage_q<T, D>(qh, i0, n, qs);
            if (threadIdx.x < n) {
                ms[threadIdx.x] = row_max[r * tau + i0 + threadIdx.x];
                izs[threadIdx.x] = row_sum ? 1.f / row_sum[r * tau + i0 + threadIdx.x] : 0.f;
            }
            __syncthreads();
            for (int ii = 0; ii < n; ++ii) {
                const int i = i0 + ii;
                const float s = dot_lds<D>(qs + ii * D, kr) * scale;
                const bool valid = (j < mb) && (j <= mb - tb + i);
                const float dlt = s - ms[ii];
                if (valid) {
                    psi += exp2_fast(dlt * kLog2e) * izs[ii];
                    cnt += (dlt >= lnp) ? 1u : 0u;
                }
            }
        }
        if (nnz) {
            cnt = wave_allreduce_sum_u32(cnt);
            if (lane == 0 && cnt) atomicAdd(nnz + r, (unsigned long long)cnt);
        }
    }
    if (scores && j < m) scores[(size_t)rk * m + j] = psi;
}

__global__ void fill_u64_kernel(uint64_t* p, size_t n, uint64_t v) {
    const size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x < n) p[x] = v;
}

__global__ void gamma_kernel(const uint64_t* __restrict__ nnz, float* __restrict__ gamma, size_t n,
                             const int32_t* __restrict__ lens, int LHq, int m, int tau) {
    const size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= n) return;
    const ReqLen rl = request_len(lens, (int)(x / LHq), m, tau);
    const double region = (double)rl.tau * (rl.m - rl.tau) + (double)rl.tau * (rl.tau + 1) / 2.0;   // entries of the causal region, Alg. 1
    gamma[x] = (float)(1.0 - (double)nnz[x] / region);
}

template <typename T, int D>
hipError_t rowstats_impl(const ScoreArgs& a) {
    const vlc_shape& s = a.s;
    const int nchunks = (s.m + kScoreChunk - 1) / kScoreChunk;
    const size_t rows = (size_t)s.B * s.L * s.Hq * s.tau;
    const unsigned grid = (unsigned)nchunks * (unsigned)(s.B * s.L * s.Hq);
    rowstats_simple_kernel<T, D><<<grid, 256, 0, a.stream>>>(
        (const T*)a.q_win, (const T*)a.k, a.sm_scale, (float2*)a.workspace, s.L, s.Hq, s.Hkv, s.m, s.tau, nchunks, s.lens);
    rowstats_merge_kernel<<<(unsigned)((rows + 255) / 256), 256, 0, a.stream>>>(
        (const float2*)a.workspace, a.row_max, a.row_sum, rows, nchunks, a.nnz,
        a.nnz ? (size_t)s.B * s.L * s.Hq : 0, s.lens, s.L * s.Hq, s.m, s.tau);
    return hipGetLastError();
}

template <typename T, int D>
hipError_t colsweep_impl(const ScoreArgs& a) {
    const vlc_shape& s = a.s;
    const int nchunks = (s.m + kScoreChunk - 1) / kScoreChunk;
    const unsigned grid = (unsigned)nchunks * (unsigned)(s.B * s.L * s.Hkv);
    colsweep_simple_kernel<T, D><<<grid, 256, 0, a.stream>>>(
        (const T*)a.q_win, (const T*)a.k, a.sm_scale, a.row_max, a.row_sum, a.scores,
        (unsigned long long*)a.nnz, logf(a.p), s.L, s.Hq, s.Hkv, s.m, s.tau, s.lens);
    return hipGetLastError();
}

}  // namespace

size_t score_simple_workspace_bytes(const vlc_shape& s) {
    const size_t nchunks = (s.m + kScoreChunk - 1) / kScoreChunk;
    return (size_t)s.B * s.L * s.Hq * s.tau * nchunks * sizeof(float2);
}

#define VLC_DISPATCH(FN, a)                                                        \
    do {                                                                           \
        if ((a).s.dtype == VLC_F32) {                                              \
            if ((a).s.d == 64) return FN<float, 64>(a);                            \
            return FN<float, 128>(a);                                              \
        }                                                                          \
        if ((a).s.d == 64) return FN<bf16_t, 64>(a);                               \
        return FN<bf16_t, 128>(a);                                                 \
    } while (0)

hipError_t launch_rowstats_simple(const ScoreArgs& a) { VLC_DISPATCH(rowstats_impl, a); }
hipError_t launch_colsweep_simple(const ScoreArgs& a) { VLC_DISPATCH(colsweep_impl, a); }

hipError_t launch_fill_u64(uint64_t* p, size_t n, uint64_t v, hipStream_t st) {
    if (n == 0) return hipSuccess;
    fill_u64_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(p, n, v);
    return hipGetLastError();
}

hipError_t launch_gamma(const vlc_shape& s, const uint64_t* nnz, float* gamma, hipStream_t st) {
    const size_t n = (size_t)s.B * s.L * s.Hq;
    gamma_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(nnz, gamma, n, s.lens, s.L * s.Hq, s.m, s.tau);
    return hipGetLastError();
}

}  // namespace vlc
