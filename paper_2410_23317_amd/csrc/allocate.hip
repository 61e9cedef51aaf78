// Sparsity-aware layer budgets (paper Alg. 1, SkewedCacheBudgetAllocation) in integer arithmetic.
// 1 - gamma'_l is proportional to n_l = sum_h nnz[l][h], so beta_l * m = n_l / N * alpha * L * m.
// The whole budget B_tot is apportioned by largest remainder and then clipped to
// [max(1, ceil(m/100)), m], the token form of the paper's clip(beta, 0.01, 1).
#include "common.h"
#include "internal.h"

namespace vlc {
namespace {

// One block per request; thread t owns layers t, t + blockDim, ...  (L <= kMaxLayers).
__global__ __launch_bounds__(256) void allocate_kernel(const uint64_t* __restrict__ nnz, int L, int Hq, int m_max, int tau,
                                                       uint64_t alpha_num, uint64_t alpha_den,
                                                       const int32_t* __restrict__ lens, int32_t* __restrict__ k_out,
                                                       float* __restrict__ beta_out) {
    __shared__ uint64_t n_l[kMaxLayers];
    __shared__ uint64_t rem[kMaxLayers];
    __shared__ uint64_t quo[kMaxLayers];
    __shared__ uint64_t red[256];
    const int b = blockIdx.x;
    const int t = threadIdx.x;
    const int m = request_len(lens, b, m_max, tau).m;                       // this request's prompt length
    const uint64_t B_tot = alpha_num * (uint64_t)L * (uint64_t)m / alpha_den;   // floor(alpha L m) tokens for the request
    uint64_t local = 0;
    for (int l = t; l < L; l += blockDim.x) {
        uint64_t s = 0;
        for (int h = 0; h < Hq; ++h) s += nnz[((size_t)b * L + l) * Hq + h];
        n_l[l] = s;
        local += s;
    }
    red[t] = local;
    __syncthreads();
    for (int o = 128; o >= 1; o >>= 1) {
        if (t < o) red[t] += red[t + o];
        __syncthreads();
    }
    const uint64_t N = red[0];
    __syncthreads();
    local = 0;
    for (int l = t; l < L; l += blockDim.x) {
        uint64_t q, r;
        if (N == 0) { q = B_tot / (uint64_t)L; r = 0; }
        else { const uint64_t prod = n_l[l] * B_tot; q = prod / N; r = prod % N; }
        quo[l] = q;
        rem[l] = r;
        local += q;
    }
    red[t] = local;
    __syncthreads();
    for (int o = 128; o >= 1; o >>= 1) {
        if (t < o) red[t] += red[t + o];
        __syncthreads();
    }
    const uint64_t extra = B_tot - red[0];          // < L tokens left after the floor quotas
    const int lo = max(1, (m + 99) / 100);
    for (int l = t; l < L; l += blockDim.x) {
        // rank of layer l by (remainder descending, layer ascending)
        uint64_t rank = 0;
        const uint64_t r = rem[l];
        for (int x = 0; x < L; ++x) rank += (rem[x] > r || (rem[x] == r && x < l)) ? 1u : 0u;
        uint64_t q = quo[l] + (rank < extra ? 1u : 0u);
        if (q < (uint64_t)lo) q = lo;
        if (q > (uint64_t)m) q = m;
        k_out[(size_t)b * L + l] = (int32_t)q;
        if (beta_out) beta_out[(size_t)b * L + l] = (float)((double)q / (double)m);
    }
}

}  // namespace

hipError_t launch_allocate(const vlc_shape& s, const uint64_t* nnz, int64_t alpha_num, int64_t alpha_den, int32_t* k_out,
                           float* beta_out, hipStream_t st) {
    allocate_kernel<<<s.B, 256, 0, st>>>(nnz, s.L, s.Hq, s.m, s.tau, (uint64_t)alpha_num, (uint64_t)alpha_den, s.lens,
                                         k_out, beta_out);
    return hipGetLastError();
}

}  // namespace vlc
