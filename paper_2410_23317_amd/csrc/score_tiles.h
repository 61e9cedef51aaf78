// Tiles of the matrix-core sweeps over the post-vision window (gfx950, v_mfma_f32_32x32x16_bf16):
// operand fragments, K chunk staging through LDS and the accumulator layout, shared by the scoring
// sweeps and the window attention kernel.
#pragma once

#include "common.h"

namespace vlc {
namespace tiles {

constexpr int kD = 128;                 // head dimension of this path
constexpr int kChunk = 128;             // keys per LDS chunk
constexpr int kPitch = kD + 8;          // bf16 elements per LDS row (272 bytes: conflict-free 16-byte reads)
constexpr int kKSteps = kD / 16;        // MFMA k-steps per tile

// Fragment of one operand: lane (l % 32) owns a row (or column) index, lane half l / 32 the
// 8 consecutive k-values [16 ks + 8 half, +8).
__device__ __forceinline__ bf16x8_t as_frag(const uint4& v) { return __builtin_bit_cast(bf16x8_t, v); }

template <int WAVES, int RB, typename Args>
__device__ __forceinline__ void load_q_frags(const Args& a, int bl, int hkv, int wave, int lane, int tb, uint4 (&qf)[RB][kKSteps]) {
    const int half = lane >> 5;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int r = (a.rb0 + wave * RB + rb) * 32 + (lane & 31);
        const int hl = r / a.tauP, iw = r % a.tauP;
        const bool ok = hl < a.g && iw < tb;
        const bf16_t* row = a.q_win + (((size_t)bl * a.Hq + (size_t)hkv * a.g + (ok ? hl : 0)) * a.tau + (ok ? iw : 0)) * kD;
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks)
            qf[rb][ks] = ok ? *reinterpret_cast<const uint4*>(row + ks * 16 + half * 8) : make_uint4(0, 0, 0, 0);
    }
}

// K chunk staging: global -> registers -> LDS.  Keys at or beyond m are zero-filled.
template <int THREADS>
struct KStage {
    static constexpr int N = kChunk * (kD / 8) / THREADS;      // 16-byte pieces per thread
    uint4 r[N];
    __device__ __forceinline__ void load(const bf16_t* kg, int key0, int m) {
        if (key0 + kChunk <= m) {               // block-uniform: a whole chunk needs no per-row test
            const uint4* src = reinterpret_cast<const uint4*>(kg + (size_t)key0 * kD) + threadIdx.x;
#pragma unroll
            for (int u = 0; u < N; ++u) r[u] = src[THREADS * u];
            return;
        }
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const int x = threadIdx.x + THREADS * u;
            const int row = x >> 4, piece = x & 15;
            const int key = key0 + row;
            r[u] = (key < m) ? *reinterpret_cast<const uint4*>(kg + (size_t)key * kD + piece * 8) : make_uint4(0, 0, 0, 0);
        }
    }
    // The same in PARTS instalments (part P fetches pieces [P N / PARTS, (P + 1) N / PARTS)), for callers
    // that spread the requests of a chunk over their compute phases.
    template <int P, int PARTS>
    __device__ __forceinline__ void load_part(const bf16_t* kg, int key0, int m) {
        static_assert(N % PARTS == 0, "pieces per thread must divide evenly");
        const bool whole = key0 + kChunk <= m;
#pragma unroll
        for (int u = P * (N / PARTS); u < (P + 1) * (N / PARTS); ++u) {
            const int x = threadIdx.x + THREADS * u;
            const int row = x >> 4, piece = x & 15;
            const int key = key0 + row;
            if (whole) r[u] = *reinterpret_cast<const uint4*>(kg + (size_t)key * kD + piece * 8);
            else r[u] = (key < m) ? *reinterpret_cast<const uint4*>(kg + (size_t)key * kD + piece * 8) : make_uint4(0, 0, 0, 0);
        }
    }
    __device__ __forceinline__ void store(bf16_t* sK) const {
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const int x = threadIdx.x + THREADS * u;
            const int row = x >> 4, piece = x & 15;
            *reinterpret_cast<uint4*>(sK + row * kPitch + piece * 8) = r[u];
        }
    }
};

__device__ __forceinline__ void load_k_frags(const bf16_t* sK, int tile, int lane, uint4 (&kf)[kKSteps]) {
    const bf16_t* row = sK + (tile * 32 + (lane & 31)) * kPitch + (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks) kf[ks] = *reinterpret_cast<const uint4*>(row + ks * 16);
}

// Row index (0..31) of accumulator element i of a 32x32 MFMA tile in lane `lane`.
__device__ __forceinline__ int acc_row(int i, int lane) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }

}  // namespace tiles
}  // namespace vlc
