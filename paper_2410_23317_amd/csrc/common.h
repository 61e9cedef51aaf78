// Device-side helpers shared by the VL-Cache kernels (gfx950 / CDNA4, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vlc {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kWave = 64;

typedef uint16_t bf16_t;                       // raw bfloat16 bits
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (inputs here are finite).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kPer16B = 4;
    __device__ static __forceinline__ float load(const float* p) { return *p; }
    __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static constexpr int kPer16B = 8;
    __device__ static __forceinline__ float load(const bf16_t* p) { return __uint_as_float(((uint32_t)*p) << 16); }
    __device__ static __forceinline__ void store(bf16_t* p, float v) { *p = (bf16_t)f32_to_bf16_bits(v); }
};

// Unpack one 16-byte chunk of storage into fp32 lanes.
__device__ __forceinline__ void unpack16(const uint4& v, float (&f)[4], const float*) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
}
__device__ __forceinline__ void unpack16(const uint4& v, float (&f)[8], const bf16_t*) {
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- data-parallel-primitive moves: lane permutations inside a 16-lane row -------------
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
constexpr int kDppRowRor(int n) { return 0x120 + n; }
constexpr int kDppQuadPerm(int a, int b, int c, int d) { return a | (b << 2) | (c << 4) | (d << 6); }
constexpr int kDppRowHalfMirror = 0x141;

// Sum over groups of LANES consecutive lanes; every lane of the group gets the total.
template <int LANES>
__device__ __forceinline__ float group_allreduce_sum(float x) {
    static_assert(LANES == 4 || LANES == 8 || LANES == 16 || LANES == 32 || LANES == 64, "group size");
    if constexpr (LANES == 16) {
        x += dpp_mov<kDppRowRor(8)>(x);
        x += dpp_mov<kDppRowRor(4)>(x);
        x += dpp_mov<kDppRowRor(2)>(x);
        x += dpp_mov<kDppRowRor(1)>(x);
    } else if constexpr (LANES == 8) {
        x += dpp_mov<kDppRowHalfMirror>(x);
        x += dpp_mov<kDppQuadPerm(1, 0, 3, 2)>(x);
        x += dpp_mov<kDppQuadPerm(2, 3, 0, 1)>(x);
    } else if constexpr (LANES == 4) {
        x += dpp_mov<kDppQuadPerm(1, 0, 3, 2)>(x);
        x += dpp_mov<kDppQuadPerm(2, 3, 0, 1)>(x);
    } else {
        for (int o = LANES / 2; o >= 1; o >>= 1) x += __shfl_xor(x, o, kWave);
    }
    return x;
}

// Max over groups of 8 or 16 consecutive lanes; every lane of the group gets the result.
template <int LANES>
__device__ __forceinline__ float group_allreduce_max(float x) {
    static_assert(LANES == 8 || LANES == 16, "group size");
    if constexpr (LANES == 16) {
        x = fmaxf(x, dpp_mov<kDppRowRor(8)>(x));
        x = fmaxf(x, dpp_mov<kDppRowRor(4)>(x));
        x = fmaxf(x, dpp_mov<kDppRowRor(2)>(x));
        x = fmaxf(x, dpp_mov<kDppRowRor(1)>(x));
    } else {
        x = fmaxf(x, dpp_mov<kDppRowHalfMirror>(x));
        x = fmaxf(x, dpp_mov<kDppQuadPerm(1, 0, 3, 2)>(x));
        x = fmaxf(x, dpp_mov<kDppQuadPerm(2, 3, 0, 1)>(x));
    }
    return x;
}

// ---- FP8 (OCP E4M3) rows with one fp32 scale per row -----------------------------------
// Quantise the 8 bf16 values a lane holds of a row whose LPR lanes are consecutive:
// scale = absmax(row) / 448 (1 for an all-zero row), code = E4M3 nearest to fp32(x / scale),
// ties to even (v_cvt_pk_fp8_f32), magnitudes clamped to 448.  Byte e of the result is element e.
template <int LPR>
__device__ __forceinline__ uint2 quantize_row_e4m3(const uint4& v, float& scale) {
    float f[8];
    unpack16(v, f, (const bf16_t*)nullptr);
    float amax = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(f[e]));
    amax = group_allreduce_max<LPR>(amax);
    scale = amax > 0.f ? amax / 448.0f : 1.0f;
    float y[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = fminf(fmaxf(f[e] / scale, -448.0f), 448.0f);
    int lo = 0, hi = 0;
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
    return make_uint2((uint32_t)lo, (uint32_t)hi);
}

// 8 E4M3 codes -> 8 bf16 values (exact: E4M3 has 3 mantissa bits), packed like a 16-byte bf16 chunk.
__device__ __forceinline__ uint4 e4m3x8_to_bf16x8(const uint2& r) {
    const auto a = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.x, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.x, true);
    const auto c = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.y, false), d = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.y, true);
    // upper halves of two fp32 words -> one word of two bf16 (first element in the low half)
    auto pack = [](float lo, float hi) { return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u); };
    return make_uint4(pack(a[0], a[1]), pack(b[0], b[1]), pack(c[0], c[1]), pack(d[0], d[1]));
}

__device__ __forceinline__ float wave_allreduce_max(float x) {
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, kWave));
    return x;
}
__device__ __forceinline__ float wave_allreduce_sum(float x) {
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, kWave);
    return x;
}
__device__ __forceinline__ uint32_t wave_allreduce_sum_u32(uint32_t x) {
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, kWave);
    return x;
}

// Prompt length and window length of request b: the shape's m and tau, or the request's own pair
// from the optional per-request array, clamped into [1, m] and [1, min(tau, m_b)] so that no
// kernel indexes outside the padded tensors whatever the array holds.
struct ReqLen { int m, tau; };
__device__ __forceinline__ ReqLen request_len(const int32_t* __restrict__ lens, int b, int m, int tau) {
    ReqLen r{m, tau};
    if (lens) {
        r.m = min(max(lens[2 * b], 1), m);
        r.tau = min(max(lens[2 * b + 1], 1), min(tau, r.m));
    }
    return r;
}

// Device-visible sticky error: first writer wins.
__device__ __forceinline__ void set_sticky(int32_t* status, int code, int b, int l, int detail) {
    if (atomicCAS(status, 0, code) == 0) { status[1] = b; status[2] = l; status[3] = detail; }
}

}  // namespace vlc
