// Device-side random stream and wave64 helpers (gfx950).
//
// Philox4x32-10 as published by Salmon, Moraes, Dror, Shaw (SC'11): ten rounds of two 32x32->64 multiplies
// on counter words 0 and 2, a word permutation with key injection, and a Weyl bump of the key per round.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace psmc {

struct U4 { uint32_t x, y, z, w; };

// hardware base-2 exponential / logarithm (v_exp_f32 / v_log_f32, about 1 ulp, denormals flushed)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1)
{
    constexpr uint32_t MUL_A = 0xD2511F53u, MUL_B = 0xCD9E8D57u;
    constexpr uint32_t WEYL_A = 0x9E3779B9u, WEYL_B = 0xBB67AE85u;
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        const uint32_t a_hi = __umulhi(MUL_A, c0), a_lo = MUL_A * c0;
        const uint32_t b_hi = __umulhi(MUL_B, c2), b_lo = MUL_B * c2;
        c0 = b_hi ^ c1 ^ k0;
        c2 = a_hi ^ c3 ^ k1;
        c1 = b_lo;
        c3 = a_lo;
        k0 += WEYL_A;
        k1 += WEYL_B;
    }
    return U4{c0, c1, c2, c3};
}

__device__ __forceinline__ uint32_t pick_word(const U4& b, uint32_t w)
{
    return w == 0 ? b.x : (w == 1 ? b.y : (w == 2 ? b.z : b.w));
}

// Gumbel variate of a 32-bit word in fp32, absolute error of a few 1e-7:
// u = (x + 1/2)/2^32;  E = -ln u;  g = -ln E.  For u > 1/2, E is taken from w = 1 - u, formed exactly from the
// complemented word: a short series for small w, and a corrected logarithm of (1 - w) otherwise.
__device__ __forceinline__ float gumbel_f32(uint32_t x)
{
    constexpr float LN2 = 0.6931471805599453f;
    float E;
    if (x < 0x80000000u) {
        const float u = ((float)x + 0.5f) * 0x1p-32f;
        E = -LN2 * fast_log2(u);
    } else {
        const float w = ((float)(~x) + 0.5f) * 0x1p-32f;          // 1 - u in (0, 1/2]
        if (w < 0x1p-6f) {
            E = w * (1.0f + w * (0.5f + w * (0.33333334f + w * 0.25f)));
        } else {
            const float tt = 1.0f - w;                           // rounded
            const float corr = ((1.0f - tt) - w) / tt;           // log((1-w)/tt) to first order
            E = -(LN2 * fast_log2(tt) + corr);
        }
    }
    return -LN2 * fast_log2(E);
}

// Same variate in fp64 (used to re-rank the few finalists of a row).
__device__ __forceinline__ double gumbel_f64(uint32_t x)
{
    double E;
    if (x < 0x80000000u) {
        E = -log(((double)x + 0.5) * 0x1p-32);
    } else {
        E = -log1p(-(((double)(~x) + 0.5) * 0x1p-32));
    }
    return -log(E);
}

__device__ __forceinline__ float wave_max_f32(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum_f32(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ double wave_max_f64(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ int lane_id() { return __lane_id(); }

// number of set bits of a wave mask below this lane
__device__ __forceinline__ int mask_rank(unsigned long long m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

}  // namespace psmc
