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

// ---- wave64 reductions through the data-parallel-primitive lane network (no LDS round trips) ----------------------
// Six combine steps: neighbours within quads (quad_perm [1,0,3,2], [2,3,0,1]), rotations by 4 and 8 within each row of
// 16 lanes, then the last lane of a row broadcast into the next row (row_bcast:15) and lane 31 into the upper half
// (row_bcast:31).  After them lane 63 holds the combination of all 64 lanes; it is handed to every lane through a
// scalar register.  All 64 lanes must be active.  The order of combination differs from a butterfly, which only
// matters for the rounding of floating-point sums.
template <int CTRL> __device__ __forceinline__ uint32_t dpp_move(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}
template <int CTRL> __device__ __forceinline__ float dpp_move(float v) { return __uint_as_float(dpp_move<CTRL>(__float_as_uint(v))); }
template <int CTRL> __device__ __forceinline__ int dpp_move(int v) { return (int)dpp_move<CTRL>((uint32_t)v); }
template <int CTRL> __device__ __forceinline__ double dpp_move(double v)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const uint32_t lo = dpp_move<CTRL>((uint32_t)b), hi = dpp_move<CTRL>((uint32_t)(b >> 32));
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
__device__ __forceinline__ float last_lane(float v) { return __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), 63)); }
__device__ __forceinline__ int last_lane(int v) { return __builtin_amdgcn_readlane(v, 63); }
__device__ __forceinline__ uint32_t last_lane(uint32_t v) { return (uint32_t)__builtin_amdgcn_readlane((int)v, 63); }
__device__ __forceinline__ double last_lane(double v)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, 63);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), 63);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

template <class T, class Op> __device__ __forceinline__ T wave_reduce(T v, Op op)
{
    v = op(v, dpp_move<0xB1>(v));      // quad_perm:[1,0,3,2]
    v = op(v, dpp_move<0x4E>(v));      // quad_perm:[2,3,0,1]
    v = op(v, dpp_move<0x124>(v));     // row_ror:4
    v = op(v, dpp_move<0x128>(v));     // row_ror:8
    v = op(v, dpp_move<0x142>(v));     // row_bcast:15
    v = op(v, dpp_move<0x143>(v));     // row_bcast:31
    return last_lane(v);
}

__device__ __forceinline__ float wave_max_f32(float v) { return wave_reduce(v, [](float a, float b) { return fmaxf(a, b); }); }
__device__ __forceinline__ float wave_sum_f32(float v) { return wave_reduce(v, [](float a, float b) { return a + b; }); }
__device__ __forceinline__ double wave_max_f64(double v) { return wave_reduce(v, [](double a, double b) { return fmax(a, b); }); }
__device__ __forceinline__ double wave_sum_f64(double v) { return wave_reduce(v, [](double a, double b) { return a + b; }); }
__device__ __forceinline__ int wave_sum_i32(int v) { return wave_reduce(v, [](int a, int b) { return a + b; }); }
__device__ __forceinline__ int wave_min_i32(int v) { return wave_reduce(v, [](int a, int b) { return a < b ? a : b; }); }

__device__ __forceinline__ int lane_id() { return __lane_id(); }

// value of `v` on lane `src`, where src is the same on every lane (a scalar read, no LDS round trip)
__device__ __forceinline__ int read_lane(int v, int src) { return __builtin_amdgcn_readlane(v, __builtin_amdgcn_readfirstlane(src)); }
__device__ __forceinline__ float read_lane(float v, int src) { return __uint_as_float((uint32_t)read_lane((int)__float_as_uint(v), src)); }
__device__ __forceinline__ double read_lane(double v, int src)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const uint32_t lo = (uint32_t)read_lane((int)(uint32_t)b, src), hi = (uint32_t)read_lane((int)(uint32_t)(b >> 32), src);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// number of set bits of a wave mask below this lane
__device__ __forceinline__ int mask_rank(unsigned long long m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

}  // namespace psmc
