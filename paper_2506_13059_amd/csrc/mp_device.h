// Device-side helpers shared by the gfx950 kernels: wave64 cross-lane primitives and bf16 bit tricks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mp {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

constexpr int kHeadDim = 128;
constexpr int kWave = 64;

// ---- bf16 <-> fp32 (bit level; a bf16 is the upper half of an fp32) ---------------------------
__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// Non-temporal loads and stores, for data a kernel touches once (whole cache lines per instruction):
// the line is not kept for a second use, which on this part moves a stream 7-12 % faster.
typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint32_t load_once(const uint32_t* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ uint4 load_once(const uint4* p)
{
    const u32x4_nt t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void store_once(uint4* p, const uint4& v)
{
    u32x4_nt t;
    t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    __builtin_nontemporal_store(t, reinterpret_cast<u32x4_nt*>(p));
}

// fp32 -> bf16, round to nearest even (NaN kept quiet).
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t x = __float_as_uint(f);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x40u);
    uint32_t lsb = (x >> 16) & 1u;
    x += 0x7fffu + lsb;
    return (uint16_t)(x >> 16);
}

// fp64 -> bf16 with ONE rounding (nearest even).  The double is first truncated to fp32 with a
// sticky bit in the last place (round to odd), which makes the second rounding exact.  Values
// whose magnitude is below 2^-126 go to signed zero; overflow goes to infinity.
__device__ __forceinline__ uint16_t f64_to_bf16_rne(double v)
{
    uint64_t b = (uint64_t)__double_as_longlong(v);
    uint32_t sign = (uint32_t)(b >> 63) << 31;
    int32_t e = (int32_t)((b >> 52) & 0x7ff);
    uint64_t man = b & 0xfffffffffffffull;
    if (e == 0x7ff) {                                   // inf / nan
        uint32_t x = sign | 0x7f800000u | (man ? 0x400000u : 0u);
        return (uint16_t)(x >> 16);
    }
    int32_t fe = e - 1023 + 127;
    if (fe <= 0) return (uint16_t)(sign >> 16);         // below the fp32 normal range (incl. zero)
    if (fe >= 255) return (uint16_t)((sign | 0x7f800000u) >> 16);
    uint32_t m23 = (uint32_t)(man >> 29);
    uint32_t sticky = (man & ((1ull << 29) - 1)) ? 1u : 0u;
    uint32_t x = sign | ((uint32_t)fe << 23) | m23 | sticky;
    uint32_t lsb = (x >> 16) & 1u;
    uint32_t mag = (x & 0x7fffffffu) + 0x7fffu + lsb;   // may carry into the exponent: correct
    if (mag >= 0x7f800000u) mag = 0x7f800000u;
    return (uint16_t)((sign | mag) >> 16);
}

// a.x*b.x + a.y*b.y + c on packed bf16 pairs (v_dot2c_f32_bf16)
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

// e^x in fp64 for the arguments a shifted log-sum-exp produces: x <= 0 up to rounding of the shift
// (any x below about 700 is fine), -inf allowed (gives 0).  x = k ln2 + r with |r| <= ln2 / 2, e^r by its
// Taylor polynomial of degree 12 (remainder below 2e-16 of the value), scaled by 2^k with ldexp.
// About a third of the instructions of the general-purpose routine; relative error below 1e-15.
__device__ __forceinline__ double exp_shifted(double x)
{
    x = fmax(x, -800.0);                                   // e^-800 is zero in fp64; keeps k finite
    const double kf = __builtin_rint(x * 1.4426950408889634074);
    double r = fma(kf, -6.93147180369123816490e-01, x);    // ln2 in two parts
    r = fma(kf, -1.90821492927058770002e-10, r);
    double p = 2.08767569878680989792e-09;                 // 1/12!
    p = fma(p, r, 2.50521083854417187751e-08);             // 1/11!
    p = fma(p, r, 2.75573192239858906526e-07);             // 1/10!
    p = fma(p, r, 2.75573192239858906526e-06);             // 1/9!
    p = fma(p, r, 2.48015873015873015873e-05);             // 1/8!
    p = fma(p, r, 1.98412698412698412698e-04);             // 1/7!
    p = fma(p, r, 1.38888888888888888889e-03);             // 1/6!
    p = fma(p, r, 8.33333333333333333333e-03);             // 1/5!
    p = fma(p, r, 4.16666666666666666667e-02);             // 1/4!
    p = fma(p, r, 1.66666666666666666667e-01);             // 1/3!
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(p, (int)kf);
}

// ---- DPP cross-lane moves inside a row of 16 lanes ----------------------------------------------
template <int kCtrl>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), kCtrl, 0xf, 0xf, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each half row
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each row

// Sum over aligned groups of 8 lanes; every lane of the group receives the total.
__device__ __forceinline__ float sum8(float v)
{
    v += dpp_f32<kDppXor1>(v);
    v += dpp_f32<kDppXor2>(v);
    v += dpp_f32<kDppHalfMirror>(v);
    return v;
}
// Sum over aligned groups of 4 lanes.
__device__ __forceinline__ float sum4(float v)
{
    v += dpp_f32<kDppXor1>(v);
    v += dpp_f32<kDppXor2>(v);
    return v;
}

template <int kCtrl>
__device__ __forceinline__ double dpp_f64(double v)
{
    long long b = __double_as_longlong(v);
    int lo = __builtin_amdgcn_mov_dpp((int)(b & 0xffffffffll), kCtrl, 0xf, 0xf, true);
    int hi = __builtin_amdgcn_mov_dpp((int)(b >> 32), kCtrl, 0xf, 0xf, true);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
__device__ __forceinline__ double sum4_f64(double v)
{
    v += dpp_f64<kDppXor1>(v);
    v += dpp_f64<kDppXor2>(v);
    return v;
}

// ---- whole-wave helpers (wave64), built from DPP row operations ----------------------------------
__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// DPP move that leaves 0 in lanes without a source lane or outside kRowMask.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ uint32_t dpp_u32_or0(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kCtrl, kRowMask, 0xf, false);
}
// Inclusive prefix sum over the 64 lanes: shifts by 1, 2, 4, 8 inside each row of 16, then the last
// lane of row 0 / row 2 is added to the following row and the last lane of the lower half to the
// upper half (row_bcast15 / row_bcast31).
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v)
{
    v += dpp_u32_or0<0x111, 0xf>(v);
    v += dpp_u32_or0<0x112, 0xf>(v);
    v += dpp_u32_or0<0x114, 0xf>(v);
    v += dpp_u32_or0<0x118, 0xf>(v);
    v += dpp_u32_or0<0x142, 0xa>(v);
    v += dpp_u32_or0<0x143, 0xc>(v);
    return v;
}
__device__ __forceinline__ double readlane_f64(double v, int src)
{
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane((int)(b & 0xffffffffll), src);
    const int hi = __builtin_amdgcn_readlane((int)(b >> 32), src);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
// Reductions over a row of 16 lanes; every lane of the row receives the result.
__device__ __forceinline__ double row_sum_f64(double v)
{
    v += dpp_f64<kDppXor1>(v);
    v += dpp_f64<kDppXor2>(v);
    v += dpp_f64<kDppHalfMirror>(v);
    v += dpp_f64<kDppMirror>(v);
    return v;
}
__device__ __forceinline__ double row_max_f64(double v)
{
    v = fmax(v, dpp_f64<kDppXor1>(v));
    v = fmax(v, dpp_f64<kDppXor2>(v));
    v = fmax(v, dpp_f64<kDppHalfMirror>(v));
    v = fmax(v, dpp_f64<kDppMirror>(v));
    return v;
}
__device__ __forceinline__ float row_max_f32(float v)
{
    v = fmaxf(v, dpp_f32<kDppXor1>(v));
    v = fmaxf(v, dpp_f32<kDppXor2>(v));
    v = fmaxf(v, dpp_f32<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_f32<kDppMirror>(v));
    return v;
}
// Whole-wave reductions; the result is wave-uniform.
__device__ __forceinline__ double wave_sum_f64(double v)
{
    v = row_sum_f64(v);
    return (readlane_f64(v, 0) + readlane_f64(v, 16)) + (readlane_f64(v, 32) + readlane_f64(v, 48));
}
__device__ __forceinline__ float wave_max_f32(float v)
{
    v = row_max_f32(v);
    const int b = __float_as_int(v);
    const float a0 = __int_as_float(__builtin_amdgcn_readlane(b, 0)), a1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
    const float a2 = __int_as_float(__builtin_amdgcn_readlane(b, 32)), a3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
    return fmaxf(fmaxf(a0, a1), fmaxf(a2, a3));
}

}  // namespace mp
