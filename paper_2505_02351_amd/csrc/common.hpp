// Device-side helpers shared by the optgqa kernels: 2-byte float handling and wave64 lane exchange.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace optgqa {

constexpr int kF16 = 0;
constexpr int kBF16 = 1;
constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Widen the low / high 2-byte element of a packed dword to fp32 (exact).
template <int DT> __device__ __forceinline__ float widen_lo(uint32_t u);
template <int DT> __device__ __forceinline__ float widen_hi(uint32_t u);
template <> __device__ __forceinline__ float widen_lo<kBF16>(uint32_t u) { return __uint_as_float(u << 16); }
template <> __device__ __forceinline__ float widen_hi<kBF16>(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
template <> __device__ __forceinline__ float widen_lo<kF16>(uint32_t u)
{
    return (float)__builtin_bit_cast(f16x2, u).x;
}
template <> __device__ __forceinline__ float widen_hi<kF16>(uint32_t u)
{
    return (float)__builtin_bit_cast(f16x2, u).y;
}

// acc + a.lo*b.lo + a.hi*b.hi with the products and the sum kept in fp32 (v_dot2c_f32_*).
template <int DT> __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc);
template <> __device__ __forceinline__ float dot2<kF16>(uint32_t a, uint32_t b, float acc)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, a), __builtin_bit_cast(f16x2, b), acc, false);
}
template <> __device__ __forceinline__ float dot2<kBF16>(uint32_t a, uint32_t b, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
}

// One rounding, nearest-even, fp32 -> 2-byte pattern.
template <int DT> __device__ __forceinline__ uint16_t narrow(float x);
template <> __device__ __forceinline__ uint16_t narrow<kF16>(float x)
{
    return __builtin_bit_cast(uint16_t, (_Float16)x);
}
template <> __device__ __forceinline__ uint16_t narrow<kBF16>(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // keep NaN a NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
// Two values at once: gfx950 has single-instruction packed conversions (v_cvt_pk_bf16_f32,
// v_cvt_pk_f16_f32), both round-to-nearest-even and NaN-preserving.
template <int DT> __device__ __forceinline__ uint32_t narrow2(float lo, float hi);
template <> __device__ __forceinline__ uint32_t narrow2<kF16>(float lo, float hi)
{
    const f16x2 r = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, r);
}
template <> __device__ __forceinline__ uint32_t narrow2<kBF16>(float lo, float hi)
{
    const bf16x2 r = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, r);
}

// Two fp32 softmax weights as a pair of bf16 heads and a pair of bf16 tails, head + tail = weight to
// 2^-16 relative: the head is the fp32 value cut to its upper 16 bits (exactly a bf16 number, one
// byte permute for the pair), the tail the rounded remainder (exact subtraction).  Six vector
// instructions per pair; rounding the head to nearest instead costs two more and buys nothing, since
// the tail carries what the head leaves.
__device__ __forceinline__ void split_bf16(float w0, float w1, uint32_t& head, uint32_t& tail)
{
    const uint32_t b0 = __float_as_uint(w0), b1 = __float_as_uint(w1);
    head = __builtin_amdgcn_perm(b1, b0, 0x07060302u);           // {b0 >> 16, b1 >> 16}
    tail = narrow2<kBF16>(w0 - __uint_as_float(b0 & 0xffff0000u), w1 - __uint_as_float(b1 & 0xffff0000u));
}

// Data-parallel-primitive lane exchange inside a row of 16 lanes (full VALU rate, no LDS).
template <int CTRL> __device__ __forceinline__ float dpp(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each half row
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each row
constexpr int kDppRowRor4 = 0x124;    // row_ror:4
constexpr int kDppRowRor8 = 0x128;
constexpr int kDppRowRor12 = 0x12C;

// Sum over the LPR (8 or 16) consecutive lanes that share a token row; every lane gets the sum.
template <int LPR> __device__ __forceinline__ float row_group_sum(float x)
{
    x += dpp<kDppXor1>(x);
    x += dpp<kDppXor2>(x);
    x += dpp<kDppHalfMirror>(x);
    if (LPR == 16) x += dpp<kDppMirror>(x);
    return x;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef float f32x2 __attribute__((ext_vector_type(2)));

// eight E4M3 codes (two dwords) -> eight DT values (one MFMA operand), exactly: every E4M3 value is
// an fp16 and a bf16 number.  One instruction per pair (gfx950's scaled conversion with scale 1;
// checked on the device for all 256 codes against the two-step conversion through fp32).
template <int DT> __device__ __forceinline__ uint32_t widen2_e4m3(uint32_t codes, bool upper_half);
template <> __device__ __forceinline__ uint32_t widen2_e4m3<kF16>(uint32_t codes, bool upper_half)
{
    return upper_half ? __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(codes, 1.0f, true))
                      : __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(codes, 1.0f, false));
}
template <> __device__ __forceinline__ uint32_t widen2_e4m3<kBF16>(uint32_t codes, bool upper_half)
{
    return upper_half ? __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes, 1.0f, true))
                      : __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes, 1.0f, false));
}
template <int DT> __device__ __forceinline__ uint4 widen8_e4m3(uint32_t lo, uint32_t hi)
{
    return make_uint4(widen2_e4m3<DT>(lo, false), widen2_e4m3<DT>(lo, true), widen2_e4m3<DT>(hi, false), widen2_e4m3<DT>(hi, true));
}

// Streaming loads: K / V tiles of a decode step are read once and never again, and the
// non-temporal hint is worth ~15 % of bandwidth on this chip (measured: 6.6-6.8 TB/s against
// 5.7-5.9 TB/s for the same random 4-8 KiB pieces with plain loads).
#ifndef OPTGQA_STREAM_NT
#define OPTGQA_STREAM_NT 1
#endif
__device__ __forceinline__ uint4 stream_load16(const void* p)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#if OPTGQA_STREAM_NT
    const u32x4 v = __builtin_nontemporal_load(static_cast<const u32x4*>(p));
#else
    const u32x4 v = *static_cast<const u32x4*>(p);
#endif
    return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ uint2 stream_load8(const void* p)
{
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#if OPTGQA_STREAM_NT
    const u32x2 v = __builtin_nontemporal_load(static_cast<const u32x2*>(p));
#else
    const u32x2 v = *static_cast<const u32x2*>(p);
#endif
    return make_uint2(v[0], v[1]);
}

// two fp32 values -> two E4M3 codes (bits 0..15): round to nearest even; the hardware conversion
// turns magnitudes beyond the format's range into NaN, so the values are clamped to +-448 first
// (saturation), and a NaN input is given the code 0x7f explicitly
__device__ __forceinline__ uint32_t e4m3_codes2(float a, float b)
{
    const float ac = fminf(fmaxf(a, -448.f), 448.f), bc = fminf(fmaxf(b, -448.f), 448.f);
    uint32_t two = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(ac, bc, 0, false) & 0xffffu;
    if (a != a) two = (two & 0xff00u) | 0x7fu;
    if (b != b) two = (two & 0x00ffu) | 0x7f00u;
    return two;
}

}  // namespace optgqa
