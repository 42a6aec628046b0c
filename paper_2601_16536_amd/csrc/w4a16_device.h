// Device-side pieces shared by the multiply kernels: operand types, the int4
// unpack, and the fp32 application of scale and zero point (Eq. 2).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace w4a16 {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));

union H2 {
    uint32_t u;
    half2_t h;
};
union H8 {
    uint4_t u;
    half8_t h;
};

constexpr int kPrefetch = 2;                   // units of weights in flight per wave beyond the one in use
constexpr uint32_t kOutOfRange = 0x80000000u;  // per-lane buffer offset beyond any slice: the load returns 0, no traffic
constexpr uint32_t kRawBuffer = 0x00020000u;   // buffer descriptor word 3: raw 32-bit data, no swizzle

// Nibble masks, kept opaque so they stay in scalar registers and each mask is one v_and_b32
// (as literals they would be re-materialised per use).
struct Masks {
    uint32_t lo, hi;  // 0x000F000F, 0x00F000F0
};
__device__ __forceinline__ Masks make_masks()
{
    Masks m;
    m.lo = 0x000F000Fu;
    m.hi = 0x00F000F0u;
    asm volatile("" : "+s"(m.lo), "+s"(m.hi));
    return m;
}

// One 32-bit word holds the codes of k = 8r .. 8r+7 of one column.  A nibble left
// in place in bits 0-3 of an otherwise zero fp16 IS the subnormal number q 2^-24,
// in bits 4-7 it is q 2^-20; the MFMA takes subnormal inputs exactly.  So four
// masks (two of them after a shift by 8) give the lane's eight B-operand halves:
// k order 0,4 | 1,5 | 2,6 | 3,7 with weights 2^-24, 2^-20, 2^-24, 2^-20.  X is
// staged in the same k order with the 2^-20 positions divided by 16.
__device__ __forceinline__ half8_t unpack8(uint32_t w, const Masks &k)
{
    const uint32_t w8 = w >> 8;
    H8 r;
    r.u = (uint4_t){w & k.lo, w & k.hi, w8 & k.lo, w8 & k.hi};
    return r.h;
}

// The eight halves of one packed row of X in unpack order, the bits-4-7 positions scaled by 1/16.
__device__ __forceinline__ uint4_t permute_x(uint4_t d)
{
    const half2_t sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    H2 p0, p1, p2, p3;
    // byte selectors of v_perm_b32: 0-3 pick from the second operand, 4-7 from the first
    p0.u = __builtin_amdgcn_perm(d[2], d[0], 0x05040100u);  // x0, x4
    p1.u = __builtin_amdgcn_perm(d[2], d[0], 0x07060302u);  // x1, x5
    p2.u = __builtin_amdgcn_perm(d[3], d[1], 0x05040100u);  // x2, x6
    p3.u = __builtin_amdgcn_perm(d[3], d[1], 0x07060302u);  // x3, x7
    p1.h = p1.h * sixteenth;
    p3.h = p3.h * sixteenth;
    return (uint4_t){p0.u, p1.u, p2.u, p3.u};
}

__device__ __forceinline__ float sum8(uint4_t d)
{
    H8 v;
    v.u = d;
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) s += (float)v.h[e];
    return s;
}

// With P = 2^-24 sum_k x_k q_k over one unit of k inside a quantisation group
// (fp32, from the MFMA) and xsum = sum_k x_k, Eq. 2 gives the unit's contribution
//   sum_k x_k s (q_k - z) = (2^24 s) P - (s z) xsum.
__device__ __forceinline__ float apply_scale_zero(float tot, float s, float z, float P, float xsum)
{
    return __builtin_fmaf(s * 16777216.0f, P, __builtin_fmaf(-s * z, xsum, tot));
}

// Symmetric quantisation (Section 2.1: z = 0 on signed codes, i.e. 8 on the stored unsigned codes) comes without a
// zero-point tensor.  The kernels then read their zero-point words through a buffer of size 0 (every load is out
// of range: it returns 0 and moves nothing) and OR this word in: eight zero points of 8.
__device__ __forceinline__ uint32_t symmetric_fill(const uint32_t *Zp) { return Zp ? 0u : 0x88888888u; }
__device__ __forceinline__ uint32_t zero_point_bytes(const uint32_t *Zp, uint32_t bytes) { return Zp ? bytes : 0u; }

__device__ __forceinline__ uint32_t pack_half2(float a, float b)
{
    H2 p;
    p.h = (half2_t){(_Float16)a, (_Float16)b};
    return p.u;
}

// ---- the 16-bit format of A and of the output ----
//
// Everything that depends on it sits behind one of two types.  With P the MFMA's sum over a unit of k of
// (staged x_k) * (operand built from q_k), and xsum = sum_k x_k, the unit's contribution to Eq. 2 is
//     sum_k x_k s (q_k - z) = (kCodeScale s) P - s (z + kCodeOffset) xsum.
//
// FP16 (the paper's format): the operand is the code left in place as a subnormal, q 2^-24 or q 2^-20 with x
// staged divided by 16 (unpack8 above): kCodeScale = 2^24, kCodeOffset = 0.
struct ActF16 {
    static constexpr bool kBF16 = false;
    static constexpr float kCodeScale = 16777216.0f;
    static constexpr float kCodeOffset = 0.0f;
    typedef half8_t operand_t;
    static __device__ __forceinline__ operand_t unpack(uint32_t w, const Masks &k) { return unpack8(w, k); }
    static __device__ __forceinline__ uint4_t stage_x(uint4_t d) { return permute_x(d); }
    static __device__ __forceinline__ float sum_x(uint4_t d) { return sum8(d); }
    static __device__ __forceinline__ operand_t x_operand(uint4_t d)
    {
        H8 v;
        v.u = d;
        return v.h;
    }
    // the operand against which the staged x sum to sum_k x_k
    static __device__ __forceinline__ operand_t ones()
    {
        return (half8_t){(_Float16)1.f, (_Float16)1.f, (_Float16)16.f, (_Float16)16.f, (_Float16)1.f, (_Float16)1.f, (_Float16)16.f, (_Float16)16.f};
    }
    static __device__ __forceinline__ float4_t mfma(operand_t x, operand_t b, float4_t c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(x, b, c, 0, 0, 0); }
    static __device__ __forceinline__ uint32_t pack2(float a, float b) { return pack_half2(a, b); }
    static constexpr uint16_t kNaN = 0x7E00u;
};

// BF16.  A bfloat16 has no room for the subnormal trick (the products with x would be FP32 subnormals), so the
// operand is 128 + q: the code ORed into the low fraction bits of 128.0 (0x4300, whose unit in the last place is 1).
// P then carries 128 xsum too much, which the zero-point term takes back: kCodeScale = 1, kCodeOffset = 128.
// Products of two bfloat16 are exact in FP32; the sum of a unit, about 128 times larger than it needs to be,
// costs about 7 of FP32's 24 bits, which leaves more than the 8 bits of the output.
typedef __bf16 bfloat8_t __attribute__((ext_vector_type(8)));
struct ActBF16 {
    static constexpr bool kBF16 = true;
    static constexpr float kCodeScale = 1.0f;
    static constexpr float kCodeOffset = 128.0f;
    typedef bfloat8_t operand_t;
    union B8 {
        uint4_t u;
        bfloat8_t b;
    };
    // k order 0,4 | 1,5 | 2,6 | 3,7 as in the FP16 form; every code moved to bits 0-3 of its half
    static __device__ __forceinline__ operand_t unpack(uint32_t w, const Masks &k)
    {
        const uint32_t base = 0x43004300u;
        B8 r;
        r.u = (uint4_t){(w & k.lo) | base, ((w >> 4) & k.lo) | base, ((w >> 8) & k.lo) | base, ((w >> 12) & k.lo) | base};
        return r.b;
    }
    static __device__ __forceinline__ uint4_t stage_x(uint4_t d)
    {
        return (uint4_t){__builtin_amdgcn_perm(d[2], d[0], 0x05040100u), __builtin_amdgcn_perm(d[2], d[0], 0x07060302u),
                         __builtin_amdgcn_perm(d[3], d[1], 0x05040100u), __builtin_amdgcn_perm(d[3], d[1], 0x07060302u)};
    }
    static __device__ __forceinline__ float sum_x(uint4_t d)
    {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) s += __builtin_bit_cast(float, d[e] << 16) + __builtin_bit_cast(float, d[e] & 0xFFFF0000u);
        return s;
    }
    static __device__ __forceinline__ operand_t x_operand(uint4_t d)
    {
        B8 v;
        v.u = d;
        return v.b;
    }
    static __device__ __forceinline__ operand_t ones()
    {
        B8 v;
        v.u = (uint4_t){0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
        return v.b;
    }
    static __device__ __forceinline__ float4_t mfma(operand_t x, operand_t b, float4_t c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, b, c, 0, 0, 0); }
    // round to nearest even (the hardware's v_cvt_pk_bf16_f32)
    static __device__ __forceinline__ uint32_t pack2(float a, float b)
    {
        typedef __bf16 bfloat2_t __attribute__((ext_vector_type(2)));
        const bfloat2_t p = {(__bf16)a, (__bf16)b};
        return __builtin_bit_cast(uint32_t, p);
    }
    static constexpr uint16_t kNaN = 0x7FC0u;
};

}  // namespace w4a16
