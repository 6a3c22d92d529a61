// Device-side helpers for the gfx950 kernels: wave64 cross-lane reductions,
// 128-bit loads/stores of packed elements, dtype widening / narrowing.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace oqm {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct In_f32 {};
struct In_bf16 {};
struct In_f16 {};

// n / d for n < 2^32 and a run-time constant d >= 1 whose m = floor(2^32 / d) (2^32 - 1 for
// d == 1) came from the host: the high product is the quotient or one less.
__device__ __forceinline__ uint32_t div_by(uint32_t n, uint32_t d, uint32_t m) {
    const uint32_t q = __umulhi(n, m);
    return n - q * d >= d ? q + 1u : q;
}

// ---- DPP lane exchange ----------------------------------------------------
// dpp_ctrl encodings: quad_perm[1,0,3,2] = 0xB1 (lane ^ 1), quad_perm[2,3,0,1] = 0x4E
// (lane ^ 2), row_half_mirror = 0x141 (lane -> 7 - lane within 8), row_mirror = 0x140
// (lane -> 15 - lane within 16).  After the first two steps all four lanes of a quad hold
// the quad's result, so the mirrors combine whole quads / whole half-rows.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// All-reduce (min and max at once) over aligned sets of LANES lanes, LANES in {1,2,4,8,16}.
template <int LANES>
__device__ __forceinline__ void group_minmax(float& mn, float& mx) {
    if constexpr (LANES >= 2) {
        mn = fminf(mn, dpp_f32<0xB1>(mn));
        mx = fmaxf(mx, dpp_f32<0xB1>(mx));
    }
    if constexpr (LANES >= 4) {
        mn = fminf(mn, dpp_f32<0x4E>(mn));
        mx = fmaxf(mx, dpp_f32<0x4E>(mx));
    }
    if constexpr (LANES >= 8) {
        mn = fminf(mn, dpp_f32<0x141>(mn));
        mx = fmaxf(mx, dpp_f32<0x141>(mx));
    }
    if constexpr (LANES >= 16) {
        mn = fminf(mn, dpp_f32<0x140>(mn));
        mx = fmaxf(mx, dpp_f32<0x140>(mx));
    }
}

// Sum of a double over all 64 lanes of the wave (result valid in every lane).
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ---- loading 8 consecutive elements as float32 -----------------------------
// p must be 16-byte aligned.  Widening bf16 / f16 to float32 is exact.
__device__ __forceinline__ void load8(const void* p, In_bf16, float (&x)[8]) {
    const u32x4 w = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i] = __uint_as_float(w[i] << 16);
        x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

__device__ __forceinline__ void load8(const void* p, In_f16, float (&x)[8]) {
    const f16x8 h = *reinterpret_cast<const f16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (float)h[i];
}

__device__ __forceinline__ void load8(const void* p, In_f32, float (&x)[8]) {
    const f32x4 a = reinterpret_cast<const f32x4*>(p)[0];
    const f32x4 b = reinterpret_cast<const f32x4*>(p)[1];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[i] = a[i];
        x[4 + i] = b[i];
    }
}


// ---- raw (not yet widened) 8-element loads, for software-pipelined loops ----
template <typename T> struct Raw8;
template <> struct Raw8<In_bf16> { u32x4 a; };
template <> struct Raw8<In_f16> { f16x8 a; };
template <> struct Raw8<In_f32> { f32x4 a, b; };

__device__ __forceinline__ void load_raw(const void* p, Raw8<In_bf16>& r) {
    r.a = *reinterpret_cast<const u32x4*>(p);
}
__device__ __forceinline__ void load_raw(const void* p, Raw8<In_f16>& r) {
    r.a = *reinterpret_cast<const f16x8*>(p);
}
__device__ __forceinline__ void load_raw(const void* p, Raw8<In_f32>& r) {
    r.a = reinterpret_cast<const f32x4*>(p)[0];
    r.b = reinterpret_cast<const f32x4*>(p)[1];
}
__device__ __forceinline__ void zero_raw(Raw8<In_bf16>& r) { r.a = u32x4{0u, 0u, 0u, 0u}; }
__device__ __forceinline__ void zero_raw(Raw8<In_f16>& r) {
#pragma unroll
    for (int i = 0; i < 8; ++i) r.a[i] = (_Float16)0.0f;
}
__device__ __forceinline__ void zero_raw(Raw8<In_f32>& r) {
    r.a = f32x4{0.f, 0.f, 0.f, 0.f};
    r.b = r.a;
}
__device__ __forceinline__ void widen(const Raw8<In_bf16>& r, float (&x)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i] = __uint_as_float(r.a[i] << 16);
        x[2 * i + 1] = __uint_as_float(r.a[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void widen(const Raw8<In_f16>& r, float (&x)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (float)r.a[i];
}
__device__ __forceinline__ void widen(const Raw8<In_f32>& r, float (&x)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[i] = r.a[i];
        x[4 + i] = r.b[i];
    }
}

// ---- correctly rounded float32 a / 15 and 1 / s in three instructions each ----
// One FMA-residual correction step on top of a multiply by the rounded constant 1/15
// (resp. on top of v_rcp_f32).  The repository's division self-check program compares
// both against IEEE division for every input the quantizer can produce (all 2^31
// non-negative finite `a`; every normal `s` up to FLT_MAX / 15) on the GPU: no mismatch.
__device__ __forceinline__ float div15_exact(float a) {
    const float c = 1.0f / 15.0f;
    const float q = __fmul_rn(a, c);
    const float e = __builtin_fmaf(-15.0f, q, a);
    return __builtin_fmaf(e, c, q);
}
// a / 3 (2-bit codes have 3 steps) by the same construction; checked the same way.
__device__ __forceinline__ float div3_exact(float a) {
    const float c = 1.0f / 3.0f;
    const float q = __fmul_rn(a, c);
    const float e = __builtin_fmaf(-3.0f, q, a);
    return __builtin_fmaf(e, c, q);
}
// (max - min) / (2^BITS - 1)
template <int BITS>
__device__ __forceinline__ float div_levels_exact(float a) {
    if constexpr (BITS == 4) return div15_exact(a);
    else return div3_exact(a);
}
__device__ __forceinline__ float rcp_exact(float s) {
    const float r = __builtin_amdgcn_rcpf(s);
    const float e = __builtin_fmaf(-s, r, 1.0f);
    return __builtin_fmaf(e, r, r);
}

// t[i] = fma(x_i - m, 1/s, 2^23): the exact product is rounded once, to an integer,
// ties to even, and that integer sits in the low mantissa bits:
// bits(t) = 0x4B000000 | code.  Packs 8 codes, even channel in the low nibble.
__device__ __forceinline__ uint32_t pack8(const float (&t)[8]) {
    uint32_t m[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) m[i] = __float_as_uint(t[i]);
    // byte 0 of (m[2j+1] << 4 | m[2j]) is packed byte j; bits 8..23 of it are zero
    const uint32_t b01 = (m[1] << 4) | m[0];
    const uint32_t b23 = (m[3] << 4) | m[2];
    const uint32_t b45 = (m[5] << 4) | m[4];
    const uint32_t b67 = (m[7] << 4) | m[6];
    const uint32_t lo = (b23 << 8) | b01;  // bytes 0, 1 valid
    const uint32_t hi = (b67 << 8) | b45;
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);  // {lo.b0, lo.b1, hi.b0, hi.b1}
}


// 2-bit codes: channel u of the lane's 8 in bits [2u, 2u + 2) of a 16-bit word.  The
// exponent bits 0x4B000000 of every t stay at or above bit 24 under the left shifts.
__device__ __forceinline__ uint32_t pack8_2bit(const float (&t)[8]) {
    uint32_t w = __float_as_uint(t[0]);
#pragma unroll
    for (int i = 1; i < 8; ++i) w |= __float_as_uint(t[i]) << (2 * i);
    return w & 0xffffu;
}

// One lane's 8 codes: a 32-bit word (4-bit codes) or a 16-bit word (2-bit codes).
template <int BITS>
__device__ __forceinline__ void store_codes8(char* p, const float (&t)[8]) {
    if constexpr (BITS == 4) *reinterpret_cast<uint32_t*>(p) = pack8(t);
    else *reinterpret_cast<uint16_t*>(p) = (uint16_t)pack8_2bit(t);
}
template <int BITS>
__device__ __forceinline__ uint32_t load_codes8(const char* p) {
    if constexpr (BITS == 4) return *reinterpret_cast<const uint32_t*>(p);
    else return *reinterpret_cast<const uint16_t*>(p);
}

// 1 / s for a scale of BITS-bit codes.  With 15 steps s <= FLT_MAX / 15 < 2^126 and the
// quotient is always normal; with 3 steps s can exceed 2^126, where the quotient is
// sub-normal and the short sequence does not hold: those (astronomically wide) groups take
// the full IEEE division.
template <int BITS>
__device__ __forceinline__ float rcp_scale(float s) {
    if constexpr (BITS == 2) {
        if (s > 0x1p126f) return __fdiv_rn(1.0f, s);
    }
    return rcp_exact(s);
}

// ---- (scale, zero) pairs as stored: two float32, or two bfloat16 in one 32-bit word -------
template <bool BF16_META> struct MetaPair;
template <> struct MetaPair<false> { typedef f32x2 type; };
template <> struct MetaPair<true> { typedef uint32_t type; };

// Rounds (s, m) to bfloat16 (nearest even, one v_cvt_pk_bf16_f32), returns the stored word
// and replaces s and m by the rounded values, which is what the codes are then taken against.
__device__ __forceinline__ uint32_t round_pair_bf16(float& s, float& m) {
    const f32x2 v = {s, m};
    const uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    s = __uint_as_float(w << 16);
    m = __uint_as_float(w & 0xffff0000u);
    return w;
}
__device__ __forceinline__ f32x2 widen_pair(f32x2 p) { return p; }
__device__ __forceinline__ f32x2 widen_pair(uint32_t w) {
    return f32x2{__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u)};
}
// code + 2^23 clamped to [2^23, 2^23 + levels]: needed once the zero point is no longer the
// exact minimum (bfloat16 metadata); one v_med3_f32
template <int BITS>
__device__ __forceinline__ float clamp_code(float t) {
    return __builtin_amdgcn_fmed3f(t, 8388608.0f, 8388608.0f + (float)((1 << BITS) - 1));
}

template <typename T> struct elem_bytes;
template <> struct elem_bytes<In_f32> { static constexpr int value = 4; };
template <> struct elem_bytes<In_bf16> { static constexpr int value = 2; };
template <> struct elem_bytes<In_f16> { static constexpr int value = 2; };

// ---- storing 8 consecutive float32 values, narrowed round-to-nearest-even ---
__device__ __forceinline__ void store8(void* p, In_bf16, const float (&x)[8]) {
    u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const f32x2 v = {x[2 * i], x[2 * i + 1]};
        w[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));  // v_cvt_pk_bf16_f32
    }
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(p));
}

__device__ __forceinline__ void store8(void* p, In_f16, const float (&x)[8]) {
    f16x8 h;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // The value must be rounded to float32 first and to binary16 second; the empty asm
        // keeps the compiler from folding a producing FMA and this narrowing into one
        // mixed-precision instruction that rounds only once.
        float v = x[i];
        asm volatile("" : "+v"(v));
        h[i] = (_Float16)v;  // v_cvt_f16_f32, ties to even
    }
    __builtin_nontemporal_store(h, reinterpret_cast<f16x8*>(p));
}

__device__ __forceinline__ void store8(void* p, In_f32, const float (&x)[8]) {
    f32x4* o = reinterpret_cast<f32x4*>(p);
    const f32x4 a = {x[0], x[1], x[2], x[3]};
    const f32x4 b = {x[4], x[5], x[6], x[7]};
    __builtin_nontemporal_store(a, o);
    __builtin_nontemporal_store(b, o + 1);
}

}  // namespace oqm
