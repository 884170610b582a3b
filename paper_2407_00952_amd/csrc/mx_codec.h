// MXFP8 element / scale codec shared by the conversion kernels and by the kernels that read or write
// compressed cut-layer buffers (OCP Microscaling Formats v1.0: FP8 E4M3 elements, bias 7, largest finite
// value 448, S.1111.111 = NaN; E8M0 block scale = 2^(code - 127); conversion per Sec. 6.3 of that document).
#pragma once
#include <hip/hip_runtime.h>

// E4M3 code of a non-negative fp32 value below 512: round to nearest, ties to even, clamp at 448.
static __device__ __forceinline__ unsigned mx_e4m3_from_f32(float a)
{
    a = fminf(a, 448.0f);
    if (a < 0.015625f)                                   // below the smallest normal 2^-6: multiples of 2^-9
        return (unsigned)__builtin_rintf(a * 512.0f);    // 8 is the code of 2^-6 itself
    unsigned b = __float_as_uint(a);
    b += 0x7FFFFu + ((b >> 20) & 1u);                    // ties to even on the 3 kept mantissa bits
    return (b >> 20) - ((127u - 7u) << 3);               // rebias the exponent
}

static __device__ __forceinline__ float mx_e4m3_to_f32(unsigned c)
{
    const unsigned e = (c >> 3) & 15u, m = c & 7u;
    const float mag = e ? __uint_as_float(((e + 120u) << 23) | (m << 20)) : (float)m * 0.001953125f;
    return (c & 0x80u) ? -mag : mag;
}

// scale code of a block from the bf16 bit pattern of its largest magnitude (sign bit cleared):
// floor(log2 max) - 8, i.e. biased exponent - 8, held at 0 (which also covers the zero block)
static __device__ __forceinline__ int mx_scale_code(unsigned max_mag_bf16_bits) { return max((int)(max_mag_bf16_bits >> 7) - 8, 0); }

// element code of one bf16 value (bit pattern h) under the block's scale code
static __device__ __forceinline__ unsigned mx_encode_bf16(unsigned h, int scode)
{
    const float v = __uint_as_float((h & 0x7FFFu) << 16);
    return mx_e4m3_from_f32(ldexpf(v, 127 - scode)) | ((h >> 8) & 0x80u);   // exact division by the scale
}

// FP4 E2M1 (bias 1; values 0, 0.5, 1, 1.5, 2, 3, 4, 6; no NaN) code of one bf16 value under the block's
// scale code: round to nearest, ties to even, clamp at 6.
static __device__ __forceinline__ unsigned mx_encode_fp4_bf16(unsigned h, int scode)
{
    float a = ldexpf(__uint_as_float((h & 0x7FFFu) << 16), 127 - scode);
    a = fminf(a, 6.0f);
    unsigned c;
    if (a < 1.0f) {
        c = (unsigned)__builtin_rintf(a * 2.0f);         // multiples of 0.5; 2 is the code of 1.0 itself
    } else {
        unsigned b = __float_as_uint(a);
        b += 0x1FFFFFu + ((b >> 22) & 1u);               // ties to even on the one kept mantissa bit
        c = (b >> 22) - ((127u - 1u) << 1);              // rebias the exponent
    }
    return c | ((h >> 12) & 0x8u);
}

// Two element codes at once (low byte: the first value) through the hardware's scaled conversion
// V_CVT_SCALEF32_PK_FP8_F32, which divides by a power-of-two scale and rounds to nearest even exactly like the
// definition above but turns a magnitude beyond 448 into NaN; MX clamps, so the values are clamped to
// +-448 * scale first (one v_med3 each).  About 2 VALU operations per element instead of 15: it is what lets the
// LayerNorm kernels and the GEMM epilogues write codes beside their bf16 output.  The smallest scale (code 0 =
// 2^-127, not a normal float) takes the arithmetic path.
static __device__ __forceinline__ unsigned mx_encode_pair_bf16(unsigned h0, unsigned h1, int scode)
{
    if (scode == 0) return mx_encode_bf16(h0, 0) | (mx_encode_bf16(h1, 0) << 8);
    typedef short v2s_ __attribute__((ext_vector_type(2)));
    const float lim = __uint_as_float(((unsigned)(scode + 8) << 23) | 0x600000u);    // 448 * 2^(scode-127)
    const float a = __builtin_amdgcn_fmed3f(__uint_as_float(h0 << 16), -lim, lim);
    const float b = __builtin_amdgcn_fmed3f(__uint_as_float(h1 << 16), -lim, lim);
    const v2s_ zero = {0, 0};
    const v2s_ r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(zero, a, b, __uint_as_float((unsigned)scode << 23), false);
    return (unsigned)(unsigned short)r[0];
}
