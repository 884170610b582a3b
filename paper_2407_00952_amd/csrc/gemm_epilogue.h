// Epilogue of the GEMM kernels (bf16 and MXFP8 main loops share it): what happens to 8 consecutive
// columns of one output row once the accumulators (+ bias) are in registers.  `Args` provides
// out0, out1, aux and ldo with the meaning given at GemmArgs.
#pragma once
#include "common.h"
#include "mx_codec.h"

// Epilogue operands that come from global memory (the residual stream, or the saved GELU derivative),
// fetched one 32-row strip ahead of their use so that their latency hides behind the LDS transpose.
struct AuxRow {
    float4 r0, r1;       // EPI_RESID: 8 fp32 residual values
    bf16x8 f;            // EPI_DGELU: 8 bf16 values of GELU'(f) saved by the forward; EPI_STORE_DELTA: 8 values of O
    bf16x8 f2;           // EPI_STORE_DELTA: the low-order bf16 term of the same 8 values of O
};

template <int EPI, class Args>
__device__ __forceinline__ void load_aux(const Args &a, int row, int col, bool ok, AuxRow &x)
{
    if (EPI == EPI_RESID) {
        x.r0 = make_float4(0.f, 0.f, 0.f, 0.f);
        x.r1 = x.r0;
        if (ok) {
            const float *p = (const float *)a.aux + (size_t)row * a.ldo + col;
            x.r0 = *(const float4 *)p;
            x.r1 = *(const float4 *)(p + 4);
        }
    } else if (EPI == EPI_DGELU) {
#pragma unroll
        for (int i = 0; i < 8; ++i) x.f[i] = f2bf(0.f);
        if (ok) x.f = *(const bf16x8 *)((const bf16 *)a.aux + (size_t)row * a.ldo + col);
    }
    if constexpr (EPI == EPI_STORE_DELTA) {
#pragma unroll
        for (int i = 0; i < 8; ++i) { x.f[i] = f2bf(0.f); x.f2[i] = f2bf(0.f); }
        if (ok) {
            x.f = *(const bf16x8 *)(a.dl_o + (size_t)row * a.ldo + col);
            x.f2 = *(const bf16x8 *)(a.dl_lo + (size_t)row * a.ldo + col);
        }
    }
}

// MXFP8 copy of 8 consecutive bf16 outputs (compressed mode): the 4 lanes that hold a block of 32 columns are
// neighbours and are active together (column limits are multiples of 32 there), two shuffles give the block maximum.
template <class Args>
__device__ __forceinline__ void store_codes8(const Args &a, int row, int col, bf16x8 w)
{
    union { bf16x8 v; unsigned short s[8]; } bits;       // the eight bit patterns
    bits.v = w;
    unsigned hb[8], mag = 0u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        hb[i] = bits.s[i];
        mag = max(mag, hb[i] & 0x7FFFu);
    }
    mag = max(mag, (unsigned)__shfl_xor((int)mag, 1, 64));
    mag = max(mag, (unsigned)__shfl_xor((int)mag, 2, 64));
    const int scode = mx_scale_code(mag);
    unsigned q[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
        q[i] = mx_encode_pair_bf16(hb[4 * i], hb[4 * i + 1], scode) | (mx_encode_pair_bf16(hb[4 * i + 2], hb[4 * i + 3], scode) << 16);
    *(uint2 *)(a.oq + (size_t)row * a.ldo + col) = make_uint2(q[0], q[1]);
    if ((col & 31) == 0) a.os[(size_t)row * (a.ldo >> 5) + (col >> 5)] = (unsigned char)scode;
}

// Epilogue on 8 consecutive columns of one output row (v already holds acc + bias).
template <int EPI, class Args>
__device__ __forceinline__ void store_row8(const Args &a, int row, int col, float (&v)[8], const AuxRow &x)
{
    const size_t o = (size_t)row * a.ldo + col;
    if constexpr (EPI == EPI_STORE_DELTA) {
        // the rounded values that are stored also enter delta, so that the attention backward's dP (formed from
        // the stored tensor) and delta cancel exactly where they should.  The 8 lanes that hold a head's 64
        // columns of this row are neighbours, all active or all not (column limits are multiples of 64): after
        // lane shifts by 1, 2 and 4 inside a row of 16 lanes, lane 7 of each group of 8 holds the group's sum.
        bf16x8 w;
        float p = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            w[i] = f2bf(v[i]);
            p += bf2f(w[i]) * (bf2f(x.f[i]) + bf2f(x.f2[i]));
        }
        *(bf16x8 *)((bf16 *)a.out0 + o) = w;
        p += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(p), 0x111, 0xF, 0xF, true));   // row_shr:1
        p += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(p), 0x112, 0xF, 0xF, true));   // row_shr:2
        p += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(p), 0x114, 0xF, 0xF, true));   // row_shr:4
        if ((threadIdx.x & 7) == 7) a.dl_out[(size_t)row * (a.N >> 6) + (col >> 6)] = p;
    } else if (EPI == EPI_STORE) {
        bf16x8 w;
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = f2bf(v[i]);
        *(bf16x8 *)((bf16 *)a.out0 + o) = w;
    } else if (EPI == EPI_RESID) {
        v[0] += x.r0.x; v[1] += x.r0.y; v[2] += x.r0.z; v[3] += x.r0.w;
        v[4] += x.r1.x; v[5] += x.r1.y; v[6] += x.r1.z; v[7] += x.r1.w;
        if (a.out0) {
            *(float4 *)((float *)a.out0 + o) = make_float4(v[0], v[1], v[2], v[3]);
            *(float4 *)((float *)a.out0 + o + 4) = make_float4(v[4], v[5], v[6], v[7]);
        }
        if (a.out1) {
            bf16x8 w;
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = f2bf(v[i]);
            *(bf16x8 *)((bf16 *)a.out1 + o) = w;
        }
    } else if (EPI == EPI_GELU) {
        bf16x8 wf, wg;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // out0 keeps GELU'(f) (all the backward needs of f), out1 = GELU(f)
            float gv, gd;
            gelu_fwd_bwd(v[i], gv, gd);
            wf[i] = f2bf(gd);
            wg[i] = f2bf(gv);
        }
        *(bf16x8 *)((bf16 *)a.out0 + o) = wf;
        if constexpr (Args::kEmitCodes) {
            // compressed mode: the bf16 copy of g is only written when somebody reads it (an adapter on the
            // next projection); the product that consumes g takes the codes
            if (a.out1) *(bf16x8 *)((bf16 *)a.out1 + o) = wg;
            if (a.oq) store_codes8(a, row, col, wg);
        } else {
            *(bf16x8 *)((bf16 *)a.out1 + o) = wg;
        }
    } else {   // EPI_DGELU
        bf16x8 w;
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = f2bf(v[i] * bf2f(x.f[i]));   // aux holds GELU'(f)
        if constexpr (Args::kEmitCodes) {
            if (a.out0) *(bf16x8 *)((bf16 *)a.out0 + o) = w;
            if (a.oq) store_codes8(a, row, col, w);
        } else {
            *(bf16x8 *)((bf16 *)a.out0 + o) = w;
        }
    }
}
