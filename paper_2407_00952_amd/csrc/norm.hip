// LayerNorm forward / input-gradient kernels for the frozen GPT-2 blocks of the server stack
// (SplitLoRA Sec. III-B step a3: the server-side forward and backward; LayerNorm gains and
// biases are frozen, Sec. III-A, so no parameter gradient is produced).
//
// One 64-lane wavefront per token row, the row held in registers, two wave reductions.
// These kernels are HBM-bound; they also carry the fp32 residual stream:
//   forward : u = (h - mu) rho * gamma + beta  (bf16 out), stats (mu, rho) saved per row.
//             For the first server block the input is gathered from the K client buffers
//             (the concatenation S = [s_1; ...; s_N]) and an fp32 copy of it is kept.  For the
//             first CLIENT block the input is the token + position embedding, summed in fp32
//             straight from the two frozen tables (client-side forward, Sec. III-B a1).
//   backward: out = dres + rho (g - mean(g) - xhat mean(g xhat)),  g = du * gamma,
//             written as fp32 (residual gradient) and/or bf16 (next GEMM operand, or the
//             per-client activation gradient scattered back to the K client buffers).
#include "common.h"
#include "mx_codec.h"
#include "prof.h"

namespace {

constexpr int MAXC = 8;   // 256-column chunks per row: d <= 2048

__device__ __forceinline__ int client_of(const ClientTable &t, int row, int &local)
{
    int c = 0, start = 0;
    while (c < t.K - 1 && row >= t.row_end[c]) { start = t.row_end[c]; ++c; }
    local = row - start;
    return c;
}

// MXFP8 copy of a row: each lane holds 4 consecutive bf16 values of a 256-column chunk, so a block of 32 columns
// is 8 neighbouring lanes (three shuffles for its maximum).  Every lane of the wave must call this; lanes
// whose columns are outside the row (`in_row` false) only take part in the shuffles.
__device__ __forceinline__ void mx_store_row4(bf16x4 o, bool in_row, int lane, unsigned char *q_row,
                                              unsigned char *s_row, int col)
{
    union { bf16x4 v; unsigned short s[4]; } bits;       // the four bit patterns
    bits.v = o;
    unsigned hb[4] = {0u, 0u, 0u, 0u}, mag = 0u;
    if (in_row) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            hb[i] = bits.s[i];
            mag = max(mag, hb[i] & 0x7FFFu);
        }
    }
    mag = max(mag, (unsigned)__shfl_xor((int)mag, 1, 64));
    mag = max(mag, (unsigned)__shfl_xor((int)mag, 2, 64));
    mag = max(mag, (unsigned)__shfl_xor((int)mag, 4, 64));
    const int scode = mx_scale_code(mag);
    if (in_row) {
        const unsigned q4 = mx_encode_pair_bf16(hb[0], hb[1], scode) | (mx_encode_pair_bf16(hb[2], hb[3], scode) << 16);
        *(unsigned *)(q_row + col) = q4;
        if ((lane & 7) == 0) s_row[col >> 5] = (unsigned char)scode;
    }
}

// SRC 0: fp32 rows of h; 1: bf16 rows gathered from the client buffers; 2: embedding lookup;
// 3: MXFP8 rows (element codes + one scale code per 32 columns) gathered from the client buffers
template <int SRC>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const float *__restrict__ h, ClientTable tab, EmbedSrc emb,
                                                     float *__restrict__ hcopy, const bf16 *__restrict__ gamma,
                                                     const bf16 *__restrict__ beta, float eps,
                                                     bf16 *__restrict__ u, float *__restrict__ stats, int T, int d,
                                                     unsigned char *__restrict__ uq, unsigned char *__restrict__ us)
{
    constexpr bool GATHER = SRC != 0;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= T) return;
    float v[MAXC][4];
    const bf16 *src16 = nullptr, *pos16 = nullptr;
    const unsigned char *srcq = nullptr, *srcs = nullptr;
    if (SRC == 3) {
        int local;
        int c = client_of(tab, row, local);
        srcq = (const unsigned char *)tab.ptr[c] + (size_t)local * d;
        srcs = (const unsigned char *)tab.aux[c] + (size_t)local * (d >> 5);
    } else if (SRC == 1) {
        int local;
        int c = client_of(tab, row, local);
        src16 = (const bf16 *)tab.ptr[c] + (size_t)local * d;
    } else if (SRC == 2) {
        const int tok = min(max(emb.tokens[row], 0), emb.vocab - 1);     // ids outside the table are clamped
        src16 = emb.wte + (size_t)tok * d;
        pos16 = emb.wpe + (size_t)(row % emb.seq_len) * d;
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int col = c * 256 + lane * 4;
        if (col < d) {
            if (SRC == 3) {
                const unsigned q4 = *(const unsigned *)(srcq + col);
                const int sc = (int)srcs[col >> 5] - 127;
#pragma unroll
                for (int i = 0; i < 4; ++i) v[c][i] = ldexpf(mx_e4m3_to_f32((q4 >> (8 * i)) & 0xFFu), sc);
                *(float4 *)(hcopy + (size_t)row * d + col) = make_float4(v[c][0], v[c][1], v[c][2], v[c][3]);
            } else if (GATHER) {
                bf16x4 t = *(const bf16x4 *)(src16 + col);
#pragma unroll
                for (int i = 0; i < 4; ++i) v[c][i] = bf2f(t[i]);
                if (SRC == 2) {
                    bf16x4 q = *(const bf16x4 *)(pos16 + col);
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[c][i] += bf2f(q[i]);
                }
                *(float4 *)(hcopy + (size_t)row * d + col) = make_float4(v[c][0], v[c][1], v[c][2], v[c][3]);
            } else {
                float4 t = *(const float4 *)(h + (size_t)row * d + col);
                v[c][0] = t.x; v[c][1] = t.y; v[c][2] = t.z; v[c][3] = t.w;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) s += v[c][i];
        }
    }
    const float mu = wave_sum(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        if (c * 256 + lane * 4 < d) {
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[c][i] -= mu; q += v[c][i] * v[c][i]; }
        }
    }
    const float rho = rsqrtf(wave_sum(q) / (float)d + eps);
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int col = c * 256 + lane * 4;
        bf16x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = f2bf(0.f);
        if (col < d) {
            bf16x4 gm = *(const bf16x4 *)(gamma + col);
            bf16x4 bt = *(const bf16x4 *)(beta + col);
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = f2bf(v[c][i] * rho * bf2f(gm[i]) + bf2f(bt[i]));
            if (u != nullptr) *(bf16x4 *)(u + (size_t)row * d + col) = o;    // (null: only the codes are wanted)
        }
        if (uq != nullptr && c * 256 < d)
            mx_store_row4(o, col < d, lane, uq + (size_t)row * d, us + (size_t)row * (d >> 5), col);
    }
    if (lane == 0) { stats[2 * row] = mu; stats[2 * row + 1] = rho; }
}

// DRES16: the residual gradient arrives as bf16 (last block: the caller's dY) instead of fp32;
// with DRES16 false a null `dres` means there is no residual gradient to add.
// SCATTER 1: the bf16 output goes to the K client buffers; 2: it goes there as MXFP8 (the value is rounded
// to bf16 first, then converted block by block: 8 neighbouring lanes hold one block of 32 columns).
template <bool DRES16, int SCATTER>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const bf16 *__restrict__ du, const float *__restrict__ h,
                                                     const float *__restrict__ stats, const bf16 *__restrict__ gamma,
                                                     const void *__restrict__ dres, float *__restrict__ out32,
                                                     bf16 *__restrict__ out16, ClientTable tab, int T, int d,
                                                     unsigned char *__restrict__ oq, unsigned char *__restrict__ os)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= T) return;
    const float mu = stats[2 * row], rho = stats[2 * row + 1];
    float gq[MAXC][4], xh[MAXC][4];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int col = c * 256 + lane * 4;
        if (col < d) {
            bf16x4 t = *(const bf16x4 *)(du + (size_t)row * d + col);
            bf16x4 gm = *(const bf16x4 *)(gamma + col);
            float4 hv = *(const float4 *)(h + (size_t)row * d + col);
            const float hh[4] = {hv.x, hv.y, hv.z, hv.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                gq[c][i] = bf2f(t[i]) * bf2f(gm[i]);
                xh[c][i] = (hh[i] - mu) * rho;
                s1 += gq[c][i];
                s2 += gq[c][i] * xh[c][i];
            }
        }
    }
    const float m1 = wave_sum(s1) / (float)d;
    const float m2 = wave_sum(s2) / (float)d;
    bf16 *dst16 = out16 ? out16 + (size_t)row * d : nullptr;
    unsigned char *dstq = nullptr, *dsts = nullptr;
    if (SCATTER) {
        int local;
        int c = client_of(tab, row, local);
        if (SCATTER == 2) {
            dstq = (unsigned char *)tab.ptr[c] + (size_t)local * d;
            dsts = (unsigned char *)tab.aux[c] + (size_t)local * (d >> 5);
            dst16 = nullptr;
        } else {
            dst16 = (bf16 *)tab.ptr[c] + (size_t)local * d;
        }
    }
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int col = c * 256 + lane * 4;
        float r_keep[4] = {0.f, 0.f, 0.f, 0.f};
        if (col < d) {
            float r[4];
            if (DRES16) {
                bf16x4 t = *(const bf16x4 *)((const bf16 *)dres + (size_t)row * d + col);
#pragma unroll
                for (int i = 0; i < 4; ++i) r[i] = bf2f(t[i]);
            } else if (dres != nullptr) {
                float4 t = *(const float4 *)((const float *)dres + (size_t)row * d + col);
                r[0] = t.x; r[1] = t.y; r[2] = t.z; r[3] = t.w;
            } else {                                     // no residual branch (the final LayerNorm)
                r[0] = r[1] = r[2] = r[3] = 0.f;
            }
            bf16x4 o16;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                r[i] += rho * (gq[c][i] - m1 - xh[c][i] * m2);
                o16[i] = f2bf(r[i]);
                r_keep[i] = r[i];
            }
            if (out32) *(float4 *)(out32 + (size_t)row * d + col) = make_float4(r[0], r[1], r[2], r[3]);
            if (dst16) *(bf16x4 *)(dst16 + col) = o16;
        }
        if (SCATTER == 2) {
            // d is a multiple of 32, so the 8 lanes of a block are either all inside the row or all outside
            bf16x4 o4;
#pragma unroll
            for (int i = 0; i < 4; ++i) o4[i] = f2bf(r_keep[i]);
            if (c * 256 < d) mx_store_row4(o4, col < d, lane, dstq, dsts, col);
        } else if (oq != nullptr && c * 256 < d) {
            bf16x4 o4;
#pragma unroll
            for (int i = 0; i < 4; ++i) o4[i] = f2bf(r_keep[i]);
            mx_store_row4(o4, col < d, lane, oq + (size_t)row * d, os + (size_t)row * (d >> 5), col);
        }
    }
}

}  // namespace

int launch_ln_fwd(const float *h_f32, const ClientTable *gather, float *h_copy, const bf16 *gamma,
                  const bf16 *beta, float eps, bf16 *u, float *stats, int T, int d, hipStream_t st,
                  const EmbedSrc *embed, unsigned char *u_codes, unsigned char *u_scales)
{
    if (T <= 0 || d <= 0 || (d % 4) || d > MAXC * 256) return SL_EINVAL;
    if (u_codes && (!u_scales || (d % 32))) return SL_EINVAL;
    if (!u && !u_codes) return SL_EINVAL;
    if (gather && gather->mx && (d % 32)) return SL_EINVAL;
    dim3 grid((T + 3) / 4), block(256);
    ClientTable none;
    none.K = 0;
    none.mx = 0;
    EmbedSrc noemb = {nullptr, nullptr, nullptr, 1, 1};
    // algorithmic bytes: the row read once (fp32, or bf16 / codes when gathered, then also kept as fp32), u written
    const double row_bytes = (embed ? 4 + 4 : gather ? (gather->mx ? 1 + 4 : 2 + 4) : 4) + (u ? 2 : 0) + (u_codes ? 1 : 0);
    const bool rec = prof_begin(PK_LN_FWD, st);
    if (embed) {
        if (!embed->tokens || !embed->wte || !embed->wpe || embed->seq_len <= 0 || embed->vocab <= 0) return SL_EINVAL;
        hipLaunchKernelGGL((ln_fwd_kernel<2>), grid, block, 0, st, nullptr, none, *embed, h_copy, gamma, beta, eps, u,
                           stats, T, d, u_codes, u_scales);
    } else if (gather && gather->mx) {
        hipLaunchKernelGGL((ln_fwd_kernel<3>), grid, block, 0, st, nullptr, *gather, noemb, h_copy, gamma, beta, eps,
                           u, stats, T, d, u_codes, u_scales);
    } else if (gather) {
        hipLaunchKernelGGL((ln_fwd_kernel<1>), grid, block, 0, st, nullptr, *gather, noemb, h_copy, gamma, beta, eps,
                           u, stats, T, d, u_codes, u_scales);
    } else {
        hipLaunchKernelGGL((ln_fwd_kernel<0>), grid, block, 0, st, h_f32, none, noemb, nullptr, gamma, beta, eps, u,
                           stats, T, d, u_codes, u_scales);
    }
    prof_end(rec, PK_LN_FWD, row_bytes * (double)T * d, st);
    SL_CHECK_LAUNCH("ln_fwd");
    return 0;
}

int launch_ln_bwd(const bf16 *du, const float *h, const float *stats, const bf16 *gamma, const float *dres_f32,
                  const bf16 *dres_bf16, float *out_f32, bf16 *out_bf16, const ClientTable *scatter, int T, int d,
                  hipStream_t st, unsigned char *o_codes, unsigned char *o_scales)
{
    if (T <= 0 || d <= 0 || (d % 4) || d > MAXC * 256) return SL_EINVAL;
    if (o_codes && (!o_scales || (d % 32) || scatter)) return SL_EINVAL;
    dim3 grid((T + 3) / 4), block(256);
    ClientTable tab;
    tab.K = 0;
    tab.mx = 0;
    if (scatter) tab = *scatter;
    // algorithmic bytes per element: du (bf16), h (fp32), the residual gradient, and each output written
    const double el_bytes = 2 + 4 + (dres_bf16 ? 2 : dres_f32 ? 4 : 0) + (out_f32 ? 4 : 0) + (out_bf16 ? 2 : 0) +
                            (scatter ? (scatter->mx ? 1 : 2) : 0) + (o_codes ? 1 : 0);
    const bool rec = prof_begin(PK_LN_BWD, st);
    if (scatter && scatter->mx) {
        // compressed activation gradients: only the first server block scatters, and its residual gradient is fp32
        if ((d % 32) || dres_bf16) return SL_EINVAL;
        hipLaunchKernelGGL((ln_bwd_kernel<false, 2>), grid, block, 0, st, du, h, stats, gamma, (const void *)dres_f32,
                           out_f32, out_bf16, tab, T, d, o_codes, o_scales);
    } else if (dres_bf16) {
        if (scatter)
            hipLaunchKernelGGL((ln_bwd_kernel<true, 1>), grid, block, 0, st, du, h, stats, gamma,
                               (const void *)dres_bf16, out_f32, out_bf16, tab, T, d, o_codes, o_scales);
        else
            hipLaunchKernelGGL((ln_bwd_kernel<true, 0>), grid, block, 0, st, du, h, stats, gamma,
                               (const void *)dres_bf16, out_f32, out_bf16, tab, T, d, o_codes, o_scales);
    } else {
        if (scatter)
            hipLaunchKernelGGL((ln_bwd_kernel<false, 1>), grid, block, 0, st, du, h, stats, gamma,
                               (const void *)dres_f32, out_f32, out_bf16, tab, T, d, o_codes, o_scales);
        else
            hipLaunchKernelGGL((ln_bwd_kernel<false, 0>), grid, block, 0, st, du, h, stats, gamma,
                               (const void *)dres_f32, out_f32, out_bf16, tab, T, d, o_codes, o_scales);
    }
    prof_end(rec, PK_LN_BWD, el_bytes * (double)T * d, st);
    SL_CHECK_LAUNCH("ln_bwd");
    return 0;
}
