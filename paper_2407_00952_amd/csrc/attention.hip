// Causal multi-head attention, forward and backward, head size 64, bf16 MFMA with fp32
// softmax arithmetic (gfx950).  Part of the server-side forward/backward of SplitLoRA
// Sec. III-B step a3; the attention block itself is the public GPT-2 one
// (softmax(Q K^T / sqrt(64)) V with future keys excluded).
//
// Layout: qkv [T, 3d] bf16 (q | k | v column blocks, head a at columns 64a..64a+63 of each),
// o / dO [T, d], lse [n_seq, H, S] fp32 in log2 units of the scaled scores, delta likewise.
//
// All three kernels use 4 wavefronts per block, each owning 32 rows (queries or keys), and
// online-softmax tiles of 64.  Scores are produced with the lane owning one query (forward,
// dQ) or one key (dK/dV), which makes the softmax statistics per-lane scalars and lets the
// probabilities feed the next MFMA straight from registers.  Operands that must be read
// along the token axis (V, K for dQ, Q and dO for dK/dV) are staged transposed in LDS.
// The backward is split into a dQ kernel and a dK/dV kernel so that no floating-point
// atomics are needed and results are bit-reproducible.
#include "common.h"

namespace {

constexpr float kScaleLog2 = 0.125f * 1.4426950408889634f;   // log2(e) / sqrt(64)
constexpr int TP = 68;                                       // pitch (elements) of transposed tiles [64][64]

__device__ __forceinline__ int swz128(int row, int chunk) { return row * 128 + ((chunk ^ (row & 7)) << 4); }

__device__ __forceinline__ f32x16 zero16()
{
    f32x16 z;
#pragma unroll
    for (int e = 0; e < 16; ++e) z[e] = 0.f;
    return z;
}

__device__ __forceinline__ bf16x8 cat4(bf16x4 a, bf16x4 b)
{
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) { r[i] = a[i]; r[4 + i] = b[i]; }
    return r;
}

// 64 rows x 64 columns of bf16 from global (pitch ld) -> LDS row-major, 16-byte XOR swizzle
__device__ __forceinline__ void stage_rows(unsigned char *dst, const bf16 *src, int ld, int tid)
{
#pragma unroll
    for (int c = tid; c < 512; c += 256) {
        const int row = c >> 3, ch = c & 7;
        *(uint4 *)(dst + swz128(row, ch)) = *(const uint4 *)(src + (size_t)row * ld + ch * 8);
    }
}
// the same tile -> LDS transposed: dst[col][row], pitch TP
__device__ __forceinline__ void stage_cols(bf16 *dst, const bf16 *src, int ld, int tid)
{
#pragma unroll
    for (int c = tid; c < 512; c += 256) {
        const int row = c >> 3, ch = c & 7;
        uint4 v = *(const uint4 *)(src + (size_t)row * ld + ch * 8);
        const bf16 *e = (const bf16 *)&v;
#pragma unroll
        for (int i = 0; i < 8; ++i) dst[(ch * 8 + i) * TP + row] = e[i];
    }
}
// both orientations from one global read
__device__ __forceinline__ void stage_both(unsigned char *rm, bf16 *tr, const bf16 *src, int ld, int tid)
{
#pragma unroll
    for (int c = tid; c < 512; c += 256) {
        const int row = c >> 3, ch = c & 7;
        uint4 v = *(const uint4 *)(src + (size_t)row * ld + ch * 8);
        *(uint4 *)(rm + swz128(row, ch)) = v;
        const bf16 *e = (const bf16 *)&v;
#pragma unroll
        for (int i = 0; i < 8; ++i) tr[(ch * 8 + i) * TP + row] = e[i];
    }
}

// A- or B-operand fragment: row (base + lane%32) of a swizzled row-major tile, k-step ks
__device__ __forceinline__ bf16x8 frag_rm(const unsigned char *t, int row, int ks, int g)
{
    return *(const bf16x8 *)(t + swz128(row, ks * 2 + g));
}
// fragment along the staged-transposed axis: 4 + 4 tokens at tok0 + 4g and tok0 + 8 + 4g
__device__ __forceinline__ bf16x8 frag_tr(const bf16 *t, int col, int tok0, int g)
{
    const bf16 *p = t + col * TP + tok0 + 4 * g;
    return cat4(*(const bf16x4 *)p, *(const bf16x4 *)(p + 8));
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_fwd_kernel(const bf16 *__restrict__ qkv, bf16 *__restrict__ o,
                                                       float *__restrict__ lse, int S, int H)
{
    __shared__ __align__(16) unsigned char Ks[64 * 128];
    __shared__ __align__(16) bf16 Vt[64 * TP];
    const int qt = gridDim.x - 1 - blockIdx.x;          // longest rows first
    const int a = blockIdx.y, n = blockIdx.z;
    const int d = H * 64, ld = 3 * d;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r32 = lane & 31, g = lane >> 5;
    const bf16 *base = qkv + (size_t)n * S * ld + a * 64;
    const int qb = qt * 128 + wave * 32;
    const bool active = qb < S;
    const int q = qb + r32;

    bf16x8 qf[4];
    if (active) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qf[ks] = *(const bf16x8 *)(base + (size_t)q * ld + ks * 16 + g * 8);
    }
    f32x16 oacc[2] = {zero16(), zero16()};
    float m = -INFINITY, l = 0.f;
    const int kv_end = min(S, qt * 128 + 128);

    for (int k0 = 0; k0 < kv_end; k0 += 64) {
        __syncthreads();
        stage_rows(Ks, base + d + (size_t)k0 * ld, ld, tid);
        stage_cols(Vt, base + 2 * d + (size_t)k0 * ld, ld, tid);
        __syncthreads();
        if (active && k0 <= qb + 31) {
            f32x16 sacc[2] = {zero16(), zero16()};
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm(Ks, mt * 32 + r32, ks, g), qf[ks],
                                                                        sacc[mt], 0, 0, 0);
            const bool need_mask = k0 + 63 > qb;
            float tmax = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = k0 + 32 * mt + 8 * (e >> 2) + 4 * g + (e & 3);
                    float v = sacc[mt][e] * kScaleLog2;
                    if (need_mask && key > q) v = -INFINITY;
                    sacc[mt][e] = v;
                    tmax = fmaxf(tmax, v);
                }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            const float m_new = fmaxf(m, tmax);
            const float alpha = exp2f(m - m_new);
            float psum = 0.f;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float p = exp2f(sacc[mt][e] - m_new);
                    sacc[mt][e] = p;
                    psum += p;
                }
            psum += __shfl_xor(psum, 32, 64);
            l = l * alpha + psum;
            m = m_new;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[dt][e] *= alpha;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    bf16x8 pb;
#pragma unroll
                    for (int i = 0; i < 8; ++i) pb[i] = f2bf(sacc[mt][8 * hh + i]);
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt)
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            frag_tr(Vt, 32 * dt + r32, 32 * mt + 16 * hh, g), pb, oacc[dt], 0, 0, 0);
                }
        }
    }
    if (active) {
        const float inv = 1.0f / l;
        bf16 *orow = o + ((size_t)n * S + q) * d + a * 64;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                bf16x4 w;
#pragma unroll
                for (int i = 0; i < 4; ++i) w[i] = f2bf(oacc[dt][4 * e4 + i] * inv);
                *(bf16x4 *)(orow + 32 * dt + 8 * e4 + 4 * g) = w;
            }
        if (g == 0) lse[((size_t)n * H + a) * S + q] = m + log2f(l);
    }
}

// ------------------------------------------------------------------------------------------
// dQ (and delta = rowsum(dO * O), which the dK/dV kernel reads afterwards)
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(const bf16 *__restrict__ qkv, const bf16 *__restrict__ o,
                                                          const bf16 *__restrict__ dout,
                                                          const float *__restrict__ lse, float *__restrict__ delta,
                                                          bf16 *__restrict__ dqkv, int S, int H)
{
    __shared__ __align__(16) unsigned char Ks[64 * 128];
    __shared__ __align__(16) unsigned char Vs[64 * 128];
    __shared__ __align__(16) bf16 Kt[64 * TP];
    const int qt = gridDim.x - 1 - blockIdx.x;
    const int a = blockIdx.y, n = blockIdx.z;
    const int d = H * 64, ld = 3 * d;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r32 = lane & 31, g = lane >> 5;
    const bf16 *base = qkv + (size_t)n * S * ld + a * 64;
    const int qb = qt * 128 + wave * 32;
    const bool active = qb < S;
    const int q = qb + r32;

    bf16x8 qf[4], dof[4];
    float lse_q = 0.f, dl = 0.f;
    if (active) {
        const bf16 *orow = o + ((size_t)n * S + q) * d + a * 64;
        const bf16 *drow = dout + ((size_t)n * S + q) * d + a * 64;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            qf[ks] = *(const bf16x8 *)(base + (size_t)q * ld + ks * 16 + g * 8);
            dof[ks] = *(const bf16x8 *)(drow + ks * 16 + g * 8);
            bf16x8 of = *(const bf16x8 *)(orow + ks * 16 + g * 8);
#pragma unroll
            for (int i = 0; i < 8; ++i) dl += bf2f(dof[ks][i]) * bf2f(of[i]);
        }
        dl += __shfl_xor(dl, 32, 64);
        lse_q = lse[((size_t)n * H + a) * S + q];
        if (g == 0) delta[((size_t)n * H + a) * S + q] = dl;
    }
    f32x16 dqacc[2] = {zero16(), zero16()};
    const int kv_end = min(S, qt * 128 + 128);

    for (int k0 = 0; k0 < kv_end; k0 += 64) {
        __syncthreads();
        stage_both(Ks, Kt, base + d + (size_t)k0 * ld, ld, tid);
        stage_rows(Vs, base + 2 * d + (size_t)k0 * ld, ld, tid);
        __syncthreads();
        if (active && k0 <= qb + 31) {
            const bool need_mask = k0 + 63 > qb;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                f32x16 sacc = zero16(), dpacc = zero16();
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm(Ks, mt * 32 + r32, ks, g), qf[ks], sacc,
                                                                    0, 0, 0);
                    dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm(Vs, mt * 32 + r32, ks, g), dof[ks],
                                                                     dpacc, 0, 0, 0);
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = k0 + 32 * mt + 8 * (e >> 2) + 4 * g + (e & 3);
                    float p = exp2f(sacc[e] * kScaleLog2 - lse_q);
                    if (need_mask && key > q) p = 0.f;
                    sacc[e] = p * (dpacc[e] - dl);
                }
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    bf16x8 dsb;
#pragma unroll
                    for (int i = 0; i < 8; ++i) dsb[i] = f2bf(sacc[8 * hh + i]);
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt)
                        dqacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            frag_tr(Kt, 32 * dt + r32, 32 * mt + 16 * hh, g), dsb, dqacc[dt], 0, 0, 0);
                }
            }
        }
    }
    if (active) {
        bf16 *drow = dqkv + ((size_t)n * S + q) * ld + a * 64;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                bf16x4 w;
#pragma unroll
                for (int i = 0; i < 4; ++i) w[i] = f2bf(dqacc[dt][4 * e4 + i] * 0.125f);
                *(bf16x4 *)(drow + 32 * dt + 8 * e4 + 4 * g) = w;
            }
    }
}

// ------------------------------------------------------------------------------------------
// dK, dV: each wavefront owns 32 keys and walks the query tiles that can see them
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(const bf16 *__restrict__ qkv,
                                                           const bf16 *__restrict__ dout,
                                                           const float *__restrict__ lse,
                                                           const float *__restrict__ delta,
                                                           bf16 *__restrict__ dqkv, int S, int H)
{
    __shared__ __align__(16) unsigned char Qs[64 * 128];
    __shared__ __align__(16) unsigned char Ds[64 * 128];
    __shared__ __align__(16) bf16 Qt[64 * TP];
    __shared__ __align__(16) bf16 Dt[64 * TP];
    __shared__ __align__(16) float lse_s[64];
    __shared__ __align__(16) float dl_s[64];
    const int kvt = blockIdx.x;                          // keys kvt*128 ..: most work first
    const int a = blockIdx.y, n = blockIdx.z;
    const int d = H * 64, ld = 3 * d;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r32 = lane & 31, g = lane >> 5;
    const bf16 *base = qkv + (size_t)n * S * ld + a * 64;
    const bf16 *dbase = dout + (size_t)n * S * d + a * 64;
    const int kb = kvt * 128 + wave * 32;
    const bool active = kb < S;
    const int key = kb + r32;

    bf16x8 kf[4], vf[4];
    if (active) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            kf[ks] = *(const bf16x8 *)(base + d + (size_t)key * ld + ks * 16 + g * 8);
            vf[ks] = *(const bf16x8 *)(base + 2 * d + (size_t)key * ld + ks * 16 + g * 8);
        }
    }
    f32x16 dkacc[2] = {zero16(), zero16()}, dvacc[2] = {zero16(), zero16()};

    for (int q0 = kvt * 128; q0 < S; q0 += 64) {
        __syncthreads();
        stage_both(Qs, Qt, base + (size_t)q0 * ld, ld, tid);
        stage_both(Ds, Dt, dbase + (size_t)q0 * d, d, tid);
        if (tid < 64) lse_s[tid] = lse[((size_t)n * H + a) * S + q0 + tid];
        else if (tid < 128) dl_s[tid - 64] = delta[((size_t)n * H + a) * S + q0 + tid - 64];
        __syncthreads();
        if (!active) continue;
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            const int qs = q0 + 32 * st;
            if (qs + 31 < kb) continue;                  // every query of the sub-tile precedes every key
            const bool need_mask = qs < kb + 31;
            f32x16 sacc = zero16(), dpacc = zero16();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm(Qs, 32 * st + r32, ks, g), kf[ks], sacc, 0,
                                                                0, 0);
                dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm(Ds, 32 * st + r32, ks, g), vf[ks], dpacc, 0,
                                                                 0, 0);
            }
            // lane = key column; element e = query row 8(e/4) + 4g + e%4 of the sub-tile
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const int ql = 32 * st + 8 * e4 + 4 * g;
                const f32x4 ls = *(const f32x4 *)(lse_s + ql);
                const f32x4 dd = *(const f32x4 *)(dl_s + ql);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int e = 4 * e4 + i;
                    float p = exp2f(sacc[e] * kScaleLog2 - ls[i]);
                    if (need_mask && key > q0 + ql + i) p = 0.f;
                    sacc[e] = p;
                    dpacc[e] = p * (dpacc[e] - dd[i]);
                }
            }
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                bf16x8 pb, dsb;
#pragma unroll
                for (int i = 0; i < 8; ++i) { pb[i] = f2bf(sacc[8 * hh + i]); dsb[i] = f2bf(dpacc[8 * hh + i]); }
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    dvacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_tr(Dt, 32 * dt + r32, 32 * st + 16 * hh, g), pb, dvacc[dt], 0, 0, 0);
                    dkacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_tr(Qt, 32 * dt + r32, 32 * st + 16 * hh, g), dsb, dkacc[dt], 0, 0, 0);
                }
            }
        }
    }
    if (active) {
        bf16 *krow = dqkv + ((size_t)n * S + key) * ld + d + a * 64;
        bf16 *vrow = krow + d;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                bf16x4 wk, wv;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    wk[i] = f2bf(dkacc[dt][4 * e4 + i] * 0.125f);
                    wv[i] = f2bf(dvacc[dt][4 * e4 + i]);
                }
                *(bf16x4 *)(krow + 32 * dt + 8 * e4 + 4 * g) = wk;
                *(bf16x4 *)(vrow + 32 * dt + 8 * e4 + 4 * g) = wv;
            }
    }
}

}  // namespace

int launch_attn_fwd(const bf16 *qkv, bf16 *o, float *lse, int n_seq, int S, int H, hipStream_t st)
{
    if (n_seq <= 0 || S <= 0 || (S % 64) || H <= 0) return -1;
    dim3 grid((S + 127) / 128, H, n_seq);
    hipLaunchKernelGGL(attn_fwd_kernel, grid, dim3(256), 0, st, qkv, o, lse, S, H);
    SL_CHECK_LAUNCH("attn_fwd");
    return 0;
}

int launch_attn_bwd(const bf16 *qkv, const bf16 *o, const bf16 *dout, const float *lse, float *delta, bf16 *dqkv,
                    int n_seq, int S, int H, hipStream_t st)
{
    if (n_seq <= 0 || S <= 0 || (S % 64) || H <= 0) return -1;
    dim3 grid((S + 127) / 128, H, n_seq);
    hipLaunchKernelGGL(attn_bwd_dq_kernel, grid, dim3(256), 0, st, qkv, o, dout, lse, delta, dqkv, S, H);
    SL_CHECK_LAUNCH("attn_bwd_dq");
    hipLaunchKernelGGL(attn_bwd_dkv_kernel, grid, dim3(256), 0, st, qkv, dout, lse, delta, dqkv, S, H);
    SL_CHECK_LAUNCH("attn_bwd_dkv");
    return 0;
}
