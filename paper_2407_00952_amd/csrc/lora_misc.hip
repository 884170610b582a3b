// Adapter-side kernels: LoRA gradients, SGD step, FedAvg, and the bf16 shadow copies.
//
//  * LoRA gradients (SplitLoRA Sec. III-B step a3: "derive the server-side LoRA adapters'
//    gradients"): with ps = s (dy B) and zs = s (x A^T) spilled by the GEMMs,
//        dA = ps^T x   [r,in]        dB = dy^T zs   [out,r]
//    Both are G[c,j] = sum_t X[t,c] Y[t,j] with a tall X [T,C] and a skinny Y [T,r]: one
//    streaming pass over X (HBM-bound), per-chunk partial sums, then a fixed-order
//    reduction over chunks -- no floating-point atomics, so results are reproducible.
//  * SGD (Eq. 4-5): p = fmaf(-lr, g, p).
//  * FedAvg (Sec. III-B step b2, Eq. 8-9): acc = fmaf(w_i, x_i[j], acc), i = 0..K-1.
#include "common.h"

namespace {

constexpr int GR_ROWS = 128;   // token rows per block (32 per wavefront)
constexpr int GR_COLS = 512;   // columns per block: 8 per lane, 16-byte loads

template <int R>
__global__ __launch_bounds__(256) void lora_grad_partial_kernel(const bf16 *__restrict__ X, int ldx, int C,
                                                                const bf16 *__restrict__ Y, int ldy, int r, int T,
                                                                float *__restrict__ partials)
{
    __shared__ float red[3][R][GR_COLS];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c0 = blockIdx.x * GR_COLS + lane * 8;
    const int chunk = blockIdx.y;
    const int t0 = chunk * GR_ROWS + wave * 32;
    const int t1 = min(t0 + 32, T);
    float acc[8][R];
#pragma unroll
    for (int cc = 0; cc < 8; ++cc)
#pragma unroll
        for (int j = 0; j < R; ++j) acc[cc][j] = 0.f;
    const bool colok = c0 < C;   // C % 8 == 0
    int t = t0;
    // four rows per trip: the four 16-byte loads are in flight together
    for (; t + 4 <= t1; t += 4) {
        bf16x8 xv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int i = 0; i < 8; ++i) xv[u][i] = f2bf(0.f);
            if (colok) xv[u] = *(const bf16x8 *)(X + (size_t)(t + u) * ldx + c0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bf16 *yr = Y + (size_t)(t + u) * ldy;      // wave-uniform address
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const float y = (j < r) ? bf2f(yr[j]) : 0.f;
#pragma unroll
                for (int cc = 0; cc < 8; ++cc) acc[cc][j] = fmaf(bf2f(xv[u][cc]), y, acc[cc][j]);
            }
        }
    }
    for (; t < t1; ++t) {
        bf16x8 xv;
#pragma unroll
        for (int i = 0; i < 8; ++i) xv[i] = f2bf(0.f);
        if (colok) xv = *(const bf16x8 *)(X + (size_t)t * ldx + c0);
        const bf16 *yr = Y + (size_t)t * ldy;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const float y = (j < r) ? bf2f(yr[j]) : 0.f;
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) acc[cc][j] = fmaf(bf2f(xv[cc]), y, acc[cc][j]);
        }
    }
    // fixed order over the four wavefronts: wave 0 adds the partial sums of waves 1, 2, 3
    if (wave > 0) {
#pragma unroll
        for (int j = 0; j < R; ++j)
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) red[wave - 1][j][cc * 64 + lane] = acc[cc][j];
    }
    __syncthreads();
    if (wave == 0 && colok) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (j < r) {
                float s[8];
#pragma unroll
                for (int cc = 0; cc < 8; ++cc) {
                    s[cc] = acc[cc][j];
                    s[cc] += red[0][j][cc * 64 + lane];
                    s[cc] += red[1][j][cc * 64 + lane];
                    s[cc] += red[2][j][cc * 64 + lane];
                }
                float *dst = partials + ((size_t)chunk * r + j) * C + c0;
                *(float4 *)dst = make_float4(s[0], s[1], s[2], s[3]);
                *(float4 *)(dst + 4) = make_float4(s[4], s[5], s[6], s[7]);
            }
        }
    }
}

// out[j, c] = sum over chunks, in a fixed order: each of the 4 wavefronts of a block sums a
// contiguous quarter of the chunks in increasing order, then the four are added in order.
__global__ __launch_bounds__(256) void lora_grad_reduce_kernel(const float *__restrict__ partials, int nchunk, int r,
                                                               int C, float *__restrict__ out, int out_is_rxC)
{
    __shared__ float red[3][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int idx = blockIdx.x * 64 + lane;              // over r*C, c fastest
    const bool ok = idx < r * C;
    const int j = ok ? idx / C : 0, c = ok ? idx - j * C : 0;
    const int per = (nchunk + 3) >> 2;
    const int k0 = wave * per, k1 = min(k0 + per, nchunk);
    float s = 0.f;
    if (ok) {
        const float *src = partials + (size_t)j * C + c;
        const size_t step = (size_t)r * C;
        int k = k0;
        // eight loads in flight, added in increasing chunk order
        for (; k + 8 <= k1; k += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[(size_t)(k + u) * step];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; k < k1; ++k) s += src[(size_t)k * step];
    }
    if (wave > 0) red[wave - 1][lane] = s;
    __syncthreads();
    if (wave == 0 && ok) {
        s += red[0][lane];
        s += red[1][lane];
        s += red[2][lane];
        if (out_is_rxC) out[(size_t)j * C + c] = s;
        else out[(size_t)c * r + j] = s;
    }
}

__global__ __launch_bounds__(256) void sgd_kernel(float *__restrict__ p, const float *__restrict__ g, float lr,
                                                  size_t n)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) p[i] = __fmaf_rn(-lr, g[i], p[i]);
}

// src fp32 [rows, cols] -> dst bf16 [drows, dcols], zero padded; optionally transposed first
__global__ __launch_bounds__(256) void cast_pad_kernel(const float *__restrict__ src, int rows, int cols,
                                                       bf16 *__restrict__ dst, int drows, int dcols, int transpose)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= drows * dcols) return;
    const int i = idx / dcols, j = idx - i * dcols;
    float v = 0.f;
    if (!transpose) {
        if (i < rows && j < cols) v = src[(size_t)i * cols + j];
    } else {
        if (j < rows && i < cols) v = src[(size_t)j * cols + i];
    }
    dst[idx] = f2bf(v);
}

__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16 *__restrict__ src, int rows, int cols,
                                                             bf16 *__restrict__ dst)
{
    __shared__ bf16 tile[64][66];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int r = i >> 6, c = i & 63;
        if (r0 + r < rows && c0 + c < cols) tile[r][c] = src[(size_t)(r0 + r) * cols + c0 + c];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int c = i >> 6, r = i & 63;
        if (r0 + r < rows && c0 + c < cols) dst[(size_t)(c0 + c) * rows + r0 + r] = tile[r][c];
    }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t *__restrict__ p, size_t nwords)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < nwords; i += stride) p[i] = 0u;
}

struct FedTable {
    const float *x[SL_MAX_CLIENTS];
    float w[SL_MAX_CLIENTS];
    int K;
};

// 4 floats per thread when everything is 16-byte aligned, else scalar
template <bool VEC>
__global__ __launch_bounds__(256) void fedavg_kernel(FedTable t, size_t n, float *__restrict__ out)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    if (VEC) {
        const size_t n4 = n >> 2;
        for (; i < n4; i += stride) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int c = 0; c < t.K; ++c) {
                const float4 v = ((const float4 *)t.x[c])[i];
                const float w = t.w[c];
                acc.x = __fmaf_rn(w, v.x, acc.x);
                acc.y = __fmaf_rn(w, v.y, acc.y);
                acc.z = __fmaf_rn(w, v.z, acc.z);
                acc.w = __fmaf_rn(w, v.w, acc.w);
            }
            ((float4 *)out)[i] = acc;
        }
        // tail of n % 4 elements
        if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
            const size_t j = (n4 << 2) + threadIdx.x;
            float acc = 0.f;
            for (int c = 0; c < t.K; ++c) acc = __fmaf_rn(t.w[c], t.x[c][j], acc);
            out[j] = acc;
        }
    } else {
        for (; i < n; i += stride) {
            float acc = 0.f;
            for (int c = 0; c < t.K; ++c) acc = __fmaf_rn(t.w[c], t.x[c][i], acc);
            out[i] = acc;
        }
    }
}

}  // namespace

size_t lora_grad_partial_floats(int T, int C)
{
    const size_t nchunk = (size_t)(T + GR_ROWS - 1) / GR_ROWS;
    return nchunk * SL_RP * (size_t)C;
}

int launch_lora_grad(const bf16 *X, int ldx, int C, const bf16 *Y, int ldy, int r, int T, float *partials,
                     float *out, int out_is_rxC, hipStream_t st)
{
    if (T <= 0 || C <= 0 || (C % 8) || (ldx % 8) || r < 1 || r > 16) return -1;
    const int nchunk = (T + GR_ROWS - 1) / GR_ROWS;
    dim3 grid((C + GR_COLS - 1) / GR_COLS, nchunk);
    if (r <= 4)
        hipLaunchKernelGGL((lora_grad_partial_kernel<4>), grid, dim3(256), 0, st, X, ldx, C, Y, ldy, r, T, partials);
    else if (r <= 8)
        hipLaunchKernelGGL((lora_grad_partial_kernel<8>), grid, dim3(256), 0, st, X, ldx, C, Y, ldy, r, T, partials);
    else
        hipLaunchKernelGGL((lora_grad_partial_kernel<16>), grid, dim3(256), 0, st, X, ldx, C, Y, ldy, r, T, partials);
    SL_CHECK_LAUNCH("lora_grad_partial");
    hipLaunchKernelGGL(lora_grad_reduce_kernel, dim3((r * C + 63) / 64), dim3(256), 0, st, partials, nchunk, r, C,
                       out, out_is_rxC);
    SL_CHECK_LAUNCH("lora_grad_reduce");
    return 0;
}

int launch_sgd(float *p, const float *g, float lr, size_t n, hipStream_t st)
{
    if (n == 0) return 0;
    size_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(sgd_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, g, lr, n);
    SL_CHECK_LAUNCH("sgd");
    return 0;
}

int launch_cast_pad(const float *src, int rows, int cols, bf16 *dst, int drows, int dcols, int transpose,
                    hipStream_t st)
{
    const int n = drows * dcols;
    hipLaunchKernelGGL(cast_pad_kernel, dim3((n + 255) / 256), dim3(256), 0, st, src, rows, cols, dst, drows, dcols,
                       transpose);
    SL_CHECK_LAUNCH("cast_pad");
    return 0;
}

int launch_transpose_bf16(const bf16 *src, int rows, int cols, bf16 *dst, hipStream_t st)
{
    dim3 grid((cols + 63) / 64, (rows + 63) / 64);
    hipLaunchKernelGGL(transpose_bf16_kernel, grid, dim3(256), 0, st, src, rows, cols, dst);
    SL_CHECK_LAUNCH("transpose");
    return 0;
}

int launch_fill_zero(void *p, size_t bytes, hipStream_t st)
{
    if (bytes == 0) return 0;
    const size_t nwords = bytes / 4;
    size_t blocks = (nwords + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (uint32_t *)p, nwords);
    SL_CHECK_LAUNCH("fill_zero");
    return 0;
}

int launch_fedavg(int K, const float *const *x, const float *w, size_t n, float *out, hipStream_t st)
{
    FedTable t;
    t.K = K;
    bool vec = (((uintptr_t)out) & 15) == 0;
    for (int i = 0; i < K; ++i) {
        t.x[i] = x[i];
        t.w[i] = w[i];
        vec = vec && ((((uintptr_t)x[i]) & 15) == 0);
    }
    const size_t work = vec ? (n >> 2) : n;
    size_t blocks = (work + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 16384) blocks = 16384;
    if (vec) hipLaunchKernelGGL((fedavg_kernel<true>), dim3((unsigned)blocks), dim3(256), 0, st, t, n, out);
    else hipLaunchKernelGGL((fedavg_kernel<false>), dim3((unsigned)blocks), dim3(256), 0, st, t, n, out);
    SL_CHECK_LAUNCH("fedavg");
    return 0;
}
