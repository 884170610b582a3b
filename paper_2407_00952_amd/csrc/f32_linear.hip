// Single-precision LoRA-adapted linear layer (SplitLoRA Sec. II-C), forward and backward.
// Every product is one launch of a small LDS-tiled FMA GEMM with general strides:
//     C[m,n] = beta * C[m,n] + alpha * sum_k A(m,k) B(k,n)  (+ bias[n])
// Sums run over k in increasing order inside one thread, so results are reproducible.
// This path exists for accuracy (<= 1e-4 against an fp64 reference), not for speed.
#include "common.h"

namespace {

constexpr int TS = 64, TK = 16;

__global__ __launch_bounds__(256) void sgemm_kernel(int M, int N, int K, const float *__restrict__ A, long sam,
                                                    long sak, const float *__restrict__ B, long sbk, long sbn,
                                                    float *__restrict__ C, long ldc, float alpha, float beta,
                                                    const float *__restrict__ bias)
{
    __shared__ float As[TK][TS + 1];
    __shared__ float Bs[TK][TS + 1];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (int k0 = 0; k0 < K; k0 += TK) {
        for (int i = threadIdx.x; i < TS * TK; i += 256) {
            // choose the fast index along the unit stride of the operand
            int mm, kk;
            if (sak == 1) { kk = i % TK; mm = i / TK; } else { mm = i % TS; kk = i / TS; }
            float v = 0.f;
            if (m0 + mm < M && k0 + kk < K) v = A[(long)(m0 + mm) * sam + (long)(k0 + kk) * sak];
            As[kk][mm] = v;
            int nn, k2;
            if (sbk == 1) { k2 = i % TK; nn = i / TK; } else { nn = i % TS; k2 = i / TS; }
            float w = 0.f;
            if (n0 + nn < N && k0 + k2 < K) w = B[(long)(k0 + k2) * sbk + (long)(n0 + nn) * sbn];
            Bs[k2][nn] = w;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float v = alpha * acc[i][j];
            if (bias) v += bias[n];
            if (beta != 0.f) v += beta * C[(long)m * ldc + n];
            C[(long)m * ldc + n] = v;
        }
    }
}

int sgemm(int M, int N, int K, const float *A, long sam, long sak, const float *B, long sbk, long sbn, float *C,
          long ldc, float alpha, float beta, const float *bias, hipStream_t st)
{
    dim3 grid((N + TS - 1) / TS, (M + TS - 1) / TS);
    hipLaunchKernelGGL(sgemm_kernel, grid, dim3(256), 0, st, M, N, K, A, sam, sak, B, sbk, sbn, C, ldc, alpha, beta,
                       bias);
    SL_CHECK_LAUNCH("sgemm");
    return 0;
}

}  // namespace

// ws: z [T,r] then p [T,r]
int f32_lora_linear_fwd(int T, int n_in, int n_out, int r, float s, const float *x, const float *W,
                        const float *bias, const float *A, const float *B, float *y, float *ws, hipStream_t st)
{
    float *z = ws;
    int rc;
    // y = x W^T + bias
    if ((rc = sgemm(T, n_out, n_in, x, n_in, 1, W, 1, n_in, y, n_out, 1.f, 0.f, bias, st))) return rc;
    // z = x A^T
    if ((rc = sgemm(T, r, n_in, x, n_in, 1, A, 1, n_in, z, r, 1.f, 0.f, nullptr, st))) return rc;
    // y += s z B^T
    return sgemm(T, n_out, r, z, r, 1, B, 1, r, y, n_out, s, 1.f, nullptr, st);
}

int f32_lora_linear_bwd(int T, int n_in, int n_out, int r, float s, const float *x, const float *dy,
                        const float *W, const float *A, const float *B, float *dx, float *dA, float *dB, float *ws,
                        hipStream_t st)
{
    float *z = ws, *p = ws + (size_t)T * r;
    int rc;
    // z = x A^T ; p = dy B
    if ((rc = sgemm(T, r, n_in, x, n_in, 1, A, 1, n_in, z, r, 1.f, 0.f, nullptr, st))) return rc;
    if ((rc = sgemm(T, r, n_out, dy, n_out, 1, B, r, 1, p, r, 1.f, 0.f, nullptr, st))) return rc;
    // dx = dy W + s p A
    if ((rc = sgemm(T, n_in, n_out, dy, n_out, 1, W, n_in, 1, dx, n_in, 1.f, 0.f, nullptr, st))) return rc;
    if ((rc = sgemm(T, n_in, r, p, r, 1, A, n_in, 1, dx, n_in, s, 1.f, nullptr, st))) return rc;
    // dA = s p^T x   [r,in] ;  dB = s dy^T z   [out,r]
    if ((rc = sgemm(r, n_in, T, p, 1, r, x, n_in, 1, dA, n_in, s, 0.f, nullptr, st))) return rc;
    return sgemm(n_out, r, T, dy, 1, n_out, z, r, 1, dB, r, s, 0.f, nullptr, st);
}
