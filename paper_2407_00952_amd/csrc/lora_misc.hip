// Adapter-side kernels: LoRA gradients, SGD step, FedAvg, and the bf16 shadow copies.
//
//  * LoRA gradients (SplitLoRA Sec. III-B step a3: "derive the server-side LoRA adapters'
//    gradients"): with ps = s (dy B) and zs = s (x A^T) spilled by the GEMMs,
//        dA = ps^T x   [r,in]        dB = dy^T zs   [out,r]
//    Both are G[c,j] = sum_t X[t,c] Y[t,j] with a tall X [T,C] and a skinny Y [T,16]: one
//    streaming pass over X (HBM-bound) feeding MFMAs whose operands are read along the token
//    axis with the LDS transpose read, per-chunk partial sums, then a fixed-order reduction
//    over chunks -- no floating-point atomics, so results are reproducible.  Y must have 16
//    readable columns per row (the spilled rank-space activations are padded with zeros).
//  * SGD (Eq. 4-5): p = fmaf(-lr, g, p).
//  * FedAvg (Sec. III-B step b2, Eq. 8-9): acc = fmaf(w_i, x_i[j], acc), i = 0..K-1.
#include "common.h"
#include "prof.h"

namespace {

constexpr int GR_ROWS = 512;   // token rows per block: 8 tiles of 64
constexpr int GR_COLS = 256;   // columns of X per block: 64 per wavefront (two MFMA row tiles)
constexpr int GX_TILE = 64 * GR_COLS * 2;   // bytes of one 64-token X tile in LDS

typedef short v4s_t __attribute__((ext_vector_type(4)));
#define LG_GLDS(gp, lp)                                                                            \
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gp),         \
                                     (__attribute__((address_space(3))) void *)(lp), 16, 0, 0)
#define LG_WAIT_VM0() __builtin_amdgcn_s_waitcnt(0x0F70)

// LDS transpose read (see attention.hip): lane (m = lane%32, g = lane/32) gets column col0 + m of the
// 8 rows tok0 + 8h + 4g + e of a row-major tile.  X tile: 512-byte rows, 64-byte granules XOR-swizzled
// with the row so that the four rows one read touches fall into different banks.
__device__ __forceinline__ bf16x8 xfrag_tr(const unsigned char *t, int col0, int tok0, int lane)
{
    const int q = lane & 3, e = (lane >> 2) & 3, half = (lane >> 4) & 1, g = lane >> 5;
    const int col = col0 + 16 * half + 4 * q;
    const int row0 = tok0 + 4 * g + e, row1 = row0 + 8;
    const unsigned char *a0 = t + row0 * 512 + ((((col >> 3)) ^ ((row0 & 7) << 2)) << 4) + (col & 7) * 2;
    const unsigned char *a1 = t + row1 * 512 + ((((col >> 3)) ^ ((row1 & 7) << 2)) << 4) + (col & 7) * 2;
    union { v4s_t s[2]; bf16x8 v; } u;
    u.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s_t *)a0);
    u.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s_t *)a1);
    return u.v;
}
// Y tile: [64 tokens][16] bf16 in 32-byte rows (every lane group reads columns 0..15; the MFMA columns
// 16..31 then hold copies that are never stored), or, for two adapters at once, [64][32] bf16 in rows of
// 96 bytes (64 used): with that pitch the four rows one read touches fall into different banks.
template <bool DUAL>
__device__ __forceinline__ bf16x8 yfrag_tr(const unsigned char *t, int tok0, int lane)
{
    constexpr int YP = DUAL ? 96 : 32;
    const int q = lane & 3, e = (lane >> 2) & 3, half = (lane >> 4) & 1, g = lane >> 5;
    const int row0 = tok0 + 4 * g + e, row1 = row0 + 8;
    const int co = (DUAL ? half * 32 : 0) + q * 8;
    union { v4s_t s[2]; bf16x8 v; } u;
    u.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s_t *)(t + row0 * YP + co));
    u.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s_t *)(t + row1 * YP + co));
    return u.v;
}

// partial[chunk][j][c] = sum over the chunk's tokens of X[t,c] * Y[t,j]  on the matrix cores:
// D[m = c][n = j] += X^T[c][t] * Y[t][j], both operands read along the token axis with the LDS
// transpose read from row-major tiles that asynchronous copies (X) and plain loads (Y) fill.
// DUAL: Y holds two adapters' rank-space columns side by side (16 + 16); their partial results are
// stored one after the other (rows 0..r-1 and r..2r-1 of the chunk), so X is streamed once for both.
template <bool DUAL>
__device__ __forceinline__ void lora_grad_partial_body(const bf16 *__restrict__ X, int ldx, int C,
                                                       const bf16 *__restrict__ Y, int ldy, int r, int T,
                                                       float *__restrict__ partials, unsigned char *X0,
                                                       unsigned char *X1, unsigned char *Y0, unsigned char *Y1)
{
    constexpr int YP = DUAL ? 96 : 32;
    const int tid = threadIdx.x, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c_blk = blockIdx.x * GR_COLS;
    const int chunk = blockIdx.y;
    const int t_begin = chunk * GR_ROWS;
    const int ntile = (min(T, t_begin + GR_ROWS) - t_begin + 63) >> 6;
    const bool wave_ok = c_blk + wave * 64 < C;          // C is a multiple of 64

    // X copy: each instruction moves 2 token rows x 512 B; lane l -> row l>>5, physical 16-byte slot
    // l&31 which holds logical slot (l&31) ^ ((row&7)<<2).  32 instructions per tile, 8 per wave.
    const int xrow = lane >> 5, xslot = lane & 31;
    // Y copy: 16 B per thread (128 threads for one adapter, 256 for two), through a register (committed
    // to LDS after the MFMA work)
    constexpr int YTHR = DUAL ? 256 : 128, YSH = DUAL ? 2 : 1, YMASK = DUAL ? 3 : 1;
    uint4 yreg = {0, 0, 0, 0};
#define LG_ISSUE(Xs, jj)                                                                           \
    {                                                                                              \
        const int t0_ = t_begin + (jj) * 64;                                                       \
        if (tid < YTHR) {                                                                          \
            const int tr_ = t0_ + (tid >> YSH);                                                    \
            yreg = make_uint4(0, 0, 0, 0);                                                         \
            if (tr_ < T) yreg = *(const uint4 *)(Y + (size_t)tr_ * ldy + (tid & YMASK) * 8);       \
        }                                                                                          \
        _Pragma("unroll") for (int p = 0; p < 8; ++p) {                                            \
            const int row_ = (wave * 8 + p) * 2 + xrow;                                            \
            const int tg_ = min(t0_ + row_, T - 1);                                                \
            const int lslot_ = xslot ^ ((row_ & 7) << 2);                                          \
            const int cg_ = min(c_blk + lslot_ * 8, C - 8);                                        \
            LG_GLDS(X + (size_t)tg_ * ldx + cg_, (Xs) + (wave * 8 + p) * 1024);                    \
        }                                                                                          \
    }
#define LG_COMMIT(Ys) if (tid < YTHR) *(uint4 *)((Ys) + (tid >> YSH) * YP + (tid & YMASK) * 16) = yreg;
#define LG_TILE(Xs, Ys)                                                                            \
    if (wave_ok) {                                                                                 \
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {                                         \
            const bf16x8 yb = yfrag_tr<DUAL>(Ys, ks * 16, lane);                                   \
            _Pragma("unroll") for (int mt = 0; mt < 2; ++mt)                                       \
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                 \
                    xfrag_tr(Xs, wave * 64 + mt * 32, ks * 16, lane), yb, acc[mt], 0, 0, 0);       \
        }                                                                                          \
    }

    f32x16 acc[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[mt][e] = 0.f;

    LG_ISSUE(X0, 0)
    LG_COMMIT(Y0)
    LG_WAIT_VM0();
    __syncthreads();
    int j = 0;
    for (; j + 2 <= ntile; j += 2) {
        LG_ISSUE(X1, j + 1)
        LG_TILE(X0, Y0)
        LG_COMMIT(Y1)
        LG_WAIT_VM0();
        __syncthreads();
        const bool more = j + 2 < ntile;
        if (more) LG_ISSUE(X0, j + 2)
        LG_TILE(X1, Y1)
        if (more) LG_COMMIT(Y0)
        LG_WAIT_VM0();
        __syncthreads();
    }
    if (j < ntile) LG_TILE(X0, Y0)
#undef LG_ISSUE
#undef LG_COMMIT
#undef LG_TILE

    // lane holds column j = lane%32 of D, rows c = 8(e/4) + 4g + e%4 of each 32-row tile
    const int nrows = DUAL ? 2 * r : r;
    const int jrow = (DUAL && r32 >= 16) ? r + r32 - 16 : r32;
    if (wave_ok && (r32 & 15) < r && (DUAL || r32 < 16)) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const int c = c_blk + wave * 64 + mt * 32 + 8 * e4 + 4 * g;
                *(float4 *)(partials + ((size_t)chunk * nrows + jrow) * C + c) =
                    make_float4(acc[mt][4 * e4], acc[mt][4 * e4 + 1], acc[mt][4 * e4 + 2], acc[mt][4 * e4 + 3]);
            }
    }
}

// One launch for every adapter gradient that is due at one point of the backward pass (after the fused
// q|k|v input-gradient product: dB of each adapted projection and dA of all of them): blockIdx.z picks the
// job.  The jobs are a few dozen microseconds of streaming each, so launching them one by one (and their
// reductions one by one) left the chip half idle between them.
struct LoraGradJob {
    const bf16 *X; const bf16 *Y;    // tall operand [T,C] (pitch ldx), skinny operand [T,16 or 32] (pitch ldy)
    float *partials;                 // this job's chunk partial sums
    float *out_a, *out_b;            // result(s); out_b only for a dual job
    int ldx, ldy, C, dual, out_is_rxC;
};
constexpr int LG_MAX_JOBS = 6;
struct LoraGradJobs { LoraGradJob j[LG_MAX_JOBS]; };

__global__ __launch_bounds__(256) void lora_grad_partial_kernel(LoraGradJobs jobs, int r, int T)
{
    __shared__ __attribute__((aligned(1024))) unsigned char X0[GX_TILE], X1[GX_TILE];
    __shared__ __attribute__((aligned(16))) unsigned char Y0[64 * 96], Y1[64 * 96];
    const LoraGradJob &jb = jobs.j[blockIdx.z];
    if ((int)blockIdx.x * GR_COLS >= jb.C) return;       // this job's operand is narrower than the widest one
    if (jb.dual) lora_grad_partial_body<true>(jb.X, jb.ldx, jb.C, jb.Y, jb.ldy, r, T, jb.partials, X0, X1, Y0, Y1);
    else lora_grad_partial_body<false>(jb.X, jb.ldx, jb.C, jb.Y, jb.ldy, r, T, jb.partials, X0, X1, Y0, Y1);
}

// out[j, c] = sum over chunks, in a fixed order: each of the 4 wavefronts of a block sums a
// contiguous quarter of the chunks in increasing order, then the four are added in order.
// With a second output, rows r..2r-1 of every chunk belong to it (two adapters reduced in one launch).
__global__ __launch_bounds__(256) void lora_grad_reduce_kernel(LoraGradJobs jobs, int nchunk, int r)
{
    __shared__ float red[3][64];
    const LoraGradJob &jb = jobs.j[blockIdx.z];
    const float *__restrict__ partials = jb.partials;
    const int C = jb.C, out_is_rxC = jb.out_is_rxC;
    float *__restrict__ out = jb.out_a;
    float *__restrict__ out_second = jb.dual ? jb.out_b : nullptr;
    if ((int)blockIdx.x * 64 >= (jb.dual ? 2 * r : r) * C) return;      // (uniform: before the barrier)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nrows = out_second ? 2 * r : r;
    const int idx = blockIdx.x * 64 + lane;              // over nrows*C, c fastest
    const bool ok = idx < nrows * C;
    const int j = ok ? idx / C : 0, c = ok ? idx - j * C : 0;
    const int per = (nchunk + 3) >> 2;
    const int k0 = wave * per, k1 = min(k0 + per, nchunk);
    float s = 0.f;
    if (ok) {
        const float *src = partials + (size_t)j * C + c;
        const size_t step = (size_t)nrows * C;
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
        float *dst = j < r ? out : out_second;
        const int jj = j < r ? j : j - r;
        if (out_is_rxC) dst[(size_t)jj * C + c] = s;
        else dst[(size_t)c * r + jj] = s;
    }
}

__global__ __launch_bounds__(256) void sgd_kernel(float *__restrict__ p, const float *__restrict__ g, float lr,
                                                  size_t n)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) p[i] = __fmaf_rn(-lr, g[i], p[i]);
}

// AdamW variant of the adapter update (the paper's Eq. 4-7 are plain SGD; this is the usual Adam rule
// with decoupled weight decay, in one fixed evaluation order so that results are bit-reproducible):
//   m = fmaf(b1, m, o1*g);  v = fmaf(b2, v, (o2*g)*g);  p = fmaf(-a, m / fmaf(sqrtf(v), c, eps), p*decay)
// with the scalars decay, a, c, o1, o2 prepared on the host in double precision.
__global__ __launch_bounds__(256) void adamw_kernel(float *__restrict__ p, const float *__restrict__ g,
                                                    float *__restrict__ m, float *__restrict__ v, size_t n, float b1,
                                                    float b2, float eps, float decay, float a, float c, float o1,
                                                    float o2)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) {
        const float gj = g[i];
        const float t1 = o1 * gj;
        const float mj = __fmaf_rn(b1, m[i], t1);
        const float t2 = o2 * gj;
        const float t3 = t2 * gj;
        const float vj = __fmaf_rn(b2, v[i], t3);
        // plain sqrtf and / are the correctly rounded ones (the compiler's default for fp32 in device code)
        const float den = __fmaf_rn(sqrtf(vj), c, eps);
        const float q = mj / den;
        const float pd = p[i] * decay;
        p[i] = __fmaf_rn(-a, q, pd);
        m[i] = mj;
        v[i] = vj;
    }
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
    return nchunk * 2 * SL_RP * (size_t)C;               // room for two adapters reduced together
}

int launch_lora_grad_jobs(const LoraGradDesc *d, int njobs, int r, int T, hipStream_t st)
{
    if (njobs < 1 || njobs > LG_MAX_JOBS || T <= 0 || r < 1 || r > 16) return SL_EINVAL;
    LoraGradJobs jobs;
    int max_c = 0, max_red = 0;
    double bytes = 0.0;
    for (int k = 0; k < njobs; ++k) {
        const LoraGradDesc &q = d[k];
        if (!q.X || !q.Y || !q.partials || !q.out_a || (q.dual && !q.out_b)) return SL_EINVAL;
        if (q.C <= 0 || (q.C % 64) || (q.ldx % 8) || (q.ldy % 8) || (q.dual && q.ldy < 32)) return SL_EINVAL;
        jobs.j[k] = {q.X, q.Y, q.partials, q.out_a, q.out_b, q.ldx, q.ldy, q.C, q.dual ? 1 : 0, q.out_is_rxC};
        max_c = q.C > max_c ? q.C : max_c;
        const int red = (q.dual ? 2 * r : r) * q.C;
        max_red = red > max_red ? red : max_red;
        bytes += 2.0 * T * (double)q.C;                  // the streaming pass: the tall operand once
    }
    const int nchunk = (T + GR_ROWS - 1) / GR_ROWS;
    const bool rec = prof_begin(PK_LORA_GRAD, st);
    hipLaunchKernelGGL(lora_grad_partial_kernel, dim3((max_c + GR_COLS - 1) / GR_COLS, nchunk, njobs), dim3(256), 0, st,
                       jobs, r, T);
    prof_end(rec, PK_LORA_GRAD, bytes, st);
    SL_CHECK_LAUNCH("lora_grad_partial");
    hipLaunchKernelGGL(lora_grad_reduce_kernel, dim3((max_red + 63) / 64, 1, njobs), dim3(256), 0, st, jobs, nchunk, r);
    SL_CHECK_LAUNCH("lora_grad_reduce");
    return 0;
}

int launch_lora_grad(const bf16 *X, int ldx, int C, const bf16 *Y, int ldy, int r, int T, float *partials,
                     float *out, int out_is_rxC, hipStream_t st)
{
    const LoraGradDesc d = {X, Y, partials, out, nullptr, ldx, ldy, C, false, out_is_rxC};
    return launch_lora_grad_jobs(&d, 1, r, T, st);
}

// Two adapters that share X: Y carries their rank-space columns in [0,16) and [16,32) of each row.
int launch_lora_grad_pair(const bf16 *X, int ldx, int C, const bf16 *Y, int ldy, int r, int T, float *partials,
                          float *out_a, float *out_b, int out_is_rxC, hipStream_t st)
{
    const LoraGradDesc d = {X, Y, partials, out_a, out_b, ldx, ldy, C, true, out_is_rxC};
    return launch_lora_grad_jobs(&d, 1, r, T, st);
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

int launch_adamw(float *p, const float *g, float *m, float *v, size_t n, float b1, float b2, float eps, float decay,
                 float a, float c, float o1, float o2, hipStream_t st)
{
    if (n == 0) return 0;
    size_t blocks = (n + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(adamw_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, g, m, v, n, b1, b2, eps, decay, a, c,
                       o1, o2);
    SL_CHECK_LAUNCH("adamw");
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
    const bool rec = prof_begin(PK_FEDAVG, st);
    if (vec) hipLaunchKernelGGL((fedavg_kernel<true>), dim3((unsigned)blocks), dim3(256), 0, st, t, n, out);
    else hipLaunchKernelGGL((fedavg_kernel<false>), dim3((unsigned)blocks), dim3(256), 0, st, t, n, out);
    prof_end(rec, PK_FEDAVG, 4.0 * (K + 1) * (double)n, st);
    SL_CHECK_LAUNCH("fedavg");
    return 0;
}
