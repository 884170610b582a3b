// bf16 MFMA GEMM for frozen linears with the rank-r LoRA branch fused on chip (gfx950).
//
//   out[M,N] = epilogue( X[M,K] . W[N,K]^T  +  zscale * (X . Z^T)[M,K2] . T[N,K2]^T )
//
// Forward (SplitLoRA Sec. II-C: W + low-rank product):  Z = A (down-projection, rows
// padded with zeros), T = B (up-projection).  Input-gradient pass: the same kernel on the
// transposed frozen weight with Z = B^T and T = A^T, so no weight gradient is ever formed.
// The rank-space product X.Z^T is accumulated inside the K loop from the X tile that is
// already in LDS, scaled, rounded to bf16, staged through LDS and applied as K2/16 extra
// MFMA steps; the first column tile of a segment also spills it ([M,K2] bf16) because the
// adapter-gradient kernels need it.
//
// Tiling: 256x256x64 block tile, 8 waves (2 x 4), wave tile 128x64 = 4x2 MFMA 32x32x16
// tiles, double-buffered LDS with register prefetch, 16-byte XOR-swizzled LDS rows.
#include "common.h"
#include <vector>

namespace {

constexpr int BM = 256, BN = 256, BK = 64, NTHR = 512;
constexpr int ROWB = BK * 2;                 // bytes per LDS row (one k-slab of a tile row)
constexpr int XB = BM * ROWB, WB = BN * ROWB;

template <int EPI>
__device__ __forceinline__ void store_one(const GemmArgs &a, int row, int col, float v)
{
    const size_t o = (size_t)row * a.ldo + col;
    if (EPI == EPI_STORE) {
        ((bf16 *)a.out0)[o] = f2bf(v);
    } else if (EPI == EPI_RESID) {
        v += ((const float *)a.aux)[o];
        if (a.out0) ((float *)a.out0)[o] = v;
        if (a.out1) ((bf16 *)a.out1)[o] = f2bf(v);
    } else if (EPI == EPI_GELU) {
        ((bf16 *)a.out0)[o] = f2bf(v);
        ((bf16 *)a.out1)[o] = f2bf(gelu_fwd(v));
    } else {   // EPI_DGELU
        float f = bf2f(((const bf16 *)a.aux)[o]);
        ((bf16 *)a.out0)[o] = f2bf(v * gelu_bwd(f));
    }
}

template <int EPI, int NZ>
__global__ __launch_bounds__(NTHR) void gemm_kernel(GemmArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int ZB = NZ * ROWB, STAGE = XB + WB + ZB;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int r32 = lane & 31, g = lane >> 5;

    // ---- tile of this block; consecutive logical tiles go to the same XCD (blocks are
    //      handed to the 8 XCDs round-robin) so an XCD's L2 sees each X row tile once.
    const int tiles_n_seg = (a.seg_n + BN - 1) / BN;
    const int tiles_n = tiles_n_seg * a.nseg;
    const int tiles_m = (a.M + BM - 1) / BM;
    const int nb = tiles_m * tiles_n;
    const int per_xcd = (nb + 7) >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= nb) return;
    const int tm = logical / tiles_n, tn = logical % tiles_n;
    const int seg = tn / tiles_n_seg;
    const int tns = tn % tiles_n_seg;
    const int n0 = seg * a.seg_n + tns * BN;
    const int n_end = (seg + 1) * a.seg_n;
    const int m0 = tm * BM;

    const bool has_z = (NZ > 0) && (a.zmat[seg] != nullptr);

    // ---- global -> register -> LDS assignment: 16-byte chunk lc of row lr + 64 p
    const int lc = tid & 7, lr = tid >> 3;
    const bf16 *xp[4], *wp[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        int row = min(m0 + lr + 64 * p, a.M - 1);
        int n = min(n0 + lr + 64 * p, n_end - 1);
        xp[p] = a.X + (size_t)row * a.ldx + lc * 8;
        wp[p] = a.W + (size_t)n * a.ldw + lc * 8;
    }
    const bf16 *zp = nullptr;
    if (NZ > 0 && has_z && tid < NZ * 8) zp = a.zmat[seg] + (size_t)lr * a.ldz + lc * 8;
    const int st_off = lr * ROWB + ((lc ^ (lr & 7)) << 4);     // (lr + 64p) & 7 == lr & 7

    // Register prefetch: fully unrolled, compile-time indices only (anything less and the staging
    // registers end up in scratch memory).
#define GEMM_GLOAD(k0)                                                           \
    _Pragma("unroll") for (int p = 0; p < 4; ++p) {                              \
        xr[p] = *(const uint4 *)(xp[p] + (k0));                                  \
        wr[p] = *(const uint4 *)(wp[p] + (k0));                                  \
    }                                                                            \
    if (NZ > 0 && zload) zr = *(const uint4 *)(zp + (k0));
#define GEMM_LSTORE(buf)                                                         \
    {                                                                            \
        unsigned char *base_ = smem + (buf) * STAGE + st_off;                    \
        _Pragma("unroll") for (int p = 0; p < 4; ++p) {                          \
            *(uint4 *)(base_ + p * 64 * ROWB) = xr[p];                           \
            *(uint4 *)(base_ + XB + p * 64 * ROWB) = wr[p];                      \
        }                                                                        \
        if (NZ > 0 && zload) *(uint4 *)(base_ + XB + WB) = zr;                   \
    }
#define GEMM_COMPUTE(buf)                                                                              \
    {                                                                                                  \
        const unsigned char *Xs = smem + (buf) * STAGE;                                                \
        const unsigned char *Ws = Xs + XB;                                                             \
        const unsigned char *Zs = Ws + WB;                                                             \
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {                                             \
            const int co = ((ks * 2 + g) ^ sw) << 4;                                                   \
            bf16x8 af[4], bfr[2];                                                                      \
            _Pragma("unroll") for (int i = 0; i < 4; ++i)                                              \
                af[i] = *(const bf16x8 *)(Xs + a_row + i * 32 * ROWB + co);                            \
            _Pragma("unroll") for (int j = 0; j < 2; ++j)                                              \
                bfr[j] = *(const bf16x8 *)(Ws + b_row + j * 32 * ROWB + co);                           \
            _Pragma("unroll") for (int i = 0; i < 4; ++i)                                              \
                _Pragma("unroll") for (int j = 0; j < 2; ++j)                                          \
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0); \
            if (NZ > 0 && has_z) {                                                                     \
                bf16x8 za = *(const bf16x8 *)(Xs + z_row + co);                                        \
                _Pragma("unroll") for (int q = 0; q < NZ / 32; ++q) {                                  \
                    bf16x8 zb = *(const bf16x8 *)(Zs + (q * 32 + r32) * ROWB + co);                    \
                    zacc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(za, zb, zacc[q], 0, 0, 0);       \
                }                                                                                      \
            }                                                                                          \
        }                                                                                              \
    }

    uint4 xr[4], wr[4], zr = {0, 0, 0, 0};
    const bool zload = (zp != nullptr);

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    f32x16 zacc[NZ > 0 ? NZ / 32 : 1];
#pragma unroll
    for (int q = 0; q < (NZ > 0 ? NZ / 32 : 1); ++q)
#pragma unroll
        for (int e = 0; e < 16; ++e) zacc[q][e] = 0.0f;

    const int a_row = (wm * 128 + r32) * ROWB;
    const int b_row = (wn * 64 + r32) * ROWB;
    const int z_row = (wm * 128 + wn * 32 + r32) * ROWB;
    const int sw = r32 & 7;

    const int nk = a.K / BK;
    GEMM_GLOAD(0)
    GEMM_LSTORE(0)
    __syncthreads();
    for (int kt = 0; kt < nk - 1; ++kt) {
        GEMM_GLOAD((kt + 1) * BK)
        GEMM_COMPUTE(kt & 1)
        GEMM_LSTORE((kt + 1) & 1)
        __syncthreads();
    }
    GEMM_COMPUTE((nk - 1) & 1)
    __syncthreads();
#undef GEMM_GLOAD
#undef GEMM_LSTORE
#undef GEMM_COMPUTE

    // ---- low-rank tail: acc += (zscale * z)[256,K2] . T[n,K2]^T -----------------------------
    if (NZ > 0 && has_z) {
        constexpr int ZP = NZ + 8;                       // LDS pitch of the z tile, in elements
        bf16 *zs = (bf16 *)smem;                         // the K loop is over: reuse stage 0
        const bf16 *tm_ = a.tmat[seg];
        const int nks = a.K2 >> 4;
        // issue the up-projection operand loads early (L2 hits; at most 4 k-steps of 16)
        bf16x8 tb[4][2];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                int n = min(n0 + wn * 64 + j * 32 + r32, n_end - 1) - seg * a.seg_n;
                if (ks < nks) tb[ks][j] = *(const bf16x8 *)(tm_ + (size_t)n * a.ldt + ks * 16 + g * 8);
            }
#pragma unroll
        for (int q = 0; q < NZ / 32; ++q)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                int row = wm * 128 + wn * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                zs[row * ZP + q * 32 + r32] = f2bf(zacc[q][e] * a.zscale);
            }
        __syncthreads();
        if (a.zspill[seg] != nullptr && tns == 0) {
            const int cpr = a.K2 >> 3;                   // 16-byte chunks per row
            for (int c = tid; c < BM * cpr; c += NTHR) {
                int row = c / cpr, cc = c - row * cpr;
                if (m0 + row < a.M)
                    *(uint4 *)(a.zspill[seg] + (size_t)(m0 + row) * a.K2 + cc * 8) =
                        *(const uint4 *)(zs + row * ZP + cc * 8);
            }
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < nks) {
                bf16x8 af[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    af[i] = *(const bf16x8 *)(zs + (wm * 128 + i * 32 + r32) * ZP + ks * 16 + g * 8);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], tb[ks][j], acc[i][j], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: lane holds column (lane & 31) of each 32x32 tile, rows 8(e/4) + 4g + e%4
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int col = n0 + wn * 64 + j * 32 + r32;
        if (col >= n_end) continue;
        const float bias = a.bias ? bf2f(a.bias[col]) : 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rb = m0 + wm * 128 + i * 32 + 4 * g;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = rb + 8 * (e >> 2) + (e & 3);
                if (row < a.M) store_one<EPI>(a, row, col, acc[i][j][e] + bias);
            }
        }
    }
}

template <int EPI, int NZ>
int launch_t(const GemmArgs &a, hipStream_t st)
{
    constexpr int smem = 2 * (XB + WB + NZ * ROWB);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_kernel<EPI, NZ>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) { set_hip_error(e, "gemm smem attribute"); return -4; }
        attr_set = true;
    }
    const int tiles_n = ((a.seg_n + BN - 1) / BN) * a.nseg;
    const int tiles_m = (a.M + BM - 1) / BM;
    const int nb = tiles_m * tiles_n;
    const int grid = ((nb + 7) / 8) * 8;
    hipLaunchKernelGGL((gemm_kernel<EPI, NZ>), dim3(grid), dim3(NTHR), smem, st, a);
    SL_CHECK_LAUNCH("gemm");
    return 0;
}

template <int EPI>
int launch_e(const GemmArgs &a, int nz, hipStream_t st)
{
    switch (nz) {
    case 0: return launch_t<EPI, 0>(a, st);
    case 32: return launch_t<EPI, 32>(a, st);
    case 64: return launch_t<EPI, 64>(a, st);
    }
    return -1;
}

// ---- optional timing of the GEMM launches with HIP events (measurement hook) ---------------------
struct GemmProf {
    bool on = false;
    std::vector<hipEvent_t> ev;      // pairs: start, stop
    size_t used = 0;
    double flop = 0.0;
} g_prof;

}  // namespace

int gemm_prof_enable(int on)
{
    if (on && g_prof.ev.empty()) {
        g_prof.ev.resize(16384);
        for (auto &e : g_prof.ev)
            if (hipEventCreate(&e) != hipSuccess) { g_prof.ev.clear(); return -4; }
    }
    g_prof.on = on != 0;
    g_prof.used = 0;
    g_prof.flop = 0.0;
    return 0;
}

int gemm_prof_read(double *ms, double *flop, int *launches)
{
    double tot = 0.0;
    for (size_t i = 0; i + 1 < g_prof.used; i += 2) {
        float t = 0.f;
        if (hipEventSynchronize(g_prof.ev[i + 1]) != hipSuccess) return -4;
        if (hipEventElapsedTime(&t, g_prof.ev[i], g_prof.ev[i + 1]) != hipSuccess) return -4;
        tot += t;
    }
    if (ms) *ms = tot;
    if (flop) *flop = g_prof.flop;
    if (launches) *launches = (int)(g_prof.used / 2);
    g_prof.used = 0;
    g_prof.flop = 0.0;
    return 0;
}

static int launch_gemm_inner(const GemmArgs &a, int epi, int nz, hipStream_t st);

int launch_gemm(const GemmArgs &a, int epi, int nz, hipStream_t st)
{
    const bool rec = g_prof.on && g_prof.used + 2 <= g_prof.ev.size();
    if (rec) (void)hipEventRecord(g_prof.ev[g_prof.used], st);
    const int rc = launch_gemm_inner(a, epi, nz, st);
    if (rec) {
        (void)hipEventRecord(g_prof.ev[g_prof.used + 1], st);
        g_prof.used += 2;
        // algorithmic work of this launch: the frozen product only (the rank-r branch adds < 1 %
        // and is left out, which understates the achieved rate slightly)
        const double f = 2.0 * a.M * (double)a.N * a.K;
        g_prof.flop += f;
    }
    return rc;
}

static int launch_gemm_inner(const GemmArgs &a, int epi, int nz, hipStream_t st)
{
    if (a.M <= 0 || a.N <= 0 || a.K <= 0 || (a.K % BK) != 0 || a.nseg < 1 || a.nseg > 3 ||
        a.nseg * a.seg_n != a.N || (a.ldx % 8) || (a.ldw % 8))
        return -1;
    if (nz > 0 && (a.K2 < 16 || a.K2 > nz || (a.K2 % 16) || (a.ldt % 8) || (a.ldz % 8))) return -1;
    switch (epi) {
    case EPI_STORE: return launch_e<EPI_STORE>(a, nz, st);
    case EPI_RESID: return launch_e<EPI_RESID>(a, nz, st);
    case EPI_GELU: return launch_e<EPI_GELU>(a, nz, st);
    case EPI_DGELU: return launch_e<EPI_DGELU>(a, nz, st);
    }
    return -1;
}
