// Compressed frozen linears and cut-layer traffic in the OCP microscaling format MXFP8 (gfx950).
//
// SplitLoRA names quantisation as the route to a more storage-, communication- and computation-
// efficient framework (Sec. V-B) without fixing a format.  The format here is MXFP8 of the OCP
// Microscaling Formats (MX) v1.0 specification: blocks of 32 consecutive elements along the
// contraction axis share one power-of-two scale (E8M0 byte, value 2^(code-127)); elements are FP8
// E4M3 (bias 7, largest finite value 448, S.1111.111 = NaN, no infinities).  CDNA4's matrix cores
// take exactly this: V_MFMA_SCALE_F32_16X16X128_F8F6F4 multiplies two 16 x 128 fp8 operands and
// applies one E8M0 scale per 32-element block of each, at twice the bf16 rate.
//
//   mx_quantize    bf16 [M,K]  -> codes u8 [M,K] + scales u8 [M,K/32]      (MX v1.0 Sec. 6.3)
//   mx_dequantize  codes + scales -> bf16 [M,K]                            (exact unless out of bf16 range)
//   linear         y[M,N] = deq(x)[M,K] . deq(W)[N,K]^T + bias             bf16 out, fp32 accumulation
//
// Operand layout of the scaled MFMA (checked on the device against a CPU product): lane l holds row
// l%16 of its operand; with g = l/16 its eight dwords are bytes [16g, 16g+16) and [64+16g, 64+16g+16)
// of the row's 128-byte k-slab; the scale it supplies (byte `opsel` of the scale register) belongs to
// block g, i.e. to bytes [32g, 32g+32) of the slab.  Output as for the bf16 shapes: column l%16,
// rows 4g + e.
#include "../../include/slora.h"
#include "common.h"
#include "gemm_epilogue.h"
#include "mx_codec.h"

namespace {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------------
// conversion kernels
// ------------------------------------------------------------------------------------------------

// Each thread converts 8 consecutive elements of a row; 4 neighbouring threads form a block of 32.
// Grid: x = row, y = 128-chunk slice of the row (no index division: the kernel is ALU-bound, not HBM-bound).
__global__ __launch_bounds__(128) void mx_quantize_kernel(const bf16 *__restrict__ x, long long ldx, long long M, int K,
                                                          unsigned char *__restrict__ codes,
                                                          unsigned char *__restrict__ scales)
{
    const int cpr = K >> 3;                              // 16-byte chunks per row
    const long long row = blockIdx.x;
    const int ch = blockIdx.y * 128 + threadIdx.x;
    const bool live = ch < cpr;
    uint4 raw = make_uint4(0u, 0u, 0u, 0u);
    if (live) raw = *(const uint4 *)(x + row * ldx + ch * 8);   // (M is the grid's x extent)
    const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
    // largest magnitude of the block, compared on the bit patterns (monotone for finite values)
    unsigned mag = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        mag = max(mag, w[i] & 0x7FFFu);
        mag = max(mag, (w[i] >> 16) & 0x7FFFu);
    }
    mag = max(mag, (unsigned)__shfl_xor((int)mag, 1, 64));
    mag = max(mag, (unsigned)__shfl_xor((int)mag, 2, 64));
    const int scode = mx_scale_code(mag);
    unsigned out[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 4; ++i)                           // w[i] holds elements 2i (low half) and 2i + 1
        out[i >> 1] |= mx_encode_pair_bf16(w[i] & 0xFFFFu, w[i] >> 16, scode) << (16 * (i & 1));
    if (live) {
        *(uint2 *)(codes + row * (long long)K + ch * 8) = make_uint2(out[0], out[1]);
        if ((ch & 3) == 0) scales[row * (long long)(K >> 5) + (ch >> 2)] = (unsigned char)scode;
    }
}

// The same for FP4 E2M1 elements (frozen weights): emax 2, so the scale code is the biased exponent - 2;
// two codes per byte, the element with the even index in the low nibble.
__global__ __launch_bounds__(128) void mx_quantize_fp4_kernel(const bf16 *__restrict__ x, long long ldx, long long M,
                                                              int K, unsigned char *__restrict__ codes,
                                                              unsigned char *__restrict__ scales)
{
    const int cpr = K >> 3;                              // 16-byte chunks per row
    const long long row = blockIdx.x;
    const int ch = blockIdx.y * 128 + threadIdx.x;
    const bool live = ch < cpr;
    uint4 raw = make_uint4(0u, 0u, 0u, 0u);
    if (live) raw = *(const uint4 *)(x + row * ldx + ch * 8);
    const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
    unsigned mag = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        mag = max(mag, w[i] & 0x7FFFu);
        mag = max(mag, (w[i] >> 16) & 0x7FFFu);
    }
    mag = max(mag, (unsigned)__shfl_xor((int)mag, 1, 64));
    mag = max(mag, (unsigned)__shfl_xor((int)mag, 2, 64));
    const int scode = max((int)(mag >> 7) - 2, 0);
    unsigned out = 0u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const unsigned h = (i & 1) ? (w[i >> 1] >> 16) : (w[i >> 1] & 0xFFFFu);
        out |= mx_encode_fp4_bf16(h, scode) << (4 * i);
    }
    if (live) {
        *(unsigned *)(codes + row * (long long)(K >> 1) + ch * 4) = out;
        if ((ch & 3) == 0) scales[row * (long long)(K >> 5) + (ch >> 2)] = (unsigned char)scode;
    }
}

__global__ __launch_bounds__(256) void mx_dequantize_kernel(const unsigned char *__restrict__ codes,
                                                            const unsigned char *__restrict__ scales, long long M,
                                                            int K, bf16 *__restrict__ y, long long ldy)
{
    const int cpr = K >> 3;
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= M * cpr) return;
    const long long row = t / cpr;
    const int ch = (int)(t - row * cpr);
    const uint2 raw = *(const uint2 *)(codes + row * (long long)K + ch * 8);
    const int scode = scales[row * (long long)(K >> 5) + (ch >> 2)];
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const unsigned c = ((i < 4 ? raw.x : raw.y) >> (8 * (i & 3))) & 0xFFu;
        o[i] = f2bf(ldexpf(mx_e4m3_to_f32(c), scode - 127));
    }
    *(bf16x8 *)(y + row * ldy + ch * 8) = o;
}

// ------------------------------------------------------------------------------------------------
// GEMM: 256 x 256 x 128 block tile, 8 waves (2 x 4), wave tile 128 x 64 = 8 x 4 scaled MFMA tiles.
// Same skeleton as the bf16 GEMM (a 128-byte LDS row is one k-slab of a tile row, two stages filled by
// asynchronous global->LDS copies, 16-byte XOR swizzle, XCD-aware tile order, LDS-transposed epilogue);
// a slab now spans 128 contraction elements, and each stage also carries the 4 scale bytes of every row.
// ------------------------------------------------------------------------------------------------
constexpr int BM = 256, BN = 256, BKB = 128, NTHR = 512;   // BKB: bytes = fp8 elements per slab row
constexpr int XB = BM * BKB, WB = BN * BKB, SB = BM * 4;   // tile bytes; scale bytes per operand tile
constexpr int STAGE = XB + WB + 2 * SB;                    // (fp8 weights; 4-bit weights need half of WB)

struct MxArgs {
    const unsigned char *X, *XS;     // codes [M,K], scales [M,K/32]
    const unsigned char *W, *WS;     // codes [N,K], scales [N,K/32]   (N = nseg * seg_n)
    const bf16 *bias;                // [N] or null
    int M, N, K;
    int nseg, seg_n;
    // low-rank branch kept in bf16, per segment (null zs = segment not adapted): out += zs . tmat^T
    const bf16 *zs[3];               // [M,K2]: scaled rank-space activations, zero beyond the rank(s)
    const bf16 *tmat[3];             // [seg_n,ldt]: up-projection(s), ldt = K2 rounded up to 32, zero padded
    int K2, ldt;
    // epilogue (meaning as in GemmArgs)
    void *out0; void *out1; const void *aux; int ldo;
    const bf16 *dl_o, *dl_lo; float *dl_out;   // EPI_STORE_DELTA (meaning as in GemmArgs)
    unsigned char *oq, *os;          // optional MXFP8 copy of the epilogue's bf16 tensor (see GemmArgs)
    static constexpr bool kEmitCodes = true;
};
// With W4 the weight operand is MXFP4: W holds two E2M1 codes per byte ([N, K/2]), a tile row is 64 bytes
// per slab, the lane's 32 elements are 16 consecutive bytes (k = 32g .. 32g+31) and the upper half of the
// operand register is unused.

__device__ __forceinline__ void glds16(const void *sbase, unsigned voff, unsigned lds)
{
    // M0 carries the LDS address; one wait state is required between its write and the copy
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds), "v"(voff), "s"(sbase) : "memory");
}
__device__ __forceinline__ void glds4(const void *sbase, unsigned voff, unsigned lds)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(lds), "v"(voff), "s"(sbase) : "memory");
}
__device__ __forceinline__ unsigned lds_addr(const void *p)
{
    return (unsigned)(unsigned long long)(const __attribute__((address_space(3))) char *)p;
}
#define MX_WAIT_VM0() __builtin_amdgcn_s_waitcnt(0x0F70)

template <bool W4, int EPI>
__global__ __launch_bounds__(NTHR) void gemm_mx_kernel(MxArgs a)
{
    constexpr int WROW = W4 ? 64 : 128;                  // bytes of one tile row of W per slab
    constexpr int WBt = BN * WROW, STAGEt = XB + WBt + 2 * SB;
    __shared__ __attribute__((aligned(1024))) unsigned char st0[STAGEt];
    __shared__ __attribute__((aligned(1024))) unsigned char st1[STAGEt];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int r16 = lane & 15, kg = lane >> 4;

    // consecutive logical tiles go to the same XCD; inside an XCD's range panels of 4 row tiles
    const int tiles_n_seg = (a.seg_n + BN - 1) / BN;
    const int tiles_n = tiles_n_seg * a.nseg, tiles_m = (a.M + BM - 1) / BM;
    const int nb = tiles_m * tiles_n;
    const int per_xcd = (nb + 7) >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= nb) return;
    constexpr int PANEL = 4;
    const int pidx = logical / (PANEL * tiles_n), prem = logical - pidx * (PANEL * tiles_n);
    const int prow = min(PANEL, tiles_m - pidx * PANEL);
    const int tn = prem / prow, tm = pidx * PANEL + prem - tn * prow;
    const int seg = tn / tiles_n_seg, tns = tn - seg * tiles_n_seg;
    const int m0 = tm * BM, n0 = seg * a.seg_n + tns * BN, n_end = (seg + 1) * a.seg_n;

    // ---- copies: per stage every wave moves 32 rows of each tile (8 rows = 1 KB per instruction, lane l
    //      -> row l>>3, physical 16-byte chunk l&7 holding logical chunk (l&7)^(l>>3)) and 64 rows' scale
    //      dwords of one operand (waves 0-3: X, waves 4-7: W)
    const int lrow = lane >> 3, lch = (lane & 7) ^ (lane >> 3);
    // per-lane byte offsets are formed at each copy (two VALU operations) instead of being held in eight
    // registers through the loop: the accumulators and fragments leave none to spare, and a spilled
    // offset would put a scratch reload, and with it a wait for every copy in flight, between the copies
    const int xrow0 = m0 + wave * 32 + lrow, wrow0 = n0 + wave * 32 + lrow;
    const unsigned lch16 = lch * 16;
    const int kb4 = a.K >> 5;                            // scale bytes per row
    const bool sx = wave < 4;
    const int srow = sx ? min(m0 + wave * 64 + lane, a.M - 1) : min(n0 + (wave - 4) * 64 + lane, n_end - 1);
    const unsigned so = (unsigned)srow * (unsigned)kb4;
    const unsigned char *Sb = sx ? a.XS : a.WS;
    const int s_lds = XB + WBt + (sx ? 0 : SB) + (wave & 3) * 256;
    // 4-bit weights: a copy instruction moves 16 rows of 64 bytes; lane l -> row l>>2, physical chunk l&3
    // holding logical chunk (l&3) ^ ((row>>1)&3), which keeps the 16-byte operand reads conflict-free
    const int w4row0 = n0 + wave * 32 + (lane >> 2);
    const unsigned w4ch16 = (unsigned)(((lane & 3) ^ ((lane >> 3) & 3)) * 16);
    const int wofs = wave * 32 * BKB;

    f32x4 acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.0f;
    // Keep the accumulators in the accumulation half of the register file (an "a" operand anywhere in
    // the kernel selects that MFMA form).  With everything in one file the 8-register fp8 fragments leave
    // so little room that the compiler rotates the accumulators through registers the fragments free up
    // and copies all 128 back at the end of every pass through the loop: 1.57 -> 1.75 PFLOP/s.
    {
        float agpr_hint = 0.0f;
        asm volatile("" : "+a"(agpr_hint));
    }

    const int a_row = (wm * 128 + r16) * BKB, b_row = (wn * 64 + r16) * WROW;
    const int sw = r16 & 7;
    const int c0 = ((kg ^ sw) << 4), c1 = (((4 + kg) ^ sw) << 4);      // the lane's two 16-byte chunks
    const int c4 = ((kg ^ ((r16 >> 1) & 3)) << 4);                      // its one chunk of a 4-bit row
    const int as_off = XB + WBt + (wm * 128 + r16) * 4 + kg, bs_off = XB + WBt + SB + (wn * 64 + r16) * 4 + kg;

#define MX_ISSUE(st, kt, p)                                                               \
    {                                                                                     \
        int xr_ = xrow0, wr_ = wrow0;                                                     \
        asm volatile("" : "+v"(xr_), "+v"(wr_));                                          \
        const unsigned xo_ = (unsigned)min(xr_ + (p) * 8, a.M - 1) * (unsigned)a.K + lch16; \
        glds16(a.X + (size_t)(kt) * BKB, xo_, lds_addr(st) + wofs + (p) * 1024);          \
        if (!W4) {                                                                        \
            const unsigned wo_ = (unsigned)min(wr_ + (p) * 8, n_end - 1) * (unsigned)a.K + lch16; \
            glds16(a.W + (size_t)(kt) * BKB, wo_, lds_addr(st) + XB + wofs + (p) * 1024); \
        } else if ((p) < 2) {                                                             \
            int w4_ = w4row0;                                                             \
            asm volatile("" : "+v"(w4_));                                                 \
            const unsigned wo_ = (unsigned)min(w4_ + (p) * 16, n_end - 1) * (unsigned)(a.K >> 1) + w4ch16; \
            glds16(a.W + (size_t)(kt) * 64, wo_, lds_addr(st) + XB + wave * 2048 + (p) * 1024); \
        }                                                                                 \
        if ((p) == 0) glds4(Sb + (size_t)(kt) * 4, so, lds_addr(st) + s_lds);             \
    }
#define MX_FRAG(dst, base, off)                                                           \
    {                                                                                     \
        (dst).lo = *(const i32x4 *)((base) + (off) + c0);                                 \
        (dst).hi = *(const i32x4 *)((base) + (off) + c1);                                 \
    }
    // one slab: the W fragments and scales once, the X fragments two row tiles at a time (the accumulators
    // take half of the register file, so only a quarter of the X operand is held at once)
#define MX_STEP(st)                                                                       \
    {                                                                                     \
        const unsigned char *S_ = (st);                                                   \
        i32x8 bfr[4];                                                                     \
        int bsc[4];                                                                       \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                   \
            if (W4) {                                                                     \
                bfr[j].lo = *(const i32x4 *)(S_ + XB + b_row + j * 16 * WROW + c4);       \
                bfr[j].hi = (i32x4){0, 0, 0, 0};                                          \
            } else {                                                                      \
                MX_FRAG(bfr[j], S_ + XB, b_row + j * 16 * WROW)                           \
            }                                                                             \
            bsc[j] = S_[bs_off + j * 64];                                                 \
        }                                                                                 \
        _Pragma("unroll") for (int iq = 0; iq < 4; ++iq) {                                \
            i32x8 af[2];                                                                  \
            int asc[2];                                                                   \
            _Pragma("unroll") for (int i = 0; i < 2; ++i) {                               \
                MX_FRAG(af[i], S_, a_row + (iq * 2 + i) * 16 * BKB)                       \
                asc[i] = S_[as_off + (iq * 2 + i) * 64];                                  \
            }                                                                             \
            _Pragma("unroll") for (int i = 0; i < 2; ++i)                                 \
                _Pragma("unroll") for (int j = 0; j < 4; ++j)                             \
                    acc[iq * 2 + i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4( \
                        af[i], bfr[j], acc[iq * 2 + i][j], 0, W4 ? 4 : 0, 0, asc[i], 0, bsc[j]); \
        }                                                                                 \
    }
#define MX_PHASE(cur, nxt, kt, doload)                                                    \
    {                                                                                     \
        if (doload) { MX_ISSUE(nxt, kt, 0) MX_ISSUE(nxt, kt, 1) MX_ISSUE(nxt, kt, 2) MX_ISSUE(nxt, kt, 3) } \
        MX_STEP(cur)                                                                      \
    }

    const int nk = a.K / BKB;
    MX_ISSUE(st0, 0, 0) MX_ISSUE(st0, 0, 1) MX_ISSUE(st0, 0, 2) MX_ISSUE(st0, 0, 3)
    MX_WAIT_VM0();
    __syncthreads();
    int kt = 0;
    for (; kt + 2 <= nk; kt += 2) {
        MX_PHASE(st0, st1, kt + 1, true)
        MX_WAIT_VM0();
        __syncthreads();
        const bool more = kt + 2 < nk;
        MX_PHASE(st1, st0, kt + 2, more)
        MX_WAIT_VM0();
        __syncthreads();
    }
    if (kt < nk) {
        MX_PHASE(st0, st1, 0, false)
        __syncthreads();
    }
#undef MX_ISSUE
#undef MX_FRAG
#undef MX_STEP
#undef MX_PHASE

    // ---- low-rank tail (SplitLoRA Sec. II-C: W + BA with the adapter kept in bf16): ldt / 32 bf16 MFMA
    //      k-steps per tile on operands read straight from global memory (a few MB: cache hits); columns
    //      of the rank-space activations beyond K2 and of the up-projection beyond the ranks are zero
    if (a.zs[seg] != nullptr) {
        const bf16 *zs_ = a.zs[seg], *tm_ = a.tmat[seg];
        for (int ks = 0; ks < (a.ldt >> 5); ++ks) {
            bf16x8 tb[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = min(n0 + wn * 64 + j * 16 + r16, n_end - 1) - seg * a.seg_n;
                tb[j] = *(const bf16x8 *)(tm_ + (size_t)n * a.ldt + ks * 32 + kg * 8);
            }
            const bool zok = ks * 32 + kg * 8 < a.K2;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = min(m0 + wm * 128 + i * 16 + r16, a.M - 1);
                bf16x8 za;
#pragma unroll
                for (int q = 0; q < 8; ++q) za[q] = f2bf(0.f);
                if (zok) za = *(const bf16x8 *)(zs_ + (size_t)row * a.K2 + ks * 32 + kg * 8);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(za, tb[j], acc[i][j], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: each wave transposes its tiles through a private LDS strip (32 rows x 64 columns
    //      fp32) so that global memory sees 16-byte accesses; only the owning wave touches its strip.
    //      The operands that come from global memory are fetched one strip ahead.
    constexpr int EP = 68;
    float *stg = (float *)((wave < 4 ? st0 : st1) + (wave & 3) * (32 * EP * 4));
    const int er = lane >> 3, ec = (lane & 7) * 8;
    const int gcol = n0 + wn * 64 + ec;
    float bias8[8];
    {
        bf16x8 b8;
#pragma unroll
        for (int i = 0; i < 8; ++i) b8[i] = f2bf(0.f);
        if (a.bias && gcol < n_end) b8 = *(const bf16x8 *)(a.bias + gcol);
#pragma unroll
        for (int i = 0; i < 8; ++i) bias8[i] = bf2f(b8[i]);
    }
    AuxRow aux[2][4];
    const int row_base = m0 + wm * 128 + er;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int row = row_base + it * 8;
        load_aux<EPI>(a, row, gcol, row < a.M && gcol < n_end, aux[0][it]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i + 1 < 4) {
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int row = row_base + (i + 1) * 32 + it * 8;
                load_aux<EPI>(a, row, gcol, row < a.M && gcol < n_end, aux[(i + 1) & 1][it]);
            }
        }
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    stg[(h * 16 + 4 * kg + e) * EP + j * 16 + r16] = acc[2 * i + h][j][e];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int rl = it * 8 + er;
            const float4 p0 = *(const float4 *)(stg + rl * EP + ec);
            const float4 p1 = *(const float4 *)(stg + rl * EP + ec + 4);
            float v[8] = {p0.x + bias8[0], p0.y + bias8[1], p0.z + bias8[2], p0.w + bias8[3],
                          p1.x + bias8[4], p1.y + bias8[5], p1.z + bias8[6], p1.w + bias8[7]};
            const int row = m0 + wm * 128 + i * 32 + rl;
            if (row < a.M && gcol < n_end) store_row8<EPI>(a, row, gcol, v, aux[i & 1][it]);
        }
    }
}

// Rank-space activations of the bf16 adapter branch: out[M, 16 NT] = scale * X[M,K] . Z[16 NT, K]^T (rows of
// Z beyond the ranks are zero), rounded to bf16.  One wave per 16 rows, operands straight from global memory
// (the kernel reads X once: HBM-bound), two k-steps in flight per column tile.
template <int NT>
__global__ __launch_bounds__(256) void rank_project_kernel(const bf16 *__restrict__ X, long long ldx, int M, int K,
                                                           const bf16 *__restrict__ Z, long long ldz, float scale,
                                                           bf16 *__restrict__ out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r16 = lane & 15, kg = lane >> 4;
    const int row0 = (blockIdx.x * 4 + wave) * 16;
    if (row0 >= M) return;
    const bf16 *xp = X + (size_t)min(row0 + r16, M - 1) * ldx + kg * 8;
    const bf16 *zp = Z + (size_t)r16 * ldz + kg * 8;
    f32x4 acc[NT][2];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[t][u][e] = 0.f;
    int k0 = 0;
    for (; k0 + 64 <= K; k0 += 64) {
        bf16x8 xa[2], zb[NT][2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            xa[u] = *(const bf16x8 *)(xp + k0 + u * 32);
#pragma unroll
            for (int t = 0; t < NT; ++t) zb[t][u] = *(const bf16x8 *)(zp + (size_t)t * 16 * ldz + k0 + u * 32);
        }
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int u = 0; u < 2; ++u)
                acc[t][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[u], zb[t][u], acc[t][u], 0, 0, 0);
    }
    for (; k0 < K; k0 += 32) {
        const bf16x8 xa = *(const bf16x8 *)(xp + k0);
#pragma unroll
        for (int t = 0; t < NT; ++t)
            acc[t][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, *(const bf16x8 *)(zp + (size_t)t * 16 * ldz + k0),
                                                                acc[t][0], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int row = row0 + 4 * kg + e;
            if (row < M) out[(size_t)row * (16 * NT) + t * 16 + r16] = f2bf((acc[t][0][e] + acc[t][1][e]) * scale);
        }
}

bool aligned(const void *p, uintptr_t n) { return (((uintptr_t)p) & (n - 1)) == 0; }
inline size_t al256(size_t v) { return (v + 255) & ~(size_t)255; }

int launch_quantize(const bf16 *x, long long ldx, long long M, int K, unsigned char *codes, unsigned char *scales,
                    hipStream_t st)
{
    hipLaunchKernelGGL(mx_quantize_kernel, dim3((unsigned)M, (unsigned)((K / 8 + 127) / 128)), dim3(128), 0, st, x, ldx,
                       M, K, codes, scales);
    SL_CHECK_LAUNCH("mx_quantize");
    return 0;
}

int launch_gemm_mx(const MxArgs &a, hipStream_t st, bool w4 = false, int epi = EPI_STORE)
{
    const int nb = ((a.M + BM - 1) / BM) * (((a.seg_n + BN - 1) / BN) * a.nseg);
    const dim3 grid(((nb + 7) / 8) * 8), block(NTHR);
    if (w4) {
        if (epi != EPI_STORE) return SL_EINVAL;
        hipLaunchKernelGGL((gemm_mx_kernel<true, EPI_STORE>), grid, block, 0, st, a);
    } else {
        switch (epi) {
        case EPI_STORE: hipLaunchKernelGGL((gemm_mx_kernel<false, EPI_STORE>), grid, block, 0, st, a); break;
        case EPI_RESID: hipLaunchKernelGGL((gemm_mx_kernel<false, EPI_RESID>), grid, block, 0, st, a); break;
        case EPI_GELU: hipLaunchKernelGGL((gemm_mx_kernel<false, EPI_GELU>), grid, block, 0, st, a); break;
        case EPI_DGELU: hipLaunchKernelGGL((gemm_mx_kernel<false, EPI_DGELU>), grid, block, 0, st, a); break;
        case EPI_STORE_DELTA:
            if (!a.dl_o || !a.dl_lo || !a.dl_out || !a.out0 || (a.N % 64) || a.nseg != 1) return SL_EINVAL;
            hipLaunchKernelGGL((gemm_mx_kernel<false, EPI_STORE_DELTA>), grid, block, 0, st, a);
            break;
        default: return SL_EINVAL;
        }
    }
    SL_CHECK_LAUNCH("gemm_mx");
    return 0;
}

// a plain product: one segment, no adapter branch, bf16 output [M,N]
MxArgs mx_plain(const void *xq, const void *xs, const void *wq, const void *ws, const void *bias, void *y, int M,
                int N, int K)
{
    MxArgs a;
    a.X = (const unsigned char *)xq; a.XS = (const unsigned char *)xs;
    a.W = (const unsigned char *)wq; a.WS = (const unsigned char *)ws;
    a.bias = (const bf16 *)bias;
    a.M = M; a.N = N; a.K = K;
    a.nseg = 1; a.seg_n = N;
    for (int i = 0; i < 3; ++i) { a.zs[i] = nullptr; a.tmat[i] = nullptr; }
    a.K2 = 16; a.ldt = 32;
    a.out0 = y; a.out1 = nullptr; a.aux = nullptr; a.ldo = N;
    a.dl_o = nullptr; a.dl_lo = nullptr; a.dl_out = nullptr;
    a.oq = nullptr; a.os = nullptr;
    return a;
}

int launch_rank_project(const bf16 *X, long long ldx, int M, int K, const bf16 *Z, long long ldz, int nz, float scale,
                        bf16 *out, hipStream_t st)
{
    const dim3 grid((M + 63) / 64), block(256);
    switch (nz) {
    case 16: hipLaunchKernelGGL((rank_project_kernel<1>), grid, block, 0, st, X, ldx, M, K, Z, ldz, scale, out); break;
    case 32: hipLaunchKernelGGL((rank_project_kernel<2>), grid, block, 0, st, X, ldx, M, K, Z, ldz, scale, out); break;
    case 48: hipLaunchKernelGGL((rank_project_kernel<3>), grid, block, 0, st, X, ldx, M, K, Z, ldz, scale, out); break;
    default: return SL_EINVAL;
    }
    SL_CHECK_LAUNCH("rank_project");
    return 0;
}

// packed frozen weight: codes and scales of W [n_out, n_in] (blocks along n_in, for the forward product)
// and of W^T [n_in, n_out] (blocks along n_out, for the input-gradient product), then packing scratch
struct MxPack { size_t wq, ws, tq, ts, scratch, total; };
MxPack mx_pack(int n_in, int n_out)
{
    MxPack p;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = al256(off + bytes); return o; };
    p.wq = take((size_t)n_out * n_in);
    p.ws = take((size_t)n_out * n_in / 32);
    p.tq = take((size_t)n_in * n_out);
    p.ts = take((size_t)n_in * n_out / 32);
    p.scratch = take(2 * (size_t)n_in * n_out);
    p.total = off;
    return p;
}

struct MxLinWs { size_t A16, B32, B16T, A32T, zs, ps, q, qs, part, total; };
MxLinWs mx_lin_ws(int T, int n_in, int n_out)
{
    MxLinWs w;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = al256(off + bytes); return o; };
    const size_t nmax = n_in > n_out ? n_in : n_out;
    w.A16 = take(2 * 16 * (size_t)n_in);
    w.B32 = take(2 * (size_t)n_out * 32);
    w.B16T = take(2 * 16 * (size_t)n_out);
    w.A32T = take(2 * (size_t)n_in * 32);
    w.zs = take(2 * (size_t)T * 16);
    w.ps = take(2 * (size_t)T * 16);
    w.q = take((size_t)T * nmax);
    w.qs = take((size_t)T * nmax / 32);
    w.part = take(4 * lora_grad_partial_floats(T, (int)nmax));
    w.total = off;
    return w;
}

bool mx_lin_args_ok(int T, int n_in, int n_out, int r)
{
    if (T <= 0 || n_in <= 0 || n_out <= 0 || r < 1 || r > SLORA_MAX_RANK) return false;
    if ((n_in % 128) || (n_out % 128)) return false;
    const unsigned long long nmax = n_in > n_out ? n_in : n_out;
    return (unsigned long long)T * nmax < (1ull << 31) && (unsigned long long)n_in * n_out < (1ull << 31);
}

}  // namespace

int launch_mx_quantize(const bf16 *x, long long ldx, long long M, int K, unsigned char *codes, unsigned char *scales,
                       hipStream_t st)
{
    if (M <= 0 || K <= 0 || (K % 32) || ldx < K) return SL_EINVAL;
    return launch_quantize(x, ldx, M, K, codes, scales, st);
}

int launch_gemm_mx_stack(const GemmArgs &g, int epi, int nz, hipStream_t st)
{
    const MxOperands &m = *g.mx;
    if ((g.K % 128) || (g.seg_n % 8) || g.ldw != g.K || !m.wq || !m.ws || !m.xq || !m.xs) return SL_EINVAL;
    if ((unsigned long long)g.M * g.K >= (1ull << 32) || (unsigned long long)g.N * g.K >= (1ull << 32)) return SL_EINVAL;
    int rc;
    if (!m.x_ready && !g.X) return SL_EINVAL;
    if (!m.x_ready && (rc = launch_quantize(g.X, g.ldx, g.M, g.K, m.xq, m.xs, st))) return rc;
    MxArgs a = mx_plain(m.xq, m.xs, m.wq, m.ws, g.bias, g.out0, g.M, g.N, g.K);
    a.nseg = g.nseg; a.seg_n = g.seg_n;
    a.out1 = g.out1; a.aux = g.aux; a.ldo = g.ldo;
    if (epi == EPI_STORE_DELTA) {
        if (nz != 0) return SL_EINVAL;
        a.dl_o = g.dl_o; a.dl_lo = g.dl_lo; a.dl_out = g.dl_out;
    }
    if (g.oq) {
        if (!g.os || (g.ldo % 32) || (g.seg_n % 32) || (epi != EPI_GELU && epi != EPI_DGELU)) return SL_EINVAL;
        a.oq = g.oq; a.os = g.os;
    }
    // the bf16 copy of the tensor that also goes out as codes may be left out; everything else must exist
    if (!(epi == EPI_GELU ? g.out0 && (g.out1 || g.oq) : epi == EPI_DGELU ? (g.out0 || g.oq) : g.out0 || g.out1))
        return SL_EINVAL;
    if (nz > 0) {
        a.K2 = g.K2; a.ldt = g.ldt;
        for (int sgm = 0; sgm < g.nseg; ++sgm) {
            if (!g.zmat[sgm]) continue;
            // the bf16 kernel forms these inside its K loop from the bf16 tile; here the tile is fp8
            if (!g.zspill[sgm] || !g.tmat[sgm] || !g.X) return SL_EINVAL;
            if ((rc = launch_rank_project(g.X, g.ldx, g.M, g.K, g.zmat[sgm], g.ldz, nz, g.zscale, g.zspill[sgm], st)))
                return rc;
            a.zs[sgm] = g.zspill[sgm];
            a.tmat[sgm] = g.tmat[sgm];
        }
    }
    return launch_gemm_mx(a, st, false, epi);
}

int slora_mx_quantize(int64_t M, int32_t K, const void *x, int64_t ldx, void *codes, void *scales, void *stream)
{
    if (M <= 0 || K <= 0 || (K % 32) || ldx < K || (ldx % 8) || !x || !codes || !scales) return SLORA_EINVAL;
    if (!aligned(x, 16) || !aligned(codes, 8)) return SLORA_EINVAL;
    if (M >= (1ll << 31) || K / 8 > 128 * 65535) return SLORA_EINVAL;
    return launch_quantize((const bf16 *)x, ldx, M, K, (unsigned char *)codes, (unsigned char *)scales,
                           (hipStream_t)stream);
}

int slora_mx_dequantize(int64_t M, int32_t K, const void *codes, const void *scales, void *y, int64_t ldy,
                        void *stream)
{
    if (M <= 0 || K <= 0 || (K % 32) || ldy < K || (ldy % 8) || !y || !codes || !scales) return SLORA_EINVAL;
    if (!aligned(y, 16) || !aligned(codes, 8)) return SLORA_EINVAL;
    const long long threads = (long long)M * (K / 8);
    if (threads > (1ll << 31) * 256ll) return SLORA_EINVAL;
    const unsigned grid = (unsigned)((threads + 255) / 256);
    hipLaunchKernelGGL(mx_dequantize_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream,
                       (const unsigned char *)codes, (const unsigned char *)scales, (long long)M, (int)K, (bf16 *)y,
                       (long long)ldy);
    SL_CHECK_LAUNCH("mx_dequantize");
    return SLORA_OK;
}

int slora_frozen_linear_mxfp8(int32_t T, int32_t n_in, int32_t n_out, const void *xq, const void *xs, const void *wq,
                              const void *ws, const void *bias, void *y, void *stream)
{
    if (T <= 0 || n_in <= 0 || n_out <= 0 || (n_in % 128) || (n_out % 8) || !xq || !xs || !wq || !ws || !y)
        return SLORA_EINVAL;
    if (!aligned(xq, 16) || !aligned(wq, 16) || !aligned(xs, 4) || !aligned(ws, 4) || !aligned(y, 16) ||
        (bias && !aligned(bias, 16)))
        return SLORA_EINVAL;
    // the copies address both operands with 32-bit byte offsets from their bases
    if ((unsigned long long)T * n_in >= (1ull << 32) || (unsigned long long)n_out * n_in >= (1ull << 32))
        return SLORA_EINVAL;
    return launch_gemm_mx(mx_plain(xq, xs, wq, ws, bias, y, T, n_out, n_in), (hipStream_t)stream);
}

int slora_mx_quantize_fp4(int64_t M, int32_t K, const void *x, int64_t ldx, void *codes, void *scales, void *stream)
{
    if (M <= 0 || K <= 0 || (K % 32) || ldx < K || (ldx % 8) || !x || !codes || !scales) return SLORA_EINVAL;
    if (!aligned(x, 16) || !aligned(codes, 4)) return SLORA_EINVAL;
    if (M >= (1ll << 31) || K / 8 > 128 * 65535) return SLORA_EINVAL;
    hipLaunchKernelGGL(mx_quantize_fp4_kernel, dim3((unsigned)M, (unsigned)((K / 8 + 127) / 128)), dim3(128), 0,
                       (hipStream_t)stream, (const bf16 *)x, (long long)ldx, (long long)M, (int)K,
                       (unsigned char *)codes, (unsigned char *)scales);
    SL_CHECK_LAUNCH("mx_quantize_fp4");
    return SLORA_OK;
}

int slora_frozen_linear_mxfp8_w4(int32_t T, int32_t n_in, int32_t n_out, const void *xq, const void *xs,
                                 const void *wq4, const void *ws, const void *bias, void *y, void *stream)
{
    if (T <= 0 || n_in <= 0 || n_out <= 0 || (n_in % 128) || (n_out % 8) || !xq || !xs || !wq4 || !ws || !y)
        return SLORA_EINVAL;
    if (!aligned(xq, 16) || !aligned(wq4, 16) || !aligned(xs, 4) || !aligned(ws, 4) || !aligned(y, 16) ||
        (bias && !aligned(bias, 16)))
        return SLORA_EINVAL;
    if ((unsigned long long)T * n_in >= (1ull << 32) || (unsigned long long)n_out * n_in >= (1ull << 32))
        return SLORA_EINVAL;
    return launch_gemm_mx(mx_plain(xq, xs, wq4, ws, bias, y, T, n_out, n_in), (hipStream_t)stream, true);
}

size_t slora_mx_weight_bytes(int32_t n_in, int32_t n_out)
{
    if (n_in <= 0 || n_out <= 0 || (n_in % 128) || (n_out % 128)) return 0;
    return mx_pack(n_in, n_out).total;
}

int slora_mx_pack_weight(int32_t n_in, int32_t n_out, const void *W, void *packed, size_t bytes, void *stream)
{
    if (n_in <= 0 || n_out <= 0 || (n_in % 128) || (n_out % 128) || !W || !packed) return SLORA_EINVAL;
    if (!aligned(W, 16) || !aligned(packed, 256)) return SLORA_EINVAL;
    const MxPack p = mx_pack(n_in, n_out);
    if (bytes < p.total) return SLORA_ENOSPC;
    hipStream_t st = (hipStream_t)stream;
    unsigned char *base = (unsigned char *)packed;
    int rc;
    if ((rc = launch_quantize((const bf16 *)W, n_in, n_out, n_in, base + p.wq, base + p.ws, st))) return rc;
    bf16 *wt = (bf16 *)(base + p.scratch);
    if ((rc = launch_transpose_bf16((const bf16 *)W, n_out, n_in, wt, st))) return rc;
    return launch_quantize(wt, n_out, n_in, n_out, base + p.tq, base + p.ts, st);
}

size_t slora_mx_lora_linear_ws_bytes(int32_t T, int32_t n_in, int32_t n_out, int32_t r)
{
    if (!mx_lin_args_ok(T, n_in, n_out, r)) return 0;
    return mx_lin_ws(T, n_in, n_out).total;
}

int slora_mx_lora_linear_fwd(int32_t T, int32_t n_in, int32_t n_out, int32_t r, float alpha, const void *x,
                             const void *packed_w, const void *bias, const float *A, const float *B, void *y,
                             void *ws, size_t ws_bytes, void *stream)
{
    if (!mx_lin_args_ok(T, n_in, n_out, r) || !x || !packed_w || !A || !B || !y || !ws) return SLORA_EINVAL;
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(packed_w, 256) || !aligned(ws, 256) ||
        (bias && !aligned(bias, 16)))
        return SLORA_EINVAL;
    const MxLinWs w = mx_lin_ws(T, n_in, n_out);
    if (ws_bytes < w.total) return SLORA_ENOSPC;
    const MxPack p = mx_pack(n_in, n_out);
    hipStream_t st = (hipStream_t)stream;
    unsigned char *base = (unsigned char *)ws;
    const unsigned char *pw = (const unsigned char *)packed_w;
    const float s = alpha / (float)r;
    int rc;
    if ((rc = launch_cast_pad(A, r, n_in, (bf16 *)(base + w.A16), 16, n_in, 0, st))) return rc;
    if ((rc = launch_cast_pad(B, n_out, r, (bf16 *)(base + w.B32), n_out, 32, 0, st))) return rc;
    if ((rc = launch_rank_project((const bf16 *)x, n_in, T, n_in, (const bf16 *)(base + w.A16), n_in, 16, s,
                                  (bf16 *)(base + w.zs), st)))
        return rc;
    if ((rc = launch_quantize((const bf16 *)x, n_in, T, n_in, base + w.q, base + w.qs, st))) return rc;
    MxArgs a = mx_plain(base + w.q, base + w.qs, pw + p.wq, pw + p.ws, bias, y, T, n_out, n_in);
    a.zs[0] = (const bf16 *)(base + w.zs); a.tmat[0] = (const bf16 *)(base + w.B32);
    return launch_gemm_mx(a, st);
}

int slora_mx_lora_linear_bwd(int32_t T, int32_t n_in, int32_t n_out, int32_t r, float alpha, const void *x,
                             const void *dy, const void *packed_w, const float *A, const float *B, void *dx,
                             float *dA, float *dB, void *ws, size_t ws_bytes, void *stream)
{
    if (!mx_lin_args_ok(T, n_in, n_out, r) || !x || !dy || !packed_w || !A || !B || !dx || !dA || !dB || !ws)
        return SLORA_EINVAL;
    if (!aligned(x, 16) || !aligned(dy, 16) || !aligned(dx, 16) || !aligned(packed_w, 256) || !aligned(ws, 256))
        return SLORA_EINVAL;
    const MxLinWs w = mx_lin_ws(T, n_in, n_out);
    if (ws_bytes < w.total) return SLORA_ENOSPC;
    const MxPack p = mx_pack(n_in, n_out);
    hipStream_t st = (hipStream_t)stream;
    unsigned char *base = (unsigned char *)ws;
    const unsigned char *pw = (const unsigned char *)packed_w;
    const float s = alpha / (float)r;
    int rc;
    // zs = s x A^T (for dB) and ps = s dy B (for dA and for the low-rank part of dx)
    if ((rc = launch_cast_pad(A, r, n_in, (bf16 *)(base + w.A16), 16, n_in, 0, st))) return rc;
    if ((rc = launch_rank_project((const bf16 *)x, n_in, T, n_in, (const bf16 *)(base + w.A16), n_in, 16, s,
                                  (bf16 *)(base + w.zs), st)))
        return rc;
    if ((rc = launch_cast_pad(B, n_out, r, (bf16 *)(base + w.B16T), 16, n_out, 1, st))) return rc;
    if ((rc = launch_cast_pad(A, r, n_in, (bf16 *)(base + w.A32T), n_in, 32, 1, st))) return rc;
    if ((rc = launch_rank_project((const bf16 *)dy, n_out, T, n_out, (const bf16 *)(base + w.B16T), n_out, 16, s,
                                  (bf16 *)(base + w.ps), st)))
        return rc;
    if ((rc = launch_quantize((const bf16 *)dy, n_out, T, n_out, base + w.q, base + w.qs, st))) return rc;
    MxArgs a = mx_plain(base + w.q, base + w.qs, pw + p.tq, pw + p.ts, nullptr, dx, T, n_in, n_out);
    a.zs[0] = (const bf16 *)(base + w.ps); a.tmat[0] = (const bf16 *)(base + w.A32T);
    if ((rc = launch_gemm_mx(a, st))) return rc;
    float *part = (float *)(base + w.part);
    if ((rc = launch_lora_grad((const bf16 *)x, n_in, n_in, (const bf16 *)(base + w.ps), 16, r, T, part, dA, 1, st)))
        return rc;
    return launch_lora_grad((const bf16 *)dy, n_out, n_out, (const bf16 *)(base + w.zs), 16, r, T, part, dB, 0, st);
}
