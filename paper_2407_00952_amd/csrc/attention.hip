// Causal multi-head attention, forward and backward, head size 64, bf16 MFMA with fp32
// softmax arithmetic (gfx950).  Part of the server-side forward/backward of SplitLoRA
// Sec. III-B step a3; the attention block itself is the public GPT-2 one
// (softmax(Q K^T / sqrt(64)) V with future keys excluded).
//
// Layout: qkv [T, 3d] bf16 (q | k | v column blocks, head a at columns 64a..64a+63 of each),
// o / dO [T, d], lse [n_seq, H, S] fp32 in log2 units of the scaled scores, delta likewise.
//
// Forward, and the backward for sequences longer than 512 (a dQ kernel, then a dK/dV kernel): 4 wavefronts
// per block, each owning 32 rows (queries or keys), online-softmax tiles of 64 staged in LDS by asynchronous
// global->LDS copies, double buffered.  Scores are produced with the lane owning one query (forward, dQ) or
// one key (dK/dV), which makes the softmax statistics per-lane scalars and lets the probabilities feed the
// next MFMA straight from registers.  Operands that must be read along the token axis (V, K for dQ, Q and
// dO for dK/dV) come from the same row-major tiles through the LDS transpose read, so nothing is
// transposed in memory.
// Backward for sequences up to 512 (the default at the paper's sequence length): one block of 8 wavefronts
// per (sequence, head) forms dQ, dK and dV in one pass; K of the whole sequence stays in LDS, scores,
// probabilities and dP are formed once (see attn_bwd_fused_kernel).
// No kernel uses floating-point atomics, so results are bit-reproducible.
#include "common.h"
#include "prof.h"

namespace {

constexpr float kScaleLog2 = 0.125f * 1.4426950408889634f;   // log2(e) / sqrt(64)
constexpr int TILE_B = 64 * 128;                             // one 64-row x 64-column bf16 tile

typedef short v4s __attribute__((ext_vector_type(4)));

#define AT_GLDS(gp, lp)                                                                            \
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gp),         \
                                     (__attribute__((address_space(3))) void *)(lp), 16, 0, 0)
#define AT_WAIT_VM0() __builtin_amdgcn_s_waitcnt(0x0F70)

// XOR mask of a tile row for the 16-byte chunks of its 128-byte LDS row.  Eight consecutive rows get
// eight different masks (row-major fragment reads: 8 lanes = 8 rows, one logical chunk), and four
// consecutive rows get masks that differ in bits 1-2 (transpose reads: 16 lanes = 4 rows x 2 adjacent
// chunks), so both kinds of operand read are bank-conflict free.
__device__ __forceinline__ int swm(int row) { return ((row & 3) << 1) | ((row >> 2) & 1); }
__device__ __forceinline__ int swz128(int row, int chunk) { return row * 128 + ((chunk ^ swm(row)) << 4); }

__device__ __forceinline__ f32x16 zero16()
{
    f32x16 z;
#pragma unroll
    for (int e = 0; e < 16; ++e) z[e] = 0.f;
    return z;
}

// Asynchronous copy of a 64 x 64 bf16 tile (global pitch ld) into a swizzled row-major LDS tile.
// Four waves, two 1 KB pieces (8 rows) each: lane l fills slot l = (row l>>3, physical chunk l&7).
__device__ __forceinline__ void tile_copy_async(unsigned char *dst, const bf16 *src, int ld, int wave, int lane)
{
    const int lrow = lane >> 3, lch = (lane & 7) ^ swm(lane >> 3);
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int r0 = (wave * 2 + p) * 8;
        AT_GLDS(src + (size_t)(r0 + lrow) * ld + lch * 8, dst + r0 * 128);
    }
}

// MFMA operand fragment from a row-major tile: row (base + lane%32), k-step ks (16 columns)
__device__ __forceinline__ bf16x8 frag_rm(const unsigned char *t, int row, int ks, int g)
{
    return *(const bf16x8 *)(t + swz128(row, ks * 2 + g));
}

// MFMA operand fragment along the ROW axis of a row-major tile (the transposed operand): lane
// (m = lane%32, g = lane/32) receives column col0 + m at the 8 rows tok0 + 8h + 4g + e
// (h = 0,1; e = 0..3), element index 4h + e.  Uses the LDS transpose read: inside each group of
// 16 lanes, lane i receives element i%4 of the 8-byte pieces addressed by lanes i/4 + 4e.
__device__ __forceinline__ bf16x8 frag_tr(const unsigned char *t, int col0, int tok0, int lane)
{
    const int q = lane & 3, e = (lane >> 2) & 3, half = (lane >> 4) & 1, g = lane >> 5;
    const int col = col0 + 16 * half + 4 * q;
    const int row0 = tok0 + 4 * g + e, row1 = row0 + 8;
    const unsigned char *a0 = t + row0 * 128 + (((col >> 3) ^ swm(row0)) << 4) + (col & 7) * 2;
    const unsigned char *a1 = t + row1 * 128 + (((col >> 3) ^ swm(row1)) << 4) + (col & 7) * 2;
    union { v4s s[2]; bf16x8 v; } u;
    u.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s *)a0);
    u.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s *)a1);
    return u.v;
}

// ------------------------------------------------------------------------------------------
constexpr int OST_PITCH = 144;                                // bytes per staged output row (128 + pad: see fwd_store)
constexpr int OST_B = 32 * OST_PITCH;

__global__ __launch_bounds__(256, 3) void attn_fwd_kernel(const bf16 *__restrict__ qkv, bf16 *__restrict__ o,
                                                       bf16 *__restrict__ o_lo, float *__restrict__ lse, int S,
                                                       int H, int n_seq)
{
    __shared__ __attribute__((aligned(1024))) unsigned char K0[TILE_B], V0[TILE_B], K1[TILE_B], V1[TILE_B];
    __shared__ __attribute__((aligned(16))) unsigned char Ost[4 * OST_B];
    // Block -> (two query tiles, head, sequence).  Workgroups go to the 8 XCDs round-robin and, inside an XCD,
    // to its compute units in a fixed rotation as well: with one 128-query tile per block and tiles ordered
    // inside a (sequence, head) pair, every compute unit kept receiving tiles of the SAME length (the rotation's
    // period is a multiple of the tiles per pair), a 4:1 load imbalance at S = 512 that left two thirds of the
    // block slots empty for most of the launch.  So a block takes query tiles j and nqt-1-j of its pair, the
    // long one first: all blocks then do the same number of key tiles (nqt + 1 halves of a tile), whatever the
    // rotation.  The blocks of one pair still get ids that land on ONE XCD, next to each other in dispatch
    // order, so its L2 serves their re-reads of K and V.
    const int nqt = (S + 127) >> 7, npb = (nqt + 1) >> 1;
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int pair = (idx / npb) * 8 + xcd;             // (sequence, head) pair
    if (pair >= H * n_seq) return;
    const int qtA = nqt - 1 - idx % npb, qtB = idx % npb;                 // qtA >= qtB
    const int ntA = min(S, qtA * 128 + 128) >> 6;                       // key tiles of 64 per query tile
    const int ntB = qtA != qtB ? (qtB * 128 + 128) >> 6 : 0;
    const int nt = ntA + ntB;
    const int a = pair % H, n = pair / H;
    const int d = H * 64, ld = 3 * d;
    const int tid = threadIdx.x, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bf16 *base = qkv + (size_t)n * S * ld + a * 64;
    int qb = qtA * 128 + wave * 32;
    bool active = qb < S;
    int q = qb + r32;

    bf16x8 qf[4];
    if (active) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qf[ks] = *(const bf16x8 *)(base + (size_t)q * ld + ks * 16 + g * 8);
    }
    f32x16 oacc[2] = {zero16(), zero16()};
    // The softmax is VALU-bound at head size 64, so the per-element work is kept to one FMA, one
    // exp2 and a share of a max and of a bf16 pack:
    //  * the row sum is taken over the bf16-ROUNDED probabilities, two per instruction (bf16 dot product
    //    against (1, 1) with an fp32 addend); a lane sums the keys it holds, the two lanes of a query are
    //    added at the end.  Summing the rounded values makes O an exact convex combination of V rows, which
    //    the backward's rowsum(dO*O) relies on.  (An all-ones MFMA did the same for 16 registers and 128
    //    cycles of the matrix pipe per tile.)
    //  * the running maximum m (log2 units, scaled) is only raised when a tile exceeds it by more
    //    than 8, so most tiles skip the rescaling of the accumulators; p <= 2^8 meanwhile.
    float lsum = 0.f;
    const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};
    float m = -INFINITY;

    // Output of one query tile: O = oacc / l, its low-order bf16 term, and the log-sum-exp.  A lane holds 4
    // consecutive columns of ONE row per register group, so direct stores would touch 32 different 128-byte
    // lines per instruction with 8 bytes each; the wave's 32 x 64 outputs go through a private LDS area
    // instead (row pitch 144 bytes: rows 16 apart share banks, a 2-way conflict on the 8-byte writes) and
    // leave as whole lines, 16 bytes per lane.  LDS operations of one wave complete in issue order, so the
    // area needs no barrier, only that the compiler keeps the order.
    auto fwd_store = [&]() {
        if (!active) return;
        unsigned char *stg = Ost + wave * OST_B;
        const float lh = lsum + __shfl_xor(lsum, 32, 64);
        const float inv = 1.0f / lh;
        const int orow = lane >> 3, och = lane & 7;
        const size_t ooff = ((size_t)n * S + qb + orow) * d + a * 64 + och * 8;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {          // 0: O, 1: its low-order term
            bf16 *dst = pass ? o_lo : o;
            if (!dst) break;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    bf16x4 w;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float v = oacc[dt][4 * e4 + i] * inv;
                        const bf16 hi = f2bf(v);
                        w[i] = pass ? f2bf(v - bf2f(hi)) : hi;       // o + o_lo carries ~16 bits
                    }
                    *(bf16x4 *)(stg + r32 * OST_PITCH + (32 * dt + 8 * e4 + 4 * g) * 2) = w;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            bf16x8 rows[4];
#pragma unroll
            for (int it = 0; it < 4; ++it) rows[it] = *(const bf16x8 *)(stg + (8 * it + orow) * OST_PITCH + och * 16);
#pragma unroll
            for (int it = 0; it < 4; ++it) *(bf16x8 *)(dst + ooff + (size_t)(8 * it) * d) = rows[it];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        if (g == 0) lse[((size_t)n * H + a) * S + q] = m + log2f(lh);
    };

    // All 8 K fragments and all 16 V fragment reads of a tile are issued before the first MFMA, so the LDS
    // latency is paid once per tile instead of once per fragment (left inline in the MFMA calls the compiler
    // emitted read, wait, MFMA for every one of them), and the two score accumulators advance alternately.
#define FWD_TILE(Ks, Vs, k0)                                                                           \
    if (active && (k0) <= qb + 31) {                                                                   \
        bf16x8 kf[2][4];                                                                               \
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                               \
            _Pragma("unroll") for (int mt = 0; mt < 2; ++mt) kf[mt][ks] = frag_rm(Ks, mt * 32 + r32, ks, g); \
        __builtin_amdgcn_sched_barrier(0);                                                             \
        f32x16 sacc[2] = {zero16(), zero16()};                                                         \
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                               \
            _Pragma("unroll") for (int mt = 0; mt < 2; ++mt)                                           \
                sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mt][ks], qf[ks], sacc[mt], 0, 0, 0); \
        if ((k0) + 63 > qb) {                                                                          \
            _Pragma("unroll") for (int mt = 0; mt < 2; ++mt)                                           \
                _Pragma("unroll") for (int e = 0; e < 16; ++e) {                                       \
                    const int key = (k0) + 32 * mt + 8 * (e >> 2) + 4 * g + (e & 3);                   \
                    if (key > q) sacc[mt][e] = -INFINITY;                                              \
                }                                                                                      \
        }                                                                                              \
        float tmax = sacc[0][0];                                                                       \
        _Pragma("unroll") for (int mt = 0; mt < 2; ++mt)                                               \
            _Pragma("unroll") for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, sacc[mt][e]);            \
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64)) * kScaleLog2;                                     \
        if (__builtin_amdgcn_ballot_w64(tmax > m + 8.0f) != 0) {                                       \
            const float m_new = fmaxf(m, tmax);                                                        \
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);                                     \
            m = m_new;                                                                                 \
            lsum *= alpha;                                                                             \
            _Pragma("unroll") for (int dt = 0; dt < 2; ++dt)                                           \
                _Pragma("unroll") for (int e = 0; e < 16; ++e) oacc[dt][e] *= alpha;                   \
        }                                                                                              \
        _Pragma("unroll") for (int mt = 0; mt < 2; ++mt) {                                             \
            bf16x8 vf[2][2];                             /* this half's V fragments, under way during its exponentials */ \
            _Pragma("unroll") for (int hh = 0; hh < 2; ++hh)                                           \
                _Pragma("unroll") for (int dt = 0; dt < 2; ++dt)                                       \
                    vf[hh][dt] = frag_tr(Vs, 32 * dt, 32 * mt + 16 * hh, lane);                        \
            __builtin_amdgcn_sched_barrier(0);                                                         \
            _Pragma("unroll") for (int hh = 0; hh < 2; ++hh) {                                         \
                bf16x8 pb;                                                                             \
                float pe[8];                                                                           \
                _Pragma("unroll") for (int i = 0; i < 8; ++i) pe[i] = fmaf(sacc[mt][8 * hh + i], kScaleLog2, -m); \
                _Pragma("unroll") for (int i = 0; i < 8; ++i) pe[i] = __builtin_amdgcn_exp2f(pe[i]);   \
                _Pragma("unroll") for (int i = 0; i < 8; ++i) pb[i] = f2bf(pe[i]);                     \
                _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                        \
                    const bf16x2 pr = {pb[2 * i], pb[2 * i + 1]};                                    \
                    lsum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, lsum, false);                    \
                }                                                                                      \
                _Pragma("unroll") for (int dt = 0; dt < 2; ++dt)                                       \
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[hh][dt], pb, oacc[dt], 0, 0, 0); \
            }                                                                                          \
        }                                                                                              \
    }
    // Step t of the block's flat tile sequence (ntA tiles of the long query tile, then ntB of the short one);
    // at the switch the finished tile goes out and the wave's state is set up for the other query rows.
#define FWD_STEP(Ks, Vs, t)                                                                            \
    {                                                                                                  \
        if ((t) == ntA) {                                                                              \
            /* the short tile's Q rows have been waiting in this wave's output staging area since the   \
               first copies: fetched from memory here they would cost the block one exposed latency */  \
            bf16x8 qn[4];                                                                              \
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) qn[ks] = frag_rm(Ost + wave * OST_B, r32, ks, g); \
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   /* read before fwd_store overwrites */ \
            fwd_store();                                                                               \
            qb = qtB * 128 + wave * 32; q = qb + r32; active = true;                                   \
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) qf[ks] = qn[ks];                          \
            oacc[0] = zero16(); oacc[1] = zero16(); lsum = 0.f; m = -INFINITY;                    \
        }                                                                                              \
        const int k0_ = ((t) < ntA ? (t) : (t) - ntA) * 64;                                            \
        FWD_TILE(Ks, Vs, k0_)                                                                          \
    }
#define FWD_COPY(Kd, Vd, t)                                                                            \
    {                                                                                                  \
        const size_t off_ = (size_t)((t) < ntA ? (t) : (t) - ntA) * 64 * ld;                           \
        tile_copy_async(Kd, kg + off_, ld, wave, lane);                                                \
        tile_copy_async(Vd, vg + off_, ld, wave, lane);                                                \
    }

    const bf16 *kg = base + d, *vg = base + 2 * d;
    FWD_COPY(K0, V0, 0)
    if (ntB > 0) {                                       // this wave's 32 Q rows of the short tile -> its staging area
        const int lrow = lane >> 3, lch = (lane & 7) ^ swm(lane >> 3);
        const bf16 *qsrc = base + (size_t)(qtB * 128 + wave * 32) * ld;
#pragma unroll
        for (int p = 0; p < 4; ++p) AT_GLDS(qsrc + (size_t)(p * 8 + lrow) * ld + lch * 8, Ost + wave * OST_B + p * 1024);
    }
    AT_WAIT_VM0();
    __syncthreads();
    for (int t = 0; t < nt; t += 2) {
        if (t + 1 < nt) FWD_COPY(K1, V1, t + 1)
        FWD_STEP(K0, V0, t)
        AT_WAIT_VM0();
        __syncthreads();
        if (t + 1 >= nt) break;
        if (t + 2 < nt) FWD_COPY(K0, V0, t + 2)
        FWD_STEP(K1, V1, t + 1)
        AT_WAIT_VM0();
        __syncthreads();
    }
#undef FWD_COPY
#undef FWD_STEP
#undef FWD_TILE
    fwd_store();
}

// ------------------------------------------------------------------------------------------
// dQ (and delta = rowsum(dO * O), which the dK/dV kernel reads afterwards)
__global__ __launch_bounds__(256, 3) void attn_bwd_dq_kernel(const bf16 *__restrict__ qkv, const bf16 *__restrict__ o,
                                                          const bf16 *__restrict__ o_lo,
                                                          const bf16 *__restrict__ dout,
                                                          const float *__restrict__ lse, float *__restrict__ delta,
                                                          bf16 *__restrict__ dqkv, int S, int H, int n_seq)
{
    __shared__ __attribute__((aligned(1024))) unsigned char K0[TILE_B], V0[TILE_B], K1[TILE_B], V1[TILE_B];
    // block ids decoded as in the forward: the query tiles of a (sequence, head) share an XCD, and a block
    // takes the tiles j and nqt-1-j one after the other so that every block has the same work
    const int nqt = (S + 127) >> 7, npb = (nqt + 1) >> 1;
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int pair = (idx / npb) * 8 + xcd;
    if (pair >= H * n_seq) return;
    const int a = pair % H, n = pair / H;
    const int d = H * 64, ld = 3 * d;
    const int tid = threadIdx.x, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bf16 *base = qkv + (size_t)n * S * ld + a * 64;
#pragma clang loop unroll(disable)
    for (int ph = 0; ph < 2; ++ph) {
    const int qt = ph == 0 ? nqt - 1 - idx % npb : idx % npb;
    if (ph == 1) {
        if (qt == nqt - 1 - idx % npb) break;            // odd tile count: the middle tile stands alone
        __syncthreads();                                 // the first pass's tiles are no longer read
    }
    const int qb = qt * 128 + wave * 32;
    const bool active = qb < S;
    const int q = qb + r32;

    bf16x8 qf[4], dof[4];
    float lse_q = 0.f, dl = 0.f;
    if (active) {
        const bf16 *orow = o + ((size_t)n * S + q) * d + a * 64;
        const bf16 *lrow = o_lo + ((size_t)n * S + q) * d + a * 64;
        const bf16 *drow = dout + ((size_t)n * S + q) * d + a * 64;
        // delta = rowsum(dO * O) with O to ~16 bits (o + o_lo): when the value rows of a head share a
        // large common component, dP - delta cancels it, and a delta built from bf16 O alone would not
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            qf[ks] = *(const bf16x8 *)(base + (size_t)q * ld + ks * 16 + g * 8);
            dof[ks] = *(const bf16x8 *)(drow + ks * 16 + g * 8);
            bf16x8 of = *(const bf16x8 *)(orow + ks * 16 + g * 8);
            bf16x8 ol = *(const bf16x8 *)(lrow + ks * 16 + g * 8);
#pragma unroll
            for (int i = 0; i < 8; ++i) dl += bf2f(dof[ks][i]) * (bf2f(of[i]) + bf2f(ol[i]));
        }
        dl += __shfl_xor(dl, 32, 64);
        lse_q = lse[((size_t)n * H + a) * S + q];
        if (g == 0) delta[((size_t)n * H + a) * S + q] = dl;
    }
    f32x16 dqacc[2] = {zero16(), zero16()};
    const int kv_end = min(S, qt * 128 + 128);
    const int ntile = kv_end >> 6;

#define DQ_TILE(Ks, Vs, k0)                                                                            \
    if (active && (k0) <= qb + 31) {                                                                   \
        const bool need_mask = (k0) + 63 > qb;                                                         \
        _Pragma("unroll") for (int mt = 0; mt < 2; ++mt) {                                             \
            f32x16 sacc = zero16(), dpacc = zero16();                                                  \
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {                                         \
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm(Ks, mt * 32 + r32, ks, g),      \
                                                                qf[ks], sacc, 0, 0, 0);                \
                dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm(Vs, mt * 32 + r32, ks, g),     \
                                                                 dof[ks], dpacc, 0, 0, 0);             \
            }                                                                                          \
            _Pragma("unroll") for (int e = 0; e < 16; ++e) {                                           \
                const int key = (k0) + 32 * mt + 8 * (e >> 2) + 4 * g + (e & 3);                       \
                float p = __builtin_amdgcn_exp2f(fmaf(sacc[e], kScaleLog2, -lse_q));                   \
                if (need_mask && key > q) p = 0.f;                                                     \
                sacc[e] = p * (dpacc[e] - dl);                                                         \
            }                                                                                          \
            _Pragma("unroll") for (int hh = 0; hh < 2; ++hh) {                                         \
                bf16x8 dsb;                                                                            \
                _Pragma("unroll") for (int i = 0; i < 8; ++i) dsb[i] = f2bf(sacc[8 * hh + i]);         \
                _Pragma("unroll") for (int dt = 0; dt < 2; ++dt)                                       \
                    dqacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                               \
                        frag_tr(Ks, 32 * dt, 32 * mt + 16 * hh, lane), dsb, dqacc[dt], 0, 0, 0);       \
            }                                                                                          \
        }                                                                                              \
    }

    const bf16 *kg = base + d, *vg = base + 2 * d;
    tile_copy_async(K0, kg, ld, wave, lane);
    tile_copy_async(V0, vg, ld, wave, lane);
    AT_WAIT_VM0();
    __syncthreads();
    int j = 0;
    for (; j + 2 <= ntile; j += 2) {
        tile_copy_async(K1, kg + (size_t)(j + 1) * 64 * ld, ld, wave, lane);
        tile_copy_async(V1, vg + (size_t)(j + 1) * 64 * ld, ld, wave, lane);
        DQ_TILE(K0, V0, j * 64)
        AT_WAIT_VM0();
        __syncthreads();
        if (j + 2 < ntile) {
            tile_copy_async(K0, kg + (size_t)(j + 2) * 64 * ld, ld, wave, lane);
            tile_copy_async(V0, vg + (size_t)(j + 2) * 64 * ld, ld, wave, lane);
        }
        DQ_TILE(K1, V1, (j + 1) * 64)
        AT_WAIT_VM0();
        __syncthreads();
    }
    if (j < ntile) DQ_TILE(K0, V0, j * 64)
#undef DQ_TILE

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
    }   // pass
}

// ------------------------------------------------------------------------------------------
// dK, dV: each wavefront owns 32 keys and walks the query tiles that can see them
__global__ __launch_bounds__(256, 2) void attn_bwd_dkv_kernel(const bf16 *__restrict__ qkv,
                                                           const bf16 *__restrict__ dout,
                                                           const float *__restrict__ lse,
                                                           const float *__restrict__ delta,
                                                           bf16 *__restrict__ dqkv, int S, int H, int n_seq)
{
    __shared__ __attribute__((aligned(1024))) unsigned char Q0[TILE_B], D0[TILE_B], Q1[TILE_B], D1[TILE_B];
    __shared__ __align__(16) float st0[128], st1[128];   // lse | delta of the 64 queries of a tile
    // block ids decoded as in the forward: the key tiles of a (sequence, head) share an XCD, and a block takes
    // the tiles j (most query tiles to walk) and nkt-1-j one after the other: equal work per block
    const int nkt = (S + 127) >> 7, npb = (nkt + 1) >> 1;
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int pair = (idx / npb) * 8 + xcd;
    if (pair >= H * n_seq) return;
    const int a = pair % H, n = pair / H;
    const int d = H * 64, ld = 3 * d;
    const int tid = threadIdx.x, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bf16 *base = qkv + (size_t)n * S * ld + a * 64;
    const bf16 *dbase = dout + (size_t)n * S * d + a * 64;
    const float *lse_b = lse + ((size_t)n * H + a) * S, *dl_b = delta + ((size_t)n * H + a) * S;
#pragma clang loop unroll(disable)
    for (int ph = 0; ph < 2; ++ph) {
    const int kvt = ph == 0 ? idx % npb : nkt - 1 - idx % npb;
    if (ph == 1) {
        if (kvt == idx % npb) break;                     // odd tile count: the middle tile stands alone
        __syncthreads();                                 // the first pass's tiles and statistics are no longer read
    }
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
    const int q_first = kvt * 128;
    const int ntile = (S - q_first) >> 6;

#define DKV_TILE(Qs, Ds, stt, q0)                                                                      \
    if (active) {                                                                                      \
        _Pragma("unroll") for (int st = 0; st < 2; ++st) {                                             \
            const int qs = (q0) + 32 * st;                                                             \
            if (qs + 31 >= kb) {                                                                       \
                const bool need_mask = qs < kb + 31;                                                   \
                f32x16 sacc = zero16(), dpacc = zero16();                                              \
                _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {                                     \
                    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm(Qs, 32 * st + r32, ks, g),  \
                                                                    kf[ks], sacc, 0, 0, 0);            \
                    dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm(Ds, 32 * st + r32, ks, g), \
                                                                     vf[ks], dpacc, 0, 0, 0);          \
                }                                                                                      \
                _Pragma("unroll") for (int e4 = 0; e4 < 4; ++e4) {                                     \
                    const int ql = 32 * st + 8 * e4 + 4 * g;                                           \
                    const f32x4 ls = *(const f32x4 *)((stt) + ql);                                     \
                    const f32x4 dd = *(const f32x4 *)((stt) + 64 + ql);                                \
                    if (need_mask) {                     /* sub-tiles that touch the diagonal */       \
                        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                \
                            const int e = 4 * e4 + i;                                                  \
                            float p = __builtin_amdgcn_exp2f(fmaf(sacc[e], kScaleLog2, -ls[i]));       \
                            if (key > (q0) + ql + i) p = 0.f;                                          \
                            sacc[e] = p;                                                               \
                            dpacc[e] = p * (dpacc[e] - dd[i]);                                         \
                        }                                                                              \
                    } else {                                                                           \
                        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                \
                            const int e = 4 * e4 + i;                                                  \
                            const float p = __builtin_amdgcn_exp2f(fmaf(sacc[e], kScaleLog2, -ls[i])); \
                            sacc[e] = p;                                                               \
                            dpacc[e] = p * (dpacc[e] - dd[i]);                                         \
                        }                                                                              \
                    }                                                                                  \
                }                                                                                      \
                _Pragma("unroll") for (int hh = 0; hh < 2; ++hh) {                                     \
                    bf16x8 pb, dsb;                                                                    \
                    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                    \
                        pb[i] = f2bf(sacc[8 * hh + i]);                                                \
                        dsb[i] = f2bf(dpacc[8 * hh + i]);                                              \
                    }                                                                                  \
                    _Pragma("unroll") for (int dt = 0; dt < 2; ++dt) {                                 \
                        dvacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                           \
                            frag_tr(Ds, 32 * dt, 32 * st + 16 * hh, lane), pb, dvacc[dt], 0, 0, 0);    \
                        dkacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                           \
                            frag_tr(Qs, 32 * dt, 32 * st + 16 * hh, lane), dsb, dkacc[dt], 0, 0, 0);   \
                    }                                                                                  \
                }                                                                                      \
            }                                                                                          \
        }                                                                                              \
    }
    // per-query statistics travel through a register so that their LDS store (which has to wait
    // for the load) sits after the MFMA work of the current tile
    float stat = 0.f;
#define DKV_ISSUE(Qs, Ds, q0)                                                                          \
    {                                                                                                  \
        tile_copy_async(Qs, base + (size_t)(q0) * ld, ld, wave, lane);                                 \
        tile_copy_async(Ds, dbase + (size_t)(q0) * d, d, wave, lane);                                  \
        if (tid < 64) stat = lse_b[(q0) + tid];                                                        \
        else if (tid < 128) stat = dl_b[(q0) + tid - 64];                                              \
    }
#define DKV_COMMIT(stt) if (tid < 128) (stt)[tid] = stat;

    DKV_ISSUE(Q0, D0, q_first)
    DKV_COMMIT(st0)
    AT_WAIT_VM0();
    __syncthreads();
    int j = 0;
    for (; j + 2 <= ntile; j += 2) {
        DKV_ISSUE(Q1, D1, q_first + (j + 1) * 64)
        DKV_TILE(Q0, D0, st0, q_first + j * 64)
        DKV_COMMIT(st1)
        AT_WAIT_VM0();
        __syncthreads();
        const bool more = j + 2 < ntile;
        if (more) DKV_ISSUE(Q0, D0, q_first + (j + 2) * 64)
        DKV_TILE(Q1, D1, st1, q_first + (j + 1) * 64)
        if (more) DKV_COMMIT(st0)
        AT_WAIT_VM0();
        __syncthreads();
    }
    if (j < ntile) DKV_TILE(Q0, D0, st0, q_first + j * 64)
#undef DKV_ISSUE
#undef DKV_COMMIT
#undef DKV_TILE

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
    }   // pass
}

// ------------------------------------------------------------------------------------------
// Fused backward for sequences of at most 512 tokens: one block of 8 wavefronts per (sequence, head)
// produces dQ, dK and dV in one pass, so the scores, the probabilities and dP are formed once instead
// of once per kernel, and K, V, Q, dO are read from memory once.
//   * K of the whole sequence sits in LDS; every wave owns two 32-key blocks (w and nb-1-w, which
//     balances the causal triangle), keeps their V fragments and their dK, dV accumulators in
//     registers, and walks the 32-query tiles that can see them (phase 1, as in the dK/dV kernel).
//   * dS of a query tile is written to LDS as dS^T [key][32 queries] bf16; after one barrier the 8
//     waves each form one 16 x 16 piece of dQ = dS K over all visible keys (phase 2), in a fixed
//     order -- no floating-point atomics, results stay bit-reproducible.
//   * Q / dO tiles (4 KB each) are double buffered asynchronous copies that also bring the tile's 32 K rows,
//     dS^T is double buffered too, so there is one barrier per query tile: phase 2 of tile i runs next to
//     phase 1 of tile i + 1.
//   * Before the arithmetic starts the block waits for one round of memory traffic: the first tile, the
//     wave's V fragments, and the operands of delta = rowsum(dO * O) of all rows, every load of which is
//     issued before the first is used.  (All blocks of a launch run in step, so this round is read by every
//     compute unit at once, at the memory's speed, with the matrix cores idle; forming delta tile by tile
//     behind the arithmetic, from rows streamed into LDS, was measured and only moved the same time into the
//     steps, whose length is set by the latency of the tile copies.)
constexpr int FB_MAXS = 512;

// XOR mask of the 8-byte slots of a dS^T row (64 bytes = 32 queries): conflict-free both for the
// phase-1 stores (16 lanes = 16 consecutive keys, one slot) and for the phase-2 transpose reads
// (16 lanes = 4 consecutive keys x 4 slots)
__device__ __forceinline__ int dsm(int key) { return (((key >> 1) & 1) << 2) | ((key >> 2) & 3); }

__global__ __launch_bounds__(512) void attn_bwd_fused_kernel(const bf16 *__restrict__ qkv, const bf16 *__restrict__ o,
                                                             const bf16 *__restrict__ o_lo,
                                                             const bf16 *__restrict__ dout,
                                                             const float *__restrict__ lse, bf16 *__restrict__ dqkv,
                                                             int S, int H, const float *__restrict__ delta_in)
{
    __shared__ __attribute__((aligned(1024))) unsigned char Ks[FB_MAXS * 128];
    __shared__ __attribute__((aligned(1024))) unsigned char dS0[FB_MAXS * 64], dS1[FB_MAXS * 64];
    __shared__ __attribute__((aligned(1024))) unsigned char Qb0[32 * 128], Db0[32 * 128], Qb1[32 * 128], Db1[32 * 128];
    __shared__ __align__(16) float lse_s[FB_MAXS], dl_s[FB_MAXS];
    const int a = blockIdx.x, n = blockIdx.y;
    const int d = H * 64, ld = 3 * d;
    const int tid = threadIdx.x, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const int i16 = lane & 15, kg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bf16 *base = qkv + (size_t)n * S * ld + a * 64;
    const bf16 *dbase = dout + (size_t)n * S * d + a * 64;
    const int nb = S >> 5;                               // 32-row blocks (even: S is a multiple of 64)

    // one 1 KB piece per wave and tile of Q (waves 0-3) and dO (waves 4-7), and the tile's 32 K rows (waves 0-3)
#define FB_COPY(Qd, Dd, it)                                                                            \
    {                                                                                                  \
        const int lrow_c = lane >> 3, lch_c = (lane & 7) ^ swm(lane >> 3);                             \
        const int row_c = 32 * (it) + (wave & 3) * 8 + lrow_c;                                         \
        if (wave < 4) {                                                                                \
            AT_GLDS(base + (size_t)row_c * ld + lch_c * 8, (Qd) + (wave & 3) * 1024);                  \
            AT_GLDS(base + d + (size_t)row_c * ld + lch_c * 8, Ks + (it) * 4096 + (wave & 3) * 1024);  \
        } else AT_GLDS(dbase + (size_t)row_c * d + lch_c * 8, (Dd) + (wave & 3) * 1024);               \
    }
    // ---- prologue: first tile (Q, dO, K rows), log-sum-exp and delta of all rows, this wave's V fragments
    FB_COPY(Qb0, Db0, 0)
    if (tid < S) lse_s[tid] = lse[((size_t)n * H + a) * S + tid];
    const bool owner = wave < (nb >> 1);                 // waves beyond the number of block pairs only do phase 2
    const int jb[2] = {wave, nb - 1 - wave};
    bf16x8 vf[2][4];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int key = min(32 * jb[b] + r32, S - 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            vf[b][ks] = *(const bf16x8 *)(base + 2 * d + (size_t)(owner ? key : 0) * ld + ks * 16 + g * 8);
    }
    // delta = rowsum(dO * (O + O_lo)): [T, H] from the product that formed dO (its epilogue has dO in registers
    // and reads O there, which saves this kernel a second pass over dO and half of its prologue's traffic), or
    if (delta_in != nullptr) {
        if (tid < S) dl_s[tid] = delta_in[((size_t)n * S + tid) * H + a];
    } else {
        // formed here: 8 lanes per row (16 bytes each, one full 128-byte line per row and
        // operand), 64 rows per pass, reduced with three shuffles; the loads of all passes go out first
        bf16x8 dv[FB_MAXS / 64], ov[FB_MAXS / 64], lv[FB_MAXS / 64];
        const size_t off_d = ((size_t)n * S + (tid >> 3)) * d + a * 64 + (tid & 7) * 8;
#pragma unroll
        for (int ps = 0; ps < FB_MAXS / 64; ++ps)
            if (64 * ps < S) {
                dv[ps] = *(const bf16x8 *)(dout + off_d + (size_t)64 * ps * d);
                ov[ps] = *(const bf16x8 *)(o + off_d + (size_t)64 * ps * d);
                lv[ps] = *(const bf16x8 *)(o_lo + off_d + (size_t)64 * ps * d);
            }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ps = 0; ps < FB_MAXS / 64; ++ps)
            if (64 * ps < S) {
                float dl = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) dl += bf2f(dv[ps][i]) * (bf2f(ov[ps][i]) + bf2f(lv[ps][i]));
                dl += __shfl_xor(dl, 1, 64);
                dl += __shfl_xor(dl, 2, 64);
                dl += __shfl_xor(dl, 4, 64);
                if ((tid & 7) == 0) dl_s[64 * ps + (tid >> 3)] = dl;
            }
    }
    f32x16 dkacc[2][2], dvacc[2][2];
    // phase 1 for query tile `it` (rows 32 it ..) against this wave's blocks that it can see.  Only the
    // block on the diagonal (j == it) needs the causal mask; the blocks below it run a copy without it.
#define FB_BLOCK(Qs, Ds, dSw, it, b, j, DIAG)                                                          \
    {                                                                                                  \
        f32x16 sacc = zero16(), dpacc = zero16();                                                      \
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {                                             \
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm(Qs, r32, ks, g),                    \
                                                            frag_rm(Ks, 32 * (j) + r32, ks, g), sacc, 0, 0, 0); \
            dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm(Ds, r32, ks, g), vf[b][ks],        \
                                                             dpacc, 0, 0, 0);                          \
        }                                                                                              \
        _Pragma("unroll") for (int e4 = 0; e4 < 4; ++e4) {                                             \
            const int ql = 8 * e4 + 4 * g;                                                             \
            const f32x4 ls = *(const f32x4 *)(lse_s + 32 * (it) + ql);                                 \
            const f32x4 dd = *(const f32x4 *)(dl_s + 32 * (it) + ql);                                  \
            bf16x4 dst4;                                                                               \
            _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                            \
                const int e = 4 * e4 + i;                                                              \
                float p = __builtin_amdgcn_exp2f(fmaf(sacc[e], kScaleLog2, -ls[i]));                   \
                if (DIAG && r32 > ql + i) p = 0.f;                                                     \
                sacc[e] = p;                                                                           \
                dpacc[e] = p * (dpacc[e] - dd[i]);                                                     \
                dst4[i] = f2bf(dpacc[e]);                                                              \
            }                                                                                          \
            const int key = 32 * (j) + r32;                                                            \
            *(bf16x4 *)((dSw) + key * 64 + (((2 * e4 + g) ^ dsm(key)) << 3)) = dst4;                   \
        }                                                                                              \
        _Pragma("unroll") for (int hh = 0; hh < 2; ++hh) {                                             \
            bf16x8 pb, dsb;                                                                            \
            _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                            \
                pb[i] = f2bf(sacc[8 * hh + i]);                                                        \
                dsb[i] = f2bf(dpacc[8 * hh + i]);                                                      \
            }                                                                                          \
            _Pragma("unroll") for (int dt = 0; dt < 2; ++dt) {                                         \
                dvacc[b][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                \
                    frag_tr(Ds, 32 * dt, 16 * hh, lane), pb, dvacc[b][dt], 0, 0, 0);                   \
                dkacc[b][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                \
                    frag_tr(Qs, 32 * dt, 16 * hh, lane), dsb, dkacc[b][dt], 0, 0, 0);                  \
            }                                                                                          \
        }                                                                                              \
    }
#define FB_PHASE1(Qs, Ds, dSw, it)                                                                     \
    if (owner) {                                                                                       \
        _Pragma("unroll") for (int b = 0; b < 2; ++b) {                                                \
            const int j = jb[b];                                                                       \
            if (j <= (it)) { const bool diag = j == (it); FB_BLOCK(Qs, Ds, dSw, it, b, j, diag) }      \
            __builtin_amdgcn_sched_barrier(0);           /* keep the two blocks' live ranges apart */   \
        }                                                                                              \
    }
    // phase 2 for query tile `it`: wave w forms dQ[16 qt .. +15][16 dt .. +15], qt = w / 4, dt = w % 4,
    // as (K^T dS^T)^T over all visible keys; the lane ends up with 4 consecutive columns of one query
    // The rows a lane reads are 32 kk + (a lane constant below 32) and neither swizzle looks above bit 3 of
    // the row, so everything but the 32 kk step is formed once here (left in the loop the compiler rebuilt the
    // swizzles for every key block: 17 VALU instructions per MFMA).
    const int p2_qt = wave >> 2, p2_dt = wave & 3;
    int p2_k[2], p2_d[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int row = 8 * kg + 4 * h + (i16 >> 2);
        const int colk = 16 * p2_dt + 4 * (i16 & 3);
        p2_k[h] = row * 128 + (((colk >> 3) ^ swm(row)) << 4) + (colk & 7) * 2;
        p2_d[h] = row * 64 + (((4 * p2_qt + (i16 & 3)) ^ dsm(row)) << 3);
    }
#define FB_PHASE2(dSr, it)                                                                             \
    {                                                                                                  \
        f32x4 qacc = {0.f, 0.f, 0.f, 0.f};                                                             \
        _Pragma("unroll 2") for (int kk = 0; kk <= (it); ++kk) {                                       \
            union { v4s s[2]; bf16x8 v; } ua, ub;                                                      \
            _Pragma("unroll") for (int h = 0; h < 2; ++h) {                                            \
                const unsigned char *pk = Ks + kk * 4096 + p2_k[h];                                    \
                const unsigned char *pd = (dSr) + kk * 2048 + p2_d[h];                                 \
                ua.s[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s *)pk); \
                ub.s[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s *)pd); \
            }                                                                                          \
            qacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua.v, ub.v, qacc, 0, 0, 0);                 \
        }                                                                                              \
        const int q = 32 * (it) + 16 * p2_qt + i16;                                                    \
        bf16x4 w4;                                                                                     \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) w4[e] = f2bf(qacc[e] * 0.125f);                  \
        *(bf16x4 *)(dqkv + ((size_t)n * S + q) * ld + a * 64 + 16 * p2_dt + 4 * kg) = w4;              \
    }

    AT_WAIT_VM0();
    __syncthreads();                                     // tile 0, its K rows and the statistics it needs are in LDS
    if (nb > 1) FB_COPY(Qb1, Db1, 1)
#pragma unroll
    for (int b = 0; b < 2; ++b) { dkacc[b][0] = zero16(); dkacc[b][1] = zero16(); dvacc[b][0] = zero16(); dvacc[b][1] = zero16(); }
    FB_PHASE1(Qb0, Db0, dS0, 0)
    for (int it = 0; it < nb; it += 2) {
        AT_WAIT_VM0();
        __syncthreads();                                 // dS^T of tile it complete; tile it + 1 and its K rows landed
        if (it + 2 < nb) FB_COPY(Qb0, Db0, it + 2)
        FB_PHASE2(dS0, it)
        if (it + 1 < nb) FB_PHASE1(Qb1, Db1, dS1, it + 1)
        if (it + 1 < nb) {
            AT_WAIT_VM0();
            __syncthreads();
            if (it + 3 < nb) FB_COPY(Qb1, Db1, it + 3)
            FB_PHASE2(dS1, it + 1)
            if (it + 2 < nb) FB_PHASE1(Qb0, Db0, dS0, it + 2)
        }
    }
#undef FB_COPY
#undef FB_PHASE1
#undef FB_BLOCK
#undef FB_PHASE2

    // dK, dV of the two key blocks leave through LDS (the dS^T buffers, free after one more barrier) as whole
    // 128-byte lines: a lane holds 4 consecutive columns of one key per register group, direct stores would
    // touch 32 lines per instruction with 8 bytes each
    __syncthreads();
    if (owner) {
        unsigned char *stg = wave < 4 ? dS0 + wave * OST_B : dS1 + (wave - 4) * OST_B;      // 4.5 KB per wave
        const int orow = lane >> 3, och = lane & 7;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            bf16 *out = dqkv + ((size_t)n * S + 32 * jb[b] + orow) * ld + d + a * 64 + och * 8;
#pragma unroll
            for (int which = 0; which < 2; ++which) {     // 0: dK (scaled), 1: dV
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        bf16x4 w;
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            w[i] = which ? f2bf(dvacc[b][dt][4 * e4 + i]) : f2bf(dkacc[b][dt][4 * e4 + i] * 0.125f);
                        *(bf16x4 *)(stg + r32 * OST_PITCH + (32 * dt + 8 * e4 + 4 * g) * 2) = w;
                    }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                bf16x8 rows[4];
#pragma unroll
                for (int it = 0; it < 4; ++it)
                    rows[it] = *(const bf16x8 *)(stg + (8 * it + orow) * OST_PITCH + och * 16);
#pragma unroll
                for (int it = 0; it < 4; ++it) *(bf16x8 *)(out + (size_t)(8 * it) * ld + which * d) = rows[it];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
}

}  // namespace

int launch_attn_fwd(const bf16 *qkv, bf16 *o, bf16 *o_lo, float *lse, int n_seq, int S, int H, hipStream_t st)
{
    if (n_seq <= 0 || S <= 0 || (S % 64) || H <= 0) return SL_EINVAL;
    const long long pairs8 = ((long long)H * n_seq + 7) / 8 * 8;
    const long long nblk = pairs8 * (((S + 127) / 128 + 1) / 2);     // two query tiles of 128 per block
    if (nblk > 0x7fffffffLL) return SL_EINVAL;
    // algorithmic work: two products over the lower triangle, 2 S d flop per token (d = 64 H)
    const bool rec = prof_begin(PK_ATTN_FWD, st);
    hipLaunchKernelGGL(attn_fwd_kernel, dim3((unsigned)nblk), dim3(256), 0, st, qkv, o, o_lo, lse, S, H, n_seq);
    prof_end(rec, PK_ATTN_FWD, 2.0 * S * 64.0 * H * ((double)n_seq * S), st);
    SL_CHECK_LAUNCH("attn_fwd");
    return 0;
}

bool attn_bwd_takes_delta(int S) { return S > 0 && S <= FB_MAXS && (S % 64) == 0; }

int launch_attn_bwd(const bf16 *qkv, const bf16 *o, const bf16 *o_lo, const bf16 *dout, const float *lse,
                    float *delta, bf16 *dqkv, int n_seq, int S, int H, hipStream_t st, bool delta_ready)
{
    if (delta_ready && !attn_bwd_takes_delta(S)) return SL_EINVAL;
    if (n_seq <= 0 || S <= 0 || (S % 64) || H <= 0) return SL_EINVAL;
    // algorithmic work: four products over the lower triangle (the recomputed scores are not counted)
    const double work = 4.0 * S * 64.0 * H * ((double)n_seq * S);
    const bool rec = prof_begin(PK_ATTN_BWD, st);
    if (S <= FB_MAXS) {
        hipLaunchKernelGGL(attn_bwd_fused_kernel, dim3(H, n_seq), dim3(512), 0, st, qkv, o, o_lo, dout, lse, dqkv, S, H,
                           delta_ready ? (const float *)delta : nullptr);
        prof_end(rec, PK_ATTN_BWD, work, st);
        SL_CHECK_LAUNCH("attn_bwd_fused");
        return 0;
    }
    const long long pairs8 = ((long long)H * n_seq + 7) / 8 * 8;
    const long long nblk = pairs8 * (((S + 127) / 128 + 1) / 2);     // two tiles of 128 rows per block
    if (nblk > 0x7fffffffLL) return SL_EINVAL;
    const dim3 grid((unsigned)nblk);
    hipLaunchKernelGGL(attn_bwd_dq_kernel, grid, dim3(256), 0, st, qkv, o, o_lo, dout, lse, delta, dqkv, S, H, n_seq);
    SL_CHECK_LAUNCH("attn_bwd_dq");
    hipLaunchKernelGGL(attn_bwd_dkv_kernel, grid, dim3(256), 0, st, qkv, dout, lse, delta, dqkv, S, H, n_seq);
    prof_end(rec, PK_ATTN_BWD, work, st);
    SL_CHECK_LAUNCH("attn_bwd_dkv");
    return 0;
}
