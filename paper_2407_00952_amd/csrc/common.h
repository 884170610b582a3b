// Internal declarations shared by the HIP sources of libslora (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

typedef __bf16 bf16;
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Return codes of the internal launchers.  They travel unchanged through the C ABI, so they carry the values of
// SLORA_OK, SLORA_EINVAL and SLORA_EHIP (asserted where the ABI header is included).
enum { SL_OK = 0, SL_EINVAL = -1, SL_EHIP = -4 };

#define SL_WAVE 64
#define SL_RP 16            // adapter rank padded to one MFMA k-step
#define SL_MAX_CLIENTS 64

static __device__ __forceinline__ float bf2f(bf16 v) { return (float)v; }
static __device__ __forceinline__ bf16 f2bf(float v) { return (bf16)v; }

// wave-wide sum through DPP-free shuffles (64 lanes)
static __device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// GELU_tanh(f) = f * sigma(2u), u = sqrt(2/pi) (f + 0.044715 f^3), and its derivative
//   GELU'(f) = sigma + f sigma (1 - sigma) * 2 sqrt(2/pi) (1 + 3 * 0.044715 f^2)
// from one sigmoid evaluation.  The exponent is formed directly in base 2 (v_exp_f32 is 2^x) and
// the polynomials are explicit FMAs: 9 full-rate and 2 quarter-rate instructions per element,
// which matters because the GEMM epilogue that calls this is ALU-bound.
static __device__ __forceinline__ void gelu_fwd_bwd(float f, float &gval, float &gder)
{
    const float c2 = 1.5957691216057308f;                  // 2 sqrt(2/pi)
    const float k = 0.044715f;
    const float l2e = 1.4426950408889634f;                 // log2(e)
    const float t = f * f;
    const float e = __builtin_amdgcn_exp2f(f * fmaf(t, -(c2 * k * l2e), -(c2 * l2e)));   // e^{-2u}
    const float sg = __builtin_amdgcn_rcpf(1.0f + e);
    gval = f * sg;
    gder = fmaf(gval * (1.0f - sg), fmaf(t, 3.0f * k * c2, c2), sg);
}

// The K clients' buffers as one logical [sum b_i * S, d] matrix (client-major concatenation).
struct ClientTable {
    void *ptr[SL_MAX_CLIENTS];     // bf16 rows, or MXFP8 element codes when mx != 0
    void *aux[SL_MAX_CLIENTS];     // MXFP8 scale codes ([rows, d/32]) when mx != 0, unused otherwise
    int row_end[SL_MAX_CLIENTS];   // exclusive prefix of rows (tokens)
    int K;
    int mx;                        // the buffers hold MXFP8 (compressed cut-layer traffic) instead of bf16
};

// Token + position embedding as the source of the first client-side block (row t of the input is
// wte[tokens[t]] + wpe[t % seq_len]).
struct EmbedSrc {
    const int *tokens;             // [T]
    const bf16 *wte, *wpe;         // [vocab, d], [>= seq_len, d]
    int seq_len, vocab;
};

// ---- GEMM ---------------------------------------------------------------------------------
// EPI_STORE_DELTA: plain store of a [M, 64 H] tensor that is the gradient of an attention output, plus
// delta[row][head] = sum over the head's 64 columns of out * (dl_o + dl_lo) (4-wave kernel only)
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_GELU = 2, EPI_DGELU = 3, EPI_STORE_DELTA = 4 };

// Compressed mode of a context: the frozen operand of a GEMM as MXFP8 codes + block scales (packed once),
// and scratch for the codes + scales of its activation operand, which is converted right before the launch.
struct MxOperands {
    const unsigned char *wq, *ws;    // [N,K] element codes, [N,K/32] scale codes
    unsigned char *xq, *xs;          // [M,K], [M,K/32]: conversion scratch, or (x_ready) codes a producer wrote
    int x_ready;                     // the kernel that produced X also wrote its codes: no conversion pass
};

struct GemmArgs {
    const bf16 *X; int ldx;          // [M,K]
    const bf16 *W; int ldw;          // [N,K]  (N = nseg * seg_n)
    int M, N, K;
    int nseg, seg_n;
    const bf16 *bias;                // [N] or null
    // low-rank branch, per segment (null zmat = segment not adapted)
    const bf16 *zmat[3]; int ldz;    // [NZ,K]: rows of the down-projection(s), 16 per adapter, zero beyond the rank
    const bf16 *tmat[3]; int ldt;    // [seg_n,ldt]: up-projection, ldt = NZ rounded up to 32, zero beyond the rank
    bf16 *zspill[3];                 // [M,K2] or null: scaled bf16 copy of the rank-space activations
    int K2; float zscale;            // K2 = NZ
    // epilogue
    void *out0; void *out1; const void *aux; int ldo;
    const bf16 *dl_o, *dl_lo; float *dl_out;   // EPI_STORE_DELTA: the two bf16 terms of O [M,ldo], delta [M,N/64] fp32
    const MxOperands *mx;            // null: bf16 product.  Else: the product runs on the fp8 matrix cores
    // compressed mode only: also write the bf16 tensor of the epilogue (GELU: out1, DGELU: out0) as MXFP8
    // codes [M,ldo] + scales [M,ldo/32], so that the product that consumes it needs no conversion pass
    unsigned char *oq, *os;
    static constexpr bool kEmitCodes = false;   // the bf16 kernel never does
    unsigned long long *clk;         // measurement hook: four words for clock stamps of this launch, or null
};

int launch_gemm(const GemmArgs &a, int epi, int nz, hipStream_t st);
// the same call with the frozen product in MXFP8 (a.mx set): converts X, forms the rank-space activations
// of the adapted segments with a separate projection kernel (into a.zspill), then one fp8 GEMM launch
int launch_gemm_mx_stack(const GemmArgs &a, int epi, int nz, hipStream_t st);
int launch_mx_quantize(const bf16 *x, long long ldx, long long M, int K, unsigned char *codes, unsigned char *scales,
                       hipStream_t st);

// ---- elementwise / norm / attention / lora-grad launchers ---------------------------------------
int launch_ln_fwd(const float *h_f32, const ClientTable *gather /*null unless block 0*/, float *h_copy,
                  const bf16 *gamma, const bf16 *beta, float eps, bf16 *u, float *stats, int T, int d,
                  hipStream_t st, const EmbedSrc *embed = nullptr, unsigned char *u_codes = nullptr,
                  unsigned char *u_scales = nullptr);   // optional MXFP8 copy of u (d a multiple of 32)
int launch_ln_bwd(const bf16 *du, const float *h, const float *stats, const bf16 *gamma,
                  const float *dres_f32, const bf16 *dres_bf16, float *out_f32, bf16 *out_bf16,
                  const ClientTable *scatter, int T, int d, hipStream_t st, unsigned char *o_codes = nullptr,
                  unsigned char *o_scales = nullptr);   // optional MXFP8 copy of out_bf16
int launch_attn_fwd(const bf16 *qkv, bf16 *o, bf16 *o_lo, float *lse, int n_seq, int S, int H, hipStream_t st);
// whether the backward at this sequence length takes delta = rowsum(dO * O) as an input ([T, H] fp32, filled by the
// product that forms dO) instead of forming it itself
bool attn_bwd_takes_delta(int S);
int launch_attn_bwd(const bf16 *qkv, const bf16 *o, const bf16 *o_lo, const bf16 *dout, const float *lse,
                    float *delta, bf16 *dqkv, int n_seq, int S, int H, hipStream_t st, bool delta_ready = false);
// G[c, j] = sum_t X[t, c] * Y[t, j], j < r; written transposed ([r, C]) when out_is_rxC.
int launch_lora_grad(const bf16 *X, int ldx, int C, const bf16 *Y, int ldy, int r, int T,
                     float *partials, float *out, int out_is_rxC, hipStream_t st);
int launch_lora_grad_pair(const bf16 *X, int ldx, int C, const bf16 *Y, int ldy, int r, int T,
                          float *partials, float *out_a, float *out_b, int out_is_rxC, hipStream_t st);
size_t lora_grad_partial_floats(int T, int C);
// several of them in one launch pair (same T and r; each with partial-sum scratch of its own)
struct LoraGradDesc {
    const bf16 *X; const bf16 *Y;    // tall operand [T,C] (pitch ldx); skinny operand [T,16] (or [T,32] when dual)
    float *partials;                 // lora_grad_partial_floats(T, C) floats
    float *out_a, *out_b;            // out_b: the second adapter of a dual job, else null
    int ldx, ldy, C; bool dual; int out_is_rxC;
};
int launch_lora_grad_jobs(const LoraGradDesc *d, int njobs, int r, int T, hipStream_t st);
int launch_fedavg(int K, const float *const *x, const float *w, size_t n, float *out, hipStream_t st);
int launch_sgd(float *p, const float *g, float lr, size_t n, hipStream_t st);
int launch_adamw(float *p, const float *g, float *m, float *v, size_t n, float b1, float b2, float eps, float decay,
                 float a, float c, float o1, float o2, hipStream_t st);
int launch_cast_pad(const float *src, int rows, int cols, bf16 *dst, int drows, int dcols, int transpose,
                    hipStream_t st);
int launch_transpose_bf16(const bf16 *src, int rows, int cols, bf16 *dst, hipStream_t st);
int launch_fill_zero(void *p, size_t bytes, hipStream_t st);

const char *set_hip_error(hipError_t e, const char *where);
#define SL_CHECK_LAUNCH(where)                                          \
    do {                                                                \
        hipError_t e__ = hipGetLastError();                             \
        if (e__ != hipSuccess) { set_hip_error(e__, where); return SL_EHIP; } \
    } while (0)
