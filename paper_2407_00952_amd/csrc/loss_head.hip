// Loss head of the server (SplitLoRA Sec. III-B: the clients send their labels with the activations
// in step a2; in step a3 the server turns its predicted value and the labels into the loss and starts
// the backward pass from it).  GPT-2's head: final LayerNorm, logits against the frozen token-embedding
// matrix Wv [V, d], token cross-entropy averaged over the labeled tokens; nothing here is trainable, so
// the only gradient produced is dY, the input of the server stack's backward pass.
//
// Schedule, per chunk of at most 16384 tokens (HBM is large: the chunk's logits are materialised once
// as bf16, 1.65 GB, instead of being recomputed):
//   u      = LN(y)                                 wave-per-row LayerNorm kernel
//   logits = u . WvP^T            [rows, Vp]       bf16 MFMA GEMM (Vp = V rounded up to 64, zero rows)
//   dlogits = (softmax(logits) - onehot) / n       one block per row, the row held in registers,
//   loss_tok = logsumexp - logits[label]           written over the logits
//   du     = dlogits . Wv         [rows, d]        the same GEMM on the transposed copy WvT [d, Vp]
//   dY     = LN^T(du)                              LayerNorm input-gradient kernel
// and one fixed-order reduction of loss_tok.  The number of labeled tokens n is counted on the device
// first; nothing synchronises the stream.
#include "../../include/slora.h"
#include "common.h"

#include <cstring>

namespace {

constexpr int CE_THR = 512;
constexpr int CE_MAXCH = 16;             // 16-byte chunks per thread: padded vocabulary <= 65536
constexpr int LH_CHUNK = 16384;          // tokens per pass

struct LabelCount { int n; float inv_n; };

inline size_t al256(size_t v) { return (v + 255) & ~(size_t)255; }
inline int vocab_padded(int V) { return (V + 63) / 64 * 64; }

__device__ __forceinline__ float block_reduce(float v, bool is_max, float *red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float w = __shfl_xor(v, o, 64);
        v = is_max ? fmaxf(v, w) : v + w;
    }
    const int wave = threadIdx.x >> 6;
    __syncthreads();                     // `red` may still be read from the previous reduction
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < CE_THR / 64; ++i) r = is_max ? fmaxf(r, red[i]) : r + red[i];
    return r;
}

// labels >= 0 (and < V) carry a loss; anything else marks a token without label
__global__ __launch_bounds__(1024) void count_labels_kernel(const int *__restrict__ labels, int T, int V,
                                                            LabelCount *__restrict__ out)
{
    __shared__ int red[16];
    int n = 0;
    for (int i = threadIdx.x; i < T; i += 1024) {
        const int l = labels[i];
        n += (l >= 0 && l < V) ? 1 : 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) n += __shfl_xor(n, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) {
        int tot = 0;
        for (int i = 0; i < 16; ++i) tot += red[i];
        out->n = tot;
        out->inv_n = tot > 0 ? 1.0f / (float)tot : 0.0f;
    }
}

// One block per token row.  logits [rows, ldl] bf16 in; the same memory receives
// d loss / d logits = (softmax - onehot) * inv_n (zero on unlabeled rows and in the padding columns).
__global__ __launch_bounds__(CE_THR) void softmax_ce_kernel(bf16 *__restrict__ logits, int ldl, int V,
                                                            const int *__restrict__ labels,
                                                            const LabelCount *__restrict__ cnt,
                                                            float *__restrict__ loss_tok)
{
    __shared__ float red[CE_THR / 64];
    const int row = blockIdx.x, tid = threadIdx.x;
    const int label = labels[row];
    bf16 *p = logits + (size_t)row * ldl;
    const int nch = ldl >> 3;
    if (label < 0 || label >= V) {
        bf16x8 z;
#pragma unroll
        for (int i = 0; i < 8; ++i) z[i] = f2bf(0.f);
        for (int c = tid; c < nch; c += CE_THR) *(bf16x8 *)(p + c * 8) = z;
        if (tid == 0) loss_tok[row] = 0.f;
        return;
    }
    const float picked = bf2f(p[label]);     // read before any thread overwrites the row (barriers below)
    const float l2e = 1.4426950408889634f;
    bf16x8 v[CE_MAXCH];
    float m = -INFINITY;
#pragma unroll
    for (int c = 0; c < CE_MAXCH; ++c) {
        const int ch = tid + c * CE_THR;
        if (ch < nch) {
            v[c] = *(const bf16x8 *)(p + ch * 8);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (ch * 8 + i < V) m = fmaxf(m, bf2f(v[c][i]));
        }
    }
    m = block_reduce(m, true, red);
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < CE_MAXCH; ++c) {
        const int ch = tid + c * CE_THR;
        if (ch < nch) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (ch * 8 + i < V) s += __builtin_amdgcn_exp2f((bf2f(v[c][i]) - m) * l2e);
        }
    }
    s = block_reduce(s, false, red);
    const float lse = m + __logf(s);
    if (tid == 0) loss_tok[row] = lse - picked;
    const float inv_n = cnt->inv_n;
#pragma unroll
    for (int c = 0; c < CE_MAXCH; ++c) {
        const int ch = tid + c * CE_THR;
        if (ch < nch) {
            bf16x8 o;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int col = ch * 8 + i;
                float g = 0.f;
                if (col < V) {
                    g = __builtin_amdgcn_exp2f((bf2f(v[c][i]) - lse) * l2e);
                    if (col == label) g -= 1.0f;
                    g *= inv_n;
                }
                o[i] = f2bf(g);
            }
            *(bf16x8 *)(p + ch * 8) = o;
        }
    }
}

// loss = (sum_t loss_tok[t]) / n, one block, fixed order, double accumulation
__global__ __launch_bounds__(1024) void loss_mean_kernel(const float *__restrict__ loss_tok, int T,
                                                         const LabelCount *__restrict__ cnt, float *__restrict__ loss)
{
    __shared__ double red[1024];
    double a = 0.0;
    for (int i = threadIdx.x; i < T; i += 1024) a += (double)loss_tok[i];
    red[threadIdx.x] = a;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = (float)(red[0] / (double)cnt->n);   // n = 0: 0/0 = NaN marks "no labeled token"
}

struct HeadWs {
    size_t WvP, WvT;                     // persistent: independent of the token count
    size_t u, hcopy, stats, du, logits, cnt, total;
};

HeadWs head_ws(int T, int d, int V)
{
    const size_t Vp = (size_t)vocab_padded(V);
    HeadWs w;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += al256(bytes); return o; };
    w.WvP = take(2 * Vp * d);
    w.WvT = take(2 * Vp * d);
    w.cnt = take(sizeof(LabelCount));
    w.u = take(2 * (size_t)T * d);
    w.hcopy = take(4 * (size_t)T * d);
    w.stats = take(8 * (size_t)T);
    w.du = take(2 * (size_t)T * d);
    w.logits = take(2 * (size_t)(T < LH_CHUNK ? T : LH_CHUNK) * Vp);
    w.total = off;
    return w;
}

bool head_args_ok(int T, int d, int V)
{
    if (T <= 0 || d <= 0 || V <= 0) return false;
    if ((d % 64) || d > 2048) return false;
    if (vocab_padded(V) > CE_MAXCH * CE_THR * 8) return false;
    return true;
}

GemmArgs plain_gemm(const bf16 *X, int ldx, const bf16 *W, int ldw, int M, int N, int K, void *out, int ldo)
{
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.X = X; a.ldx = ldx; a.W = W; a.ldw = ldw; a.M = M; a.N = N; a.K = K;
    a.nseg = 1; a.seg_n = N; a.ldo = ldo; a.out0 = out; a.K2 = 16; a.ldz = K; a.ldt = 32;
    return a;
}

}  // namespace

extern "C" {

size_t slora_loss_head_ws_bytes(int32_t max_tokens, int32_t d_model, int32_t vocab)
{
    if (!head_args_ok(max_tokens, d_model, vocab)) return 0;
    return head_ws(max_tokens, d_model, vocab).total;
}

int slora_loss_head_prepare(int32_t d_model, int32_t vocab, const void *Wv, void *ws, size_t ws_bytes, void *stream)
{
    if (!head_args_ok(1, d_model, vocab) || !Wv || !ws) return SLORA_EINVAL;
    if ((((uintptr_t)ws) & 255) || (((uintptr_t)Wv) & 15)) return SLORA_EINVAL;
    const HeadWs w = head_ws(1, d_model, vocab);
    if (ws_bytes < w.total) return SLORA_ENOSPC;
    hipStream_t st = (hipStream_t)stream;
    char *base = (char *)ws;
    const int Vp = vocab_padded(vocab);
    const hipError_t e = hipMemcpyAsync(base + w.WvP, Wv, 2 * (size_t)vocab * d_model, hipMemcpyDeviceToDevice, st);
    if (e != hipSuccess) { set_hip_error(e, "loss_head_prepare copy"); return SLORA_EHIP; }
    int rc;
    if ((rc = launch_fill_zero(base + w.WvP + 2 * (size_t)vocab * d_model, 2 * (size_t)(Vp - vocab) * d_model, st)))
        return rc;
    return launch_transpose_bf16((const bf16 *)(base + w.WvP), Vp, d_model, (bf16 *)(base + w.WvT), st);
}

int slora_loss_head(int32_t T, int32_t d_model, int32_t vocab, const void *y, const void *lnf_g, const void *lnf_b,
                    float eps, const int32_t *labels, void *ws, size_t ws_bytes, float *loss_tok, float *loss,
                    void *dy, void *stream)
{
    if (!head_args_ok(T, d_model, vocab) || !y || !lnf_g || !lnf_b || !labels || !ws || !loss_tok || !loss || !dy)
        return SLORA_EINVAL;
    if ((((uintptr_t)ws) & 255) || ((((uintptr_t)y) | ((uintptr_t)dy)) & 15)) return SLORA_EINVAL;
    const HeadWs w = head_ws(T, d_model, vocab);
    if (ws_bytes < w.total) return SLORA_ENOSPC;
    hipStream_t st = (hipStream_t)stream;
    char *base = (char *)ws;
    const int d = d_model, Vp = vocab_padded(vocab);
    bf16 *u = (bf16 *)(base + w.u), *du = (bf16 *)(base + w.du), *logits = (bf16 *)(base + w.logits);
    float *hcopy = (float *)(base + w.hcopy), *stats = (float *)(base + w.stats);
    LabelCount *cnt = (LabelCount *)(base + w.cnt);
    int rc;

    ClientTable one;                      // the stack output as a single "client" buffer of bf16 rows
    one.mx = 0;
    one.K = 1;
    one.ptr[0] = const_cast<void *>(y);
    one.row_end[0] = T;
    if ((rc = launch_ln_fwd(nullptr, &one, hcopy, (const bf16 *)lnf_g, (const bf16 *)lnf_b, eps, u, stats, T, d, st)))
        return rc;
    hipLaunchKernelGGL(count_labels_kernel, dim3(1), dim3(1024), 0, st, labels, T, vocab, cnt);
    SL_CHECK_LAUNCH("count_labels");

    for (int r0 = 0; r0 < T; r0 += LH_CHUNK) {
        const int rows = (T - r0 < LH_CHUNK) ? T - r0 : LH_CHUNK;
        GemmArgs a = plain_gemm(u + (size_t)r0 * d, d, (const bf16 *)(base + w.WvP), d, rows, Vp, d, logits, Vp);
        if ((rc = launch_gemm(a, EPI_STORE, 0, st))) return rc;
        hipLaunchKernelGGL(softmax_ce_kernel, dim3(rows), dim3(CE_THR), 0, st, logits, Vp, vocab, labels + r0, cnt,
                           loss_tok + r0);
        SL_CHECK_LAUNCH("softmax_ce");
        GemmArgs b = plain_gemm(logits, Vp, (const bf16 *)(base + w.WvT), Vp, rows, d, Vp, du + (size_t)r0 * d, d);
        if ((rc = launch_gemm(b, EPI_STORE, 0, st))) return rc;
    }
    if ((rc = launch_ln_bwd(du, hcopy, stats, (const bf16 *)lnf_g, nullptr, nullptr, nullptr, (bf16 *)dy, nullptr, T, d,
                            st)))
        return rc;
    hipLaunchKernelGGL(loss_mean_kernel, dim3(1), dim3(1024), 0, st, loss_tok, T, cnt, loss);
    SL_CHECK_LAUNCH("loss_mean");
    return SLORA_OK;
}

}  // extern "C"
