// C ABI of libslora: context, workspace layout and the per-block kernel schedule of the
// server-side step of split federated LoRA fine-tuning (SplitLoRA Sec. III-B a3, a4, b2).
// Host code only; every device operation is a kernel launch on the caller's stream.
#include "../../include/slora.h"
#include "common.h"
#include "prof.h"

#include <array>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

int f32_lora_linear_fwd(int T, int n_in, int n_out, int r, float s, const float *x, const float *W,
                        const float *bias, const float *A, const float *B, float *y, float *ws, hipStream_t st);
int f32_lora_linear_bwd(int T, int n_in, int n_out, int r, float s, const float *x, const float *dy,
                        const float *W, const float *A, const float *B, float *dx, float *dA, float *dB, float *ws,
                        hipStream_t st);

static_assert(PK_GEMM == SLORA_PROF_GEMM && PK_LN_FWD == SLORA_PROF_LN_FWD && PK_LN_BWD == SLORA_PROF_LN_BWD &&
              PK_LORA_GRAD == SLORA_PROF_LORA_GRAD && PK_SGD == SLORA_PROF_SGD && PK_ATTN_FWD == SLORA_PROF_ATTN_FWD &&
              PK_ATTN_BWD == SLORA_PROF_ATTN_BWD && PK_FEDAVG == SLORA_PROF_FEDAVG && PK_COUNT == SLORA_PROF_KINDS,
              "kinds of the measurement hook");
static_assert(SL_OK == SLORA_OK && SL_EINVAL == SLORA_EINVAL && SL_EHIP == SLORA_EHIP,
              "internal launcher codes must be the ABI's codes");


// ---- descriptor-driven batched kernels (one launch for every adapter of every block) ----------
struct CastDesc {            // fp32 [rows,cols] (optionally transposed) -> bf16 block [drows,dcols], pitch ld
    const float *src; bf16 *dst;
    int rows, cols, transpose, ld, drows, dcols;
};
struct SgdDesc { float *p; const float *g; int n; int pad; };

__global__ __launch_bounds__(256) void cast_table_kernel(const CastDesc *__restrict__ tab)
{
    const CastDesc d = tab[blockIdx.y];
    const int total = d.drows * d.dcols;
    for (int idx = blockIdx.x * 256 + threadIdx.x; idx < total; idx += gridDim.x * 256) {
        const int i = idx / d.dcols, j = idx - i * d.dcols;
        float v = 0.f;
        if (!d.transpose) {
            if (i < d.rows && j < d.cols) v = d.src[(size_t)i * d.cols + j];
        } else {
            if (j < d.rows && i < d.cols) v = d.src[(size_t)j * d.cols + i];
        }
        d.dst[(size_t)i * d.ld + j] = f2bf(v);
    }
}

__global__ __launch_bounds__(256) void sgd_table_kernel(const SgdDesc *__restrict__ tab, float lr)
{
    const SgdDesc d = tab[blockIdx.y];
    for (int i = blockIdx.x * 256 + threadIdx.x; i < d.n; i += gridDim.x * 256)
        d.p[i] = __fmaf_rn(-lr, d.g[i], d.p[i]);
}

// A table built on the host reaches the device as kernel arguments (copied when the launch is queued), so no
// host buffer has to outlive the call, nothing blocks, and the call can be captured into a graph.
struct TableChunk { uint32_t w[960]; };      // 3840 bytes per launch, within the kernel-argument limit
__global__ __launch_bounds__(256) void table_upload_kernel(uint32_t *__restrict__ dst, TableChunk c, int nwords)
{
    for (int i = threadIdx.x; i < nwords; i += 256) dst[i] = c.w[i];
}

// ---- error text --------------------------------------------------------------------------------
static thread_local char g_hip_err[256] = "";
const char *set_hip_error(hipError_t e, const char *where)
{
    snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s", where, hipGetErrorString(e));
    return g_hip_err;
}

namespace {

inline size_t al256(size_t v) { return (v + 255) & ~(size_t)255; }

struct AdapterBind { float *A, *B, *dA, *dB; };

struct BlockWs {
    // persistent: transposed frozen weights and bf16 adapter shadows
    size_t WqkvT, WoT, WfcT, WprT;
    size_t fz[SLORA_NPROJ], ft[SLORA_NPROJ];   // forward: down-projection [16,in], up-projection [out,32]
    size_t bz[SLORA_NPROJ], bt[SLORA_NPROJ];   // backward (o, fc, pr): B^T [16,out], A^T [in,32]
    size_t bz_qkv, bt_qkv;                     // backward, fused q|k|v: block-diagonal B^T [16n,3d], A^T [d,K2P]
    // saved between forward and backward
    size_t h_in, stats1, qkv, o, o_lo, lse, h_mid, stats2, f, u, u2, g;
    size_t zs[SLORA_NPROJ];
    // compressed mode: MXFP8 codes / scales of the eight GEMM weight operands (MXW_* below)
    size_t mxq[8], mxs[8];
};

// the frozen operand of each of a block's eight GEMMs
enum { MXW_QKV = 0, MXW_O, MXW_FC, MXW_PR, MXW_QKVT, MXW_OT, MXW_FCT, MXW_PRT };

}  // namespace

struct slora_ctx {
    slora_config cfg;
    int d, H, dff, L, r, S, maxT;
    float s;
    uint32_t mask;
    int n_qkv, qkv_idx[3], nz_qkv, k2_qkv, k2p_qkv;   // adapters among q,k,v and their slot in the fused operands
    std::vector<std::array<const bf16 *, SLORA_NFROZEN>> frozen;
    std::vector<std::array<AdapterBind, SLORA_NPROJ>> adapters;
    std::vector<BlockWs> bw;
    // transients
    size_t t_u, t_u2, t_g, t_df, t_du2, t_do, t_dqkv, t_du, t_ps, t_delta, t_part;
    size_t t_dh32[2], t_dh16[2];
    bool mx;                                    // frozen products in MXFP8 (SLORA_DTYPE_MXFP8)
    size_t t_xq, t_xs;                          // codes / scales of the activation operand of the current GEMM
    size_t t_qa, t_qas, t_qb, t_qbs;            // codes / scales written by producers: [T,d] (LayerNorm outputs and
                                                // gradients), [T,dff] (GELU output, its gradient)
    size_t shadow_begin, shadow_end, cast_tab, sgd_tab;
    std::vector<CastDesc> h_cast;
    std::vector<SgdDesc> h_sgd;
    size_t need;
    char *ws;
    size_t ws_bytes;
    bool prepared, shadows_dirty;
    int state;                                  // 0 idle, 1 forward done, 2 backward done
    int K, n_seq, T;
    int row_end[SLORA_MAX_CLIENTS];
};

namespace {

void proj_shape(const slora_ctx *c, int p, int &n_in, int &n_out)
{
    n_in = (p == SLORA_PROJ_PR) ? c->dff : c->d;
    n_out = (p == SLORA_PROJ_FC) ? c->dff : c->d;
}
inline bool adapted(const slora_ctx *c, int p) { return (c->mask >> p) & 1u; }

void plan_workspace(slora_ctx *c)
{
    const size_t T = (size_t)c->maxT, d = c->d, dff = c->dff, H = c->H;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = al256(off + bytes); return o; };
    c->bw.resize(c->L);
    for (int l = 0; l < c->L; ++l) {
        BlockWs &b = c->bw[l];
        b.WqkvT = take(2 * d * 3 * d);
        b.WoT = take(2 * d * d);
        b.WfcT = take(2 * d * dff);
        b.WprT = take(2 * dff * d);
        if (c->mx) {
            // [N,K] of each operand: Wqkv [3d,d], Wo [d,d], Wfc [dff,d], Wpr [d,dff] and their transposes
            const size_t nk[8][2] = {{3 * d, d}, {d, d}, {dff, d}, {d, dff}, {d, 3 * d}, {d, d}, {d, dff}, {dff, d}};
            for (int i = 0; i < 8; ++i) {
                b.mxq[i] = take(nk[i][0] * nk[i][1]);
                b.mxs[i] = take(nk[i][0] * nk[i][1] / 32);
            }
        }
    }
    c->shadow_begin = off;
    for (int l = 0; l < c->L; ++l) {
        BlockWs &b = c->bw[l];
        for (int p = 0; p < SLORA_NPROJ; ++p) {
            b.fz[p] = b.ft[p] = b.bz[p] = b.bt[p] = 0;
            if (!adapted(c, p)) continue;
            int n_in, n_out;
            proj_shape(c, p, n_in, n_out);
            b.fz[p] = take(2 * 16 * (size_t)n_in);
            b.ft[p] = take(2 * (size_t)n_out * 32);
            if (p >= SLORA_PROJ_O) {
                b.bz[p] = take(2 * 16 * (size_t)n_out);
                b.bt[p] = take(2 * (size_t)n_in * 32);
            }
        }
        b.bz_qkv = b.bt_qkv = 0;
        if (c->n_qkv) {
            b.bz_qkv = take(2 * (size_t)c->nz_qkv * 3 * d);
            b.bt_qkv = take(2 * d * (size_t)c->k2p_qkv);
        }
    }
    c->shadow_end = off;
    c->cast_tab = take(sizeof(CastDesc) * (size_t)c->L * SLORA_NPROJ * 4);
    c->sgd_tab = take(sizeof(SgdDesc) * (size_t)c->L * SLORA_NPROJ * 2);
    const bool qkv_ad = c->n_qkv > 0;
    for (int l = 0; l < c->L; ++l) {
        BlockWs &b = c->bw[l];
        b.h_in = take(4 * T * d);
        b.stats1 = take(8 * T);
        b.qkv = take(2 * T * 3 * d);
        b.o = take(2 * T * d);
        b.o_lo = take(2 * T * d);
        b.lse = take(4 * T * H);
        b.h_mid = take(4 * T * d);
        b.stats2 = take(8 * T);
        b.f = take(2 * T * dff);
        b.u = qkv_ad ? take(2 * T * d) : 0;
        b.u2 = adapted(c, SLORA_PROJ_FC) ? take(2 * T * d) : 0;
        b.g = adapted(c, SLORA_PROJ_PR) ? take(2 * T * dff) : 0;
        for (int p = 0; p < SLORA_NPROJ; ++p) b.zs[p] = adapted(c, p) ? take(2 * T * SL_RP) : 0;
    }
    c->t_u = take(2 * T * d);
    c->t_u2 = take(2 * T * d);
    c->t_g = take(2 * T * dff);
    c->t_df = take(2 * T * dff);
    c->t_du2 = take(2 * T * d);
    c->t_do = take(2 * T * d);
    c->t_dqkv = take(2 * T * 3 * d);
    c->t_du = take(2 * T * d);
    c->t_ps = take(2 * T * 64);
    c->t_delta = take(4 * T * H);
    // adapter-gradient partial sums: the five jobs of the q|k|v group (width d each), or the dA + dB pair of
    // one of the other projections (widths d and d_ff at most)
    {
        const size_t fd = lora_grad_partial_floats(c->maxT, (int)d), ff = lora_grad_partial_floats(c->maxT, (int)dff);
        c->t_part = take(4 * (5 * fd > fd + ff ? 5 * fd : fd + ff));
    }
    c->t_xq = c->t_xs = c->t_qa = c->t_qas = c->t_qb = c->t_qbs = 0;
    if (c->mx) {
        const size_t kmax = dff > 3 * d ? dff : 3 * d;
        c->t_xq = take(T * kmax);
        c->t_xs = take(T * kmax / 32);
        c->t_qa = take(T * d);
        c->t_qas = take(T * d / 32);
        c->t_qb = take(T * dff);
        c->t_qbs = take(T * dff / 32);
    }
    for (int i = 0; i < 2; ++i) {
        c->t_dh32[i] = take(4 * T * d);
        c->t_dh16[i] = take(2 * T * d);
    }
    c->need = off;
}

template <class Tp>
inline Tp *at(const slora_ctx *c, size_t off) { return (Tp *)(c->ws + off); }

void build_tables(slora_ctx *c)
{
    c->h_cast.clear();
    c->h_sgd.clear();
    for (int l = 0; l < c->L; ++l) {
        const BlockWs &b = c->bw[l];
        for (int p = 0; p < SLORA_NPROJ; ++p) {
            if (!adapted(c, p)) continue;
            const AdapterBind &ab = c->adapters[l][p];
            int n_in, n_out;
            proj_shape(c, p, n_in, n_out);
            // forward operands
            c->h_cast.push_back({ab.A, at<bf16>(c, b.fz[p]), c->r, n_in, 0, n_in, 16, n_in});
            c->h_cast.push_back({ab.B, at<bf16>(c, b.ft[p]), n_out, c->r, 0, 32, n_out, 32});
            // backward operands
            if (p >= SLORA_PROJ_O) {
                c->h_cast.push_back({ab.B, at<bf16>(c, b.bz[p]), n_out, c->r, 1, n_out, 16, n_out});
                c->h_cast.push_back({ab.A, at<bf16>(c, b.bt[p]), c->r, n_in, 1, 32, n_in, 32});
            } else {
                const int idx = c->qkv_idx[p];
                // rows 16 idx .. of the block-diagonal B^T, columns p d ..; other entries stay zero
                c->h_cast.push_back({ab.B, at<bf16>(c, b.bz_qkv) + (size_t)16 * idx * 3 * c->d + (size_t)p * c->d,
                                     n_out, c->r, 1, 3 * c->d, SL_RP, n_out});
                c->h_cast.push_back({ab.A, at<bf16>(c, b.bt_qkv) + 16 * idx, c->r, n_in, 1, c->k2p_qkv, n_in, SL_RP});
            }
            c->h_sgd.push_back({ab.A, ab.dA, c->r * n_in, 0});
            c->h_sgd.push_back({ab.B, ab.dB, n_out * c->r, 0});
        }
    }
}

int refresh_shadows(slora_ctx *c, hipStream_t st)
{
    if (c->h_cast.empty()) return 0;
    const int max_elems = 32 * (c->dff > c->d ? c->dff : c->d);
    int gx = (max_elems + 255) / 256;
    if (gx > 64) gx = 64;
    hipLaunchKernelGGL(cast_table_kernel, dim3(gx, (unsigned)c->h_cast.size()), dim3(256), 0, st,
                       at<CastDesc>(c, c->cast_tab));
    SL_CHECK_LAUNCH("cast_table");
    return 0;
}

int upload_table(void *dst, const void *src, size_t bytes, hipStream_t st)
{
    static_assert(sizeof(CastDesc) % 4 == 0 && sizeof(SgdDesc) % 4 == 0, "tables are copied word by word");
    for (size_t off = 0; off < bytes; off += sizeof(TableChunk)) {
        const size_t n = bytes - off < sizeof(TableChunk) ? bytes - off : sizeof(TableChunk);
        TableChunk ch;
        memcpy(ch.w, (const char *)src + off, n);
        hipLaunchKernelGGL(table_upload_kernel, dim3(1), dim3(256), 0, st, (uint32_t *)((char *)dst + off), ch,
                           (int)(n / 4));
        SL_CHECK_LAUNCH("table_upload");
    }
    return 0;
}

int prepare(slora_ctx *c, hipStream_t st)
{
    int rc;
    build_tables(c);
    if (!c->h_cast.empty()) {
        if ((rc = upload_table(at<void>(c, c->cast_tab), c->h_cast.data(), sizeof(CastDesc) * c->h_cast.size(), st)))
            return rc;
        if ((rc = upload_table(at<void>(c, c->sgd_tab), c->h_sgd.data(), sizeof(SgdDesc) * c->h_sgd.size(), st)))
            return rc;
        if ((rc = launch_fill_zero(at<void>(c, c->shadow_begin), c->shadow_end - c->shadow_begin, st))) return rc;
    }
    for (int l = 0; l < c->L; ++l) {
        const BlockWs &b = c->bw[l];
        const auto &fz = c->frozen[l];
        if ((rc = launch_transpose_bf16(fz[SLORA_WQKV], 3 * c->d, c->d, at<bf16>(c, b.WqkvT), st))) return rc;
        if ((rc = launch_transpose_bf16(fz[SLORA_WO], c->d, c->d, at<bf16>(c, b.WoT), st))) return rc;
        if ((rc = launch_transpose_bf16(fz[SLORA_WFC], c->dff, c->d, at<bf16>(c, b.WfcT), st))) return rc;
        if ((rc = launch_transpose_bf16(fz[SLORA_WPR], c->d, c->dff, at<bf16>(c, b.WprT), st))) return rc;
        if (c->mx) {
            const int d = c->d, dff = c->dff;
            const bf16 *w[8] = {fz[SLORA_WQKV], fz[SLORA_WO], fz[SLORA_WFC], fz[SLORA_WPR], at<bf16>(c, b.WqkvT),
                                at<bf16>(c, b.WoT), at<bf16>(c, b.WfcT), at<bf16>(c, b.WprT)};
            const int nk[8][2] = {{3 * d, d}, {d, d}, {dff, d}, {d, dff}, {d, 3 * d}, {d, d}, {d, dff}, {dff, d}};
            for (int i = 0; i < 8; ++i)
                if ((rc = launch_mx_quantize(w[i], nk[i][1], nk[i][0], nk[i][1], at<unsigned char>(c, b.mxq[i]),
                                             at<unsigned char>(c, b.mxs[i]), st)))
                    return rc;
        }
    }
    c->prepared = true;
    c->shadows_dirty = true;
    return 0;
}

int check_bound(const slora_ctx *c)
{
    if (!c->ws) return SLORA_ESTATE;
    for (int l = 0; l < c->L; ++l) {
        for (int w = 0; w < SLORA_NFROZEN; ++w)
            if (!c->frozen[l][w]) return SLORA_ESTATE;
        for (int p = 0; p < SLORA_NPROJ; ++p)
            if (adapted(c, p)) {
                const AdapterBind &ab = c->adapters[l][p];
                if (!ab.A || !ab.B || !ab.dA || !ab.dB) return SLORA_ESTATE;
            }
    }
    return 0;
}

// one frozen linear with optional adapter: fills the common GemmArgs fields
GemmArgs gemm_base(const bf16 *X, int ldx, const bf16 *W, int M, int N, int K, const bf16 *bias, float s)
{
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.X = X; a.ldx = ldx; a.W = W; a.ldw = K; a.M = M; a.N = N; a.K = K;
    a.nseg = 1; a.seg_n = N; a.bias = bias; a.ldo = N; a.zscale = s; a.K2 = 16; a.ldz = K; a.ldt = 32;
    return a;
}

// compressed mode: point a GEMM at the packed form of its frozen operand and at the conversion scratch
// `ready`: 0 = convert X into the scratch; 1 = its producer wrote the codes into the [T,d] buffer; 2 = into the
// [T,dff] buffer
inline void set_mx(const slora_ctx *c, int l, int which, GemmArgs &a, MxOperands &m, int ready = 0)
{
    if (!c->mx) return;
    m.wq = at<unsigned char>(c, c->bw[l].mxq[which]);
    m.ws = at<unsigned char>(c, c->bw[l].mxs[which]);
    m.xq = at<unsigned char>(c, ready == 1 ? c->t_qa : ready == 2 ? c->t_qb : c->t_xq);
    m.xs = at<unsigned char>(c, ready == 1 ? c->t_qas : ready == 2 ? c->t_qbs : c->t_xs);
    m.x_ready = ready != 0;
    a.mx = &m;
}
// the producers' code outputs (null outside the compressed mode)
inline unsigned char *qa(const slora_ctx *c) { return c->mx ? at<unsigned char>(c, c->t_qa) : nullptr; }
inline unsigned char *qas(const slora_ctx *c) { return c->mx ? at<unsigned char>(c, c->t_qas) : nullptr; }

int lora_grads(slora_ctx *c, int l, int p, const bf16 *x, int ldx, const bf16 *dy, int ldy_, const bf16 *ps, int ldps,
               hipStream_t st)
{
    int n_in, n_out, rc;
    proj_shape(c, p, n_in, n_out);
    const AdapterBind &ab = c->adapters[l][p];
    float *part = at<float>(c, c->t_part);
    // dA [r,in] = ps^T x and dB [out,r] = dy^T zs, one launch for the two
    const LoraGradDesc jobs[2] = {
        {x, ps, part, ab.dA, nullptr, ldx, ldps, n_in, false, 1},
        {dy, at<bf16>(c, c->bw[l].zs[p]), part + lora_grad_partial_floats(c->maxT, n_in), ab.dB, nullptr, ldy_, SL_RP, n_out,
         false, 0}};
    return launch_lora_grad_jobs(jobs, 2, c->r, c->T, st);
}

}  // namespace

// =================================================================================================
extern "C" {

const char *slora_strerror(int code)
{
    switch (code) {
    case SLORA_OK: return "ok";
    case SLORA_EINVAL: return "invalid argument or unsupported configuration";
    case SLORA_ESTATE: return "call order violated or weights/adapters/workspace not bound";
    case SLORA_ENOSPC: return "workspace too small";
    case SLORA_EHIP: return "HIP call failed";
    case SLORA_EZERO: return "negative sample count or zero total";
    }
    return "unknown error";
}

const char *slora_last_hip_error(void) { return g_hip_err; }

int slora_prof_enable(int kinds)
{
    if (kinds < 0 || (kinds >> PK_COUNT)) return SLORA_EINVAL;
    return prof_enable((unsigned)kinds) ? SLORA_EHIP : SLORA_OK;
}

int slora_prof_read_kind(int kind, double *h_ms, double *h_work, int *h_launches)
{
    if (kind < 0 || kind >= PK_COUNT) return SLORA_EINVAL;
    return prof_read(kind, h_ms, h_work, h_launches) ? SLORA_EHIP : SLORA_OK;
}

int slora_prof_read_clock(double *h_mhz, int *h_samples)
{
    return prof_read_clock(h_mhz, h_samples) ? SLORA_EHIP : SLORA_OK;
}

int slora_prof_read(double *h_gemm_ms, double *h_gemm_flop, int *h_launches)
{
    return slora_prof_read_kind(SLORA_PROF_GEMM, h_gemm_ms, h_gemm_flop, h_launches);
}

int slora_create(const slora_config *cfg, slora_ctx **out)
{
    if (!cfg || !out) return SLORA_EINVAL;
    *out = nullptr;
    if (cfg->dtype != SLORA_DTYPE_BF16 && cfg->dtype != SLORA_DTYPE_MXFP8) return SLORA_EINVAL;
    if (cfg->dtype == SLORA_DTYPE_MXFP8 && ((cfg->d_model % 128) || (cfg->d_ff % 128))) return SLORA_EINVAL;
    if (cfg->d_model <= 0 || cfg->n_head <= 0 || cfg->d_model % 64 || cfg->d_model != cfg->n_head * 64)
        return SLORA_EINVAL;
    if (cfg->d_model > 2048) return SLORA_EINVAL;
    if (cfg->d_ff <= 0 || cfg->d_ff % 64) return SLORA_EINVAL;
    if (cfg->n_blocks <= 0 || cfg->n_blocks > 1024) return SLORA_EINVAL;
    if (cfg->lora_r < 1 || cfg->lora_r > SLORA_MAX_RANK) return SLORA_EINVAL;
    if (cfg->lora_mask >> SLORA_NPROJ) return SLORA_EINVAL;
    if (!(cfg->ln_eps > 0.f) || !(cfg->lora_alpha == cfg->lora_alpha)) return SLORA_EINVAL;
    if (cfg->max_seqs <= 0 || cfg->seq_len <= 0 || cfg->seq_len % 64) return SLORA_EINVAL;
    if ((long long)cfg->max_seqs * cfg->seq_len > (1ll << 24)) return SLORA_EINVAL;
    {   // 32-bit byte offsets into the widest GEMM operand ([T, 3 d_model] or [T, d_ff], bf16)
        const long long wide = 3ll * cfg->d_model > cfg->d_ff ? 3ll * cfg->d_model : cfg->d_ff;
        if ((long long)cfg->max_seqs * cfg->seq_len * wide >= (1ll << 31)) return SLORA_EINVAL;
    }
    slora_ctx *c = new (std::nothrow) slora_ctx();
    if (!c) return SLORA_EINVAL;
    c->cfg = *cfg;
    c->d = cfg->d_model; c->H = cfg->n_head; c->dff = cfg->d_ff; c->L = cfg->n_blocks; c->r = cfg->lora_r;
    c->S = cfg->seq_len; c->maxT = cfg->max_seqs * cfg->seq_len;
    c->s = cfg->lora_alpha / (float)cfg->lora_r;
    c->mask = cfg->lora_mask;
    c->mx = cfg->dtype == SLORA_DTYPE_MXFP8;
    c->n_qkv = 0;
    for (int p = 0; p < 3; ++p) c->qkv_idx[p] = adapted(c, p) ? c->n_qkv++ : -1;
    c->nz_qkv = 16 * c->n_qkv;
    c->k2_qkv = 16 * c->n_qkv;
    c->k2p_qkv = (c->k2_qkv + 31) / 32 * 32;
    c->frozen.assign(c->L, {});
    c->adapters.assign(c->L, {});
    c->ws = nullptr; c->ws_bytes = 0;
    c->prepared = false; c->shadows_dirty = true; c->state = 0;
    c->K = 0; c->n_seq = 0; c->T = 0;
    plan_workspace(c);
    *out = c;
    return SLORA_OK;
}

int slora_destroy(slora_ctx *ctx)
{
    if (!ctx) return SLORA_EINVAL;
    delete ctx;
    return SLORA_OK;
}

size_t slora_workspace_bytes(const slora_ctx *ctx) { return ctx ? ctx->need : 0; }

int slora_bind_workspace(slora_ctx *ctx, void *ws, size_t bytes)
{
    if (!ctx || !ws) return SLORA_EINVAL;
    if (((uintptr_t)ws) & 255) return SLORA_EINVAL;
    if (bytes < ctx->need) return SLORA_ENOSPC;
    ctx->ws = (char *)ws;
    ctx->ws_bytes = bytes;
    ctx->prepared = false;
    ctx->state = 0;
    return SLORA_OK;
}

int slora_bind_frozen(slora_ctx *ctx, int block, int which, const void *w)
{
    if (!ctx || !w || block < 0 || block >= ctx->L || which < 0 || which >= SLORA_NFROZEN) return SLORA_EINVAL;
    if (((uintptr_t)w) & 15) return SLORA_EINVAL;
    ctx->frozen[block][which] = (const bf16 *)w;
    ctx->prepared = false;
    ctx->state = 0;
    return SLORA_OK;
}

int slora_bind_adapter(slora_ctx *ctx, int block, int proj, float *A, float *B, float *dA, float *dB)
{
    if (!ctx || !A || !B || !dA || !dB || block < 0 || block >= ctx->L || proj < 0 || proj >= SLORA_NPROJ)
        return SLORA_EINVAL;
    if (!adapted(ctx, proj)) return SLORA_EINVAL;
    if ((((uintptr_t)A) | ((uintptr_t)B) | ((uintptr_t)dA) | ((uintptr_t)dB)) & 15) return SLORA_EINVAL;
    ctx->adapters[block][proj] = {A, B, dA, dB};
    ctx->prepared = false;
    ctx->state = 0;
    return SLORA_OK;
}

// Forward through the blocks of a context.  The input of block 0 is either the concatenation of the
// client buffers in `tab` (server side) or the embedding lookup `emb` (client side).
static int stack_fwd(slora_ctx *c, const ClientTable *tabp, const EmbedSrc *emb, void *y, hipStream_t st)
{
    int rc;
    if (!c->prepared && (rc = prepare(c, st))) return rc;
    if (c->shadows_dirty) {
        if ((rc = refresh_shadows(c, st))) return rc;
        c->shadows_dirty = false;
    }
    c->state = 0;
    const int T = c->T, d = c->d, dff = c->dff;
    for (int l = 0; l < c->L; ++l) {
        const BlockWs &b = c->bw[l];
        const auto &fz = c->frozen[l];
        float *h_in = at<float>(c, b.h_in);
        // the compressed context reads u, u2 and g as codes; their bf16 copies exist only where an adapter reads them
        bf16 *u = (c->mx && !b.u) ? nullptr : at<bf16>(c, b.u ? b.u : c->t_u);
        // LN1 (block 0 gathers the clients' activations: S = [s_1; ...; s_N], or looks the embedding up)
        if ((rc = launch_ln_fwd(l == 0 ? nullptr : h_in, l == 0 ? tabp : nullptr, h_in, fz[SLORA_LN1_G],
                                fz[SLORA_LN1_B], c->cfg.ln_eps, u, at<float>(c, b.stats1), T, d, st,
                                l == 0 ? emb : nullptr, qa(c), qas(c))))
            return rc;
        // q | k | v = u Wqkv^T + b (+ adapters)
        {
            GemmArgs a = gemm_base(u, d, fz[SLORA_WQKV], T, 3 * d, d, fz[SLORA_BQKV], c->s);
            a.nseg = 3; a.seg_n = d; a.out0 = at<bf16>(c, b.qkv); a.ldo = 3 * d;
            for (int p = 0; p < 3; ++p)
                if (adapted(c, p)) {
                    a.zmat[p] = at<bf16>(c, b.fz[p]); a.tmat[p] = at<bf16>(c, b.ft[p]);
                    a.zspill[p] = at<bf16>(c, b.zs[p]);
                }
            MxOperands mxo;
            set_mx(c, l, MXW_QKV, a, mxo, 1);
            if ((rc = launch_gemm(a, EPI_STORE, c->n_qkv ? 16 : 0, st))) return rc;
        }
        if ((rc = launch_attn_fwd(at<bf16>(c, b.qkv), at<bf16>(c, b.o), at<bf16>(c, b.o_lo), at<float>(c, b.lse), c->n_seq,
                                  c->S, c->H,
                                  st)))
            return rc;
        // h' = h + o Wo^T + bo (+ adapter)
        {
            GemmArgs a = gemm_base(at<bf16>(c, b.o), d, fz[SLORA_WO], T, d, d, fz[SLORA_BO], c->s);
            a.aux = h_in; a.out0 = at<float>(c, b.h_mid);
            const bool ad = adapted(c, SLORA_PROJ_O);
            if (ad) {
                a.zmat[0] = at<bf16>(c, b.fz[SLORA_PROJ_O]); a.tmat[0] = at<bf16>(c, b.ft[SLORA_PROJ_O]);
                a.zspill[0] = at<bf16>(c, b.zs[SLORA_PROJ_O]);
            }
            MxOperands mxo;
            set_mx(c, l, MXW_O, a, mxo);
            if ((rc = launch_gemm(a, EPI_RESID, ad ? 16 : 0, st))) return rc;
        }
        bf16 *u2 = (c->mx && !b.u2) ? nullptr : at<bf16>(c, b.u2 ? b.u2 : c->t_u2);
        if ((rc = launch_ln_fwd(at<float>(c, b.h_mid), nullptr, nullptr, fz[SLORA_LN2_G], fz[SLORA_LN2_B],
                                c->cfg.ln_eps, u2, at<float>(c, b.stats2), T, d, st, nullptr, qa(c), qas(c))))
            return rc;
        // f = u2 Wfc^T + bfc (+ adapter); g = GELU(f); the slot `f` keeps GELU'(f), all the backward needs
        bf16 *g = (c->mx && !b.g) ? nullptr : at<bf16>(c, b.g ? b.g : c->t_g);
        {
            GemmArgs a = gemm_base(u2, d, fz[SLORA_WFC], T, dff, d, fz[SLORA_BFC], c->s);
            a.out0 = at<bf16>(c, b.f); a.out1 = g;
            const bool ad = adapted(c, SLORA_PROJ_FC);
            if (ad) {
                a.zmat[0] = at<bf16>(c, b.fz[SLORA_PROJ_FC]); a.tmat[0] = at<bf16>(c, b.ft[SLORA_PROJ_FC]);
                a.zspill[0] = at<bf16>(c, b.zs[SLORA_PROJ_FC]);
            }
            MxOperands mxo;
            set_mx(c, l, MXW_FC, a, mxo, 1);
            if (c->mx) { a.oq = at<unsigned char>(c, c->t_qb); a.os = at<unsigned char>(c, c->t_qbs); }   // codes of g
            if ((rc = launch_gemm(a, EPI_GELU, ad ? 16 : 0, st))) return rc;
        }
        // h'' = h' + g Wpr^T + bpr (+ adapter): next block's input, or y for the last block
        {
            GemmArgs a = gemm_base(g, dff, fz[SLORA_WPR], T, d, dff, fz[SLORA_BPR], c->s);
            a.aux = at<float>(c, b.h_mid);
            if (l + 1 < c->L) a.out0 = at<float>(c, c->bw[l + 1].h_in);
            else a.out1 = y;
            const bool ad = adapted(c, SLORA_PROJ_PR);
            if (ad) {
                a.zmat[0] = at<bf16>(c, b.fz[SLORA_PROJ_PR]); a.tmat[0] = at<bf16>(c, b.ft[SLORA_PROJ_PR]);
                a.zspill[0] = at<bf16>(c, b.zs[SLORA_PROJ_PR]);
            }
            MxOperands mxo;
            set_mx(c, l, MXW_PR, a, mxo, 2);
            if ((rc = launch_gemm(a, EPI_RESID, ad ? 16 : 0, st))) return rc;
        }
    }
    c->state = 1;
    return SLORA_OK;
}

// shared by the bf16 and the compressed form of the server forward: `h_scales` null = bf16 client buffers
static int server_fwd_common(slora_ctx *c, int K, const void *const *h_x_clients, const void *const *h_scales,
                             const int32_t *h_batch, void *y, void *stream)
{
    if (!c || !h_x_clients || !h_batch || !y) return SLORA_EINVAL;
    if (K <= 0 || K > SLORA_MAX_CLIENTS) return SLORA_EINVAL;
    long long nseq = 0;
    for (int i = 0; i < K; ++i) {
        if (!h_x_clients[i] || h_batch[i] <= 0) return SLORA_EINVAL;
        if (((uintptr_t)h_x_clients[i]) & 7) return SLORA_EINVAL;
        if (h_scales && !h_scales[i]) return SLORA_EINVAL;
        nseq += h_batch[i];
    }
    if (nseq > c->cfg.max_seqs) return SLORA_EINVAL;
    if (((uintptr_t)y) & 7) return SLORA_EINVAL;
    int rc;
    if ((rc = check_bound(c))) return rc;
    c->K = K; c->n_seq = (int)nseq; c->T = c->n_seq * c->S;
    ClientTable tab;
    tab.K = K;
    tab.mx = h_scales ? 1 : 0;
    int rows = 0;
    for (int i = 0; i < K; ++i) {
        rows += h_batch[i] * c->S;
        tab.ptr[i] = (void *)h_x_clients[i];
        tab.aux[i] = h_scales ? (void *)h_scales[i] : nullptr;
        tab.row_end[i] = rows;
        c->row_end[i] = rows;
    }
    return stack_fwd(c, &tab, nullptr, y, (hipStream_t)stream);
}

int slora_server_fwd(slora_ctx *c, int K, const void *const *h_x_clients, const int32_t *h_batch, void *y,
                     void *stream)
{
    return server_fwd_common(c, K, h_x_clients, nullptr, h_batch, y, stream);
}

int slora_server_fwd_mx(slora_ctx *c, int K, const void *const *h_xq_clients, const void *const *h_xs_clients,
                        const int32_t *h_batch, void *y, void *stream)
{
    if (!h_xs_clients) return SLORA_EINVAL;
    return server_fwd_common(c, K, h_xq_clients, h_xs_clients, h_batch, y, stream);
}

int slora_client_fwd(slora_ctx *c, int32_t batch, const int32_t *tokens, int32_t vocab, const void *wte,
                     const void *wpe, void *act, void *stream)
{
    if (!c || !tokens || !wte || !wpe || !act) return SLORA_EINVAL;
    if (batch <= 0 || batch > c->cfg.max_seqs || vocab <= 0) return SLORA_EINVAL;
    if ((((uintptr_t)wte) | ((uintptr_t)wpe) | ((uintptr_t)act)) & 7) return SLORA_EINVAL;
    int rc;
    if ((rc = check_bound(c))) return rc;
    c->K = 1; c->n_seq = batch; c->T = batch * c->S;
    c->row_end[0] = c->T;
    EmbedSrc emb = {tokens, (const bf16 *)wte, (const bf16 *)wpe, c->S, vocab};
    return stack_fwd(c, nullptr, &emb, act, (hipStream_t)stream);
}

// Backward through the blocks of a context.  `tabp` = where the activation gradients of block 0's input
// go (server side: the clients' buffers); null = nobody needs them (client side: the embedding is frozen).
static int stack_bwd(slora_ctx *c, const void *dy, const ClientTable *tabp, hipStream_t st)
{
    const int T = c->T, d = c->d, dff = c->dff;
    int rc;
    // gradient of the residual stream entering the block from above: fp32 (+ bf16 GEMM operand)
    const float *dh2_32 = nullptr;
    const bf16 *dh2_16 = (const bf16 *)dy;
    // compressed mode: the gradient entering a block is also held as codes (written by the LayerNorm backward
    // of the block above; for the caller's dY by one conversion pass here)
    if (c->mx && (rc = launch_mx_quantize(dh2_16, d, T, d, qa(c), qas(c), st))) return rc;
    for (int l = c->L - 1; l >= 0; --l) {
        const BlockWs &b = c->bw[l];
        const auto &fz = c->frozen[l];
        // compressed mode: df, dh' and the gradient handed down travel as codes; the bf16 copies are written
        // only where an adapter's products read them
        bf16 *df = (c->mx && !adapted(c, SLORA_PROJ_FC)) ? nullptr : at<bf16>(c, c->t_df);
        bf16 *ps = at<bf16>(c, c->t_ps);
        // dg = dh'' Wpr (+ adapter);  df = dg * GELU'(f)
        {
            GemmArgs a = gemm_base(dh2_16, d, at<bf16>(c, b.WprT), T, dff, d, nullptr, c->s);
            a.aux = at<bf16>(c, b.f); a.out0 = df;
            const bool ad = adapted(c, SLORA_PROJ_PR);
            if (ad) {
                a.zmat[0] = at<bf16>(c, b.bz[SLORA_PROJ_PR]); a.tmat[0] = at<bf16>(c, b.bt[SLORA_PROJ_PR]);
                a.zspill[0] = ps;
            }
            MxOperands mxo;
            set_mx(c, l, MXW_PRT, a, mxo, 1);
            if (c->mx) { a.oq = at<unsigned char>(c, c->t_qb); a.os = at<unsigned char>(c, c->t_qbs); }   // codes of df
            if ((rc = launch_gemm(a, EPI_DGELU, ad ? 16 : 0, st))) return rc;
            if (ad && (rc = lora_grads(c, l, SLORA_PROJ_PR, at<bf16>(c, b.g), dff, dh2_16, d, ps, SL_RP, st)))
                return rc;
        }
        // du2 = df Wfc (+ adapter)
        bf16 *du2 = at<bf16>(c, c->t_du2);
        {
            GemmArgs a = gemm_base(df, dff, at<bf16>(c, b.WfcT), T, d, dff, nullptr, c->s);
            a.out0 = du2;
            const bool ad = adapted(c, SLORA_PROJ_FC);
            if (ad) {
                a.zmat[0] = at<bf16>(c, b.bz[SLORA_PROJ_FC]); a.tmat[0] = at<bf16>(c, b.bt[SLORA_PROJ_FC]);
                a.zspill[0] = ps;
            }
            MxOperands mxo;
            set_mx(c, l, MXW_FCT, a, mxo, 2);
            if ((rc = launch_gemm(a, EPI_STORE, ad ? 16 : 0, st))) return rc;
            if (ad && (rc = lora_grads(c, l, SLORA_PROJ_FC, at<bf16>(c, b.u2), d, df, dff, ps, SL_RP, st))) return rc;
        }
        // dh' = dh'' + LN2^T(du2)
        float *dh1_32 = at<float>(c, c->t_dh32[1]);
        bf16 *dh1_16 = (c->mx && !adapted(c, SLORA_PROJ_O)) ? nullptr : at<bf16>(c, c->t_dh16[1]);
        if ((rc = launch_ln_bwd(du2, at<float>(c, b.h_mid), at<float>(c, b.stats2), fz[SLORA_LN2_G], dh2_32,
                                dh2_32 ? nullptr : dh2_16, dh1_32, dh1_16, nullptr, T, d, st, qa(c), qas(c))))
            return rc;
        // do = dh' Wo (+ adapter)
        bf16 *dob = at<bf16>(c, c->t_do);
        bool gemm_delta = false;
        {
            GemmArgs a = gemm_base(dh1_16, d, at<bf16>(c, b.WoT), T, d, d, nullptr, c->s);
            a.out0 = dob;
            const bool ad = adapted(c, SLORA_PROJ_O);
            if (ad) {
                a.zmat[0] = at<bf16>(c, b.bz[SLORA_PROJ_O]); a.tmat[0] = at<bf16>(c, b.bt[SLORA_PROJ_O]);
                a.zspill[0] = ps;
            }
            MxOperands mxo;
            set_mx(c, l, MXW_OT, a, mxo, 1);
            // where this product has no adapter branch (the 4-wave kernel, or the MXFP8 one) and the fused attention
            // backward follows, the epilogue also forms delta = rowsum(dO * O) per head, [T, H]
            gemm_delta = !ad && attn_bwd_takes_delta(c->S);
            if (gemm_delta) {
                a.dl_o = at<bf16>(c, b.o); a.dl_lo = at<bf16>(c, b.o_lo); a.dl_out = at<float>(c, c->t_delta);
            }
            if ((rc = launch_gemm(a, gemm_delta ? EPI_STORE_DELTA : EPI_STORE, ad ? 16 : 0, st))) return rc;
            if (ad && (rc = lora_grads(c, l, SLORA_PROJ_O, at<bf16>(c, b.o), d, dh1_16, d, ps, SL_RP, st))) return rc;
        }
        // attention backward
        bf16 *dqkv = at<bf16>(c, c->t_dqkv);
        if ((rc = launch_attn_bwd(at<bf16>(c, b.qkv), at<bf16>(c, b.o), at<bf16>(c, b.o_lo), dob, at<float>(c, b.lse),
                                  at<float>(c, c->t_delta), dqkv, c->n_seq, c->S, c->H, st, gemm_delta)))
            return rc;
        // du = [dq dk dv] Wqkv (+ adapters): one GEMM with contraction 3d
        bf16 *dub = at<bf16>(c, c->t_du);
        {
            GemmArgs a = gemm_base(dqkv, 3 * d, at<bf16>(c, b.WqkvT), T, d, 3 * d, nullptr, c->s);
            a.out0 = dub;
            if (c->n_qkv) {
                a.zmat[0] = at<bf16>(c, b.bz_qkv); a.tmat[0] = at<bf16>(c, b.bt_qkv); a.zspill[0] = ps;
                a.K2 = c->k2_qkv; a.ldt = c->k2p_qkv;
            }
            MxOperands mxo;
            set_mx(c, l, MXW_QKVT, a, mxo);
            if ((rc = launch_gemm(a, EPI_STORE, c->n_qkv ? c->nz_qkv : 0, st))) return rc;
            // dB per adapted projection (its own slice of dq|dk|dv against its own zs); dA for the adapters
            // two at a time: they share the operand u, and their rank-space gradients sit side by side in ps.
            // All of them go out as one launch (each with partial-sum scratch of its own).
            if (c->n_qkv) {
                const size_t part_stride = lora_grad_partial_floats(c->maxT, d);
                float *part = at<float>(c, c->t_part);
                LoraGradDesc jobs[5];
                int nj = 0, slot_proj[3], nslot = 0;
                for (int p = 0; p < 3; ++p)
                    if (adapted(c, p)) {
                        slot_proj[c->qkv_idx[p]] = p;
                        ++nslot;
                        jobs[nj] = {dqkv + (size_t)p * d, at<bf16>(c, b.zs[p]), part + nj * part_stride,
                                    c->adapters[l][p].dB, nullptr, 3 * d, SL_RP, d, false, 0};
                        ++nj;
                    }
                for (int sl = 0; sl < nslot; sl += 2) {
                    const bool pair = sl + 1 < nslot;
                    jobs[nj] = {at<bf16>(c, b.u), ps + 16 * sl, part + nj * part_stride, c->adapters[l][slot_proj[sl]].dA,
                                pair ? c->adapters[l][slot_proj[sl + 1]].dA : nullptr, d, c->k2_qkv, d, pair, 1};
                    ++nj;
                }
                if ((rc = launch_lora_grad_jobs(jobs, nj, c->r, T, st))) return rc;
            }
        }
        // dh = dh' + LN1^T(du): next block's incoming gradient, or the clients' activation gradients
        float *nx32 = at<float>(c, c->t_dh32[0]);
        bf16 *nx16 = (c->mx && !adapted(c, SLORA_PROJ_PR)) ? nullptr : at<bf16>(c, c->t_dh16[0]);
        if (l > 0) {
            if ((rc = launch_ln_bwd(dub, at<float>(c, b.h_in), at<float>(c, b.stats1), fz[SLORA_LN1_G], dh1_32,
                                    nullptr, nx32, nx16, nullptr, T, d, st, qa(c), qas(c))))
                return rc;
            dh2_32 = nx32;
            dh2_16 = nx16;
        } else if (tabp) {
            if ((rc = launch_ln_bwd(dub, at<float>(c, b.h_in), at<float>(c, b.stats1), fz[SLORA_LN1_G], dh1_32,
                                    nullptr, nullptr, nullptr, tabp, T, d, st)))
                return rc;
        }
    }
    c->state = 2;
    return SLORA_OK;
}

static int server_bwd_common(slora_ctx *c, const void *dy, void *const *h_dx_clients, void *const *h_scales,
                             void *stream)
{
    if (!c || !dy || !h_dx_clients) return SLORA_EINVAL;
    if (c->state != 1) return SLORA_ESTATE;
    for (int i = 0; i < c->K; ++i) {
        if (!h_dx_clients[i] || (((uintptr_t)h_dx_clients[i]) & 7)) return SLORA_EINVAL;
        if (h_scales && !h_scales[i]) return SLORA_EINVAL;
    }
    if (((uintptr_t)dy) & 15) return SLORA_EINVAL;
    ClientTable tab;
    tab.K = c->K;
    tab.mx = h_scales ? 1 : 0;
    for (int i = 0; i < c->K; ++i) {
        tab.ptr[i] = h_dx_clients[i];
        tab.aux[i] = h_scales ? h_scales[i] : nullptr;
        tab.row_end[i] = c->row_end[i];
    }
    return stack_bwd(c, dy, &tab, (hipStream_t)stream);
}

int slora_server_bwd(slora_ctx *c, const void *dy, void *const *h_dx_clients, void *stream)
{
    return server_bwd_common(c, dy, h_dx_clients, nullptr, stream);
}

int slora_server_bwd_mx(slora_ctx *c, const void *dy, void *const *h_dxq_clients, void *const *h_dxs_clients,
                        void *stream)
{
    if (!h_dxs_clients) return SLORA_EINVAL;
    return server_bwd_common(c, dy, h_dxq_clients, h_dxs_clients, stream);
}

int slora_client_bwd(slora_ctx *c, const void *dact, void *stream)
{
    if (!c || !dact) return SLORA_EINVAL;
    if (c->state != 1) return SLORA_ESTATE;
    if (((uintptr_t)dact) & 15) return SLORA_EINVAL;
    return stack_bwd(c, dact, nullptr, (hipStream_t)stream);
}

int slora_adapters_changed(slora_ctx *c)
{
    if (!c) return SLORA_EINVAL;
    if (c->state == 1) return SLORA_ESTATE;      // between forward and backward the adapters must not move
    c->shadows_dirty = true;
    c->state = 0;
    return SLORA_OK;
}

int slora_adapter_step(slora_ctx *c, float lr, void *stream)
{
    if (!c) return SLORA_EINVAL;
    if (c->state != 2) return SLORA_ESTATE;
    if (!(lr == lr)) return SLORA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    if (!c->h_sgd.empty()) {
        int max_n = 0;
        for (const SgdDesc &d : c->h_sgd) max_n = d.n > max_n ? d.n : max_n;
        int gx = (max_n + 255) / 256;
        if (gx > 64) gx = 64;
        double n_par = 0.0;
        for (const SgdDesc &d : c->h_sgd) n_par += d.n;
        const bool rec = prof_begin(PK_SGD, st);
        hipLaunchKernelGGL(sgd_table_kernel, dim3(gx, (unsigned)c->h_sgd.size()), dim3(256), 0, st,
                           at<SgdDesc>(c, c->sgd_tab), lr);
        prof_end(rec, PK_SGD, 12.0 * n_par, st);     // parameter and gradient read, parameter written
        SL_CHECK_LAUNCH("sgd_table");
        int rc = refresh_shadows(c, st);
        if (rc) return rc;
    }
    c->shadows_dirty = false;
    c->state = 0;
    return SLORA_OK;
}

int slora_fedavg(int K, const float *const *h_client_params, const int64_t *h_sample_counts, size_t n, float *out,
                 void *stream)
{
    if (!h_client_params || !h_sample_counts || !out) return SLORA_EINVAL;
    if (K <= 0 || K > SLORA_MAX_CLIENTS) return SLORA_EINVAL;
    double tot = 0.0;
    for (int i = 0; i < K; ++i) {
        if (!h_client_params[i]) return SLORA_EINVAL;
        if (h_sample_counts[i] < 0) return SLORA_EZERO;
        tot += (double)h_sample_counts[i];
    }
    if (!(tot > 0.0)) return SLORA_EZERO;
    if (n == 0) return SLORA_OK;
    float w[SLORA_MAX_CLIENTS];
    for (int i = 0; i < K; ++i) w[i] = (float)((double)h_sample_counts[i] / tot);
    return launch_fedavg(K, h_client_params, w, n, out, (hipStream_t)stream);
}

int slora_adamw(size_t n, float *p, const float *g, float *m, float *v, float lr, float beta1, float beta2, float eps,
                float weight_decay, int32_t step, void *stream)
{
    if (!p || !g || !m || !v) return SLORA_EINVAL;
    if (step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps > 0.f) || !(lr == lr) ||
        !(weight_decay == weight_decay))
        return SLORA_EINVAL;
    const float decay = (float)(1.0 - (double)lr * (double)weight_decay);
    const float a = (float)((double)lr / (1.0 - pow((double)beta1, (double)step)));
    const float c = (float)(1.0 / sqrt(1.0 - pow((double)beta2, (double)step)));
    const float o1 = (float)(1.0 - (double)beta1), o2 = (float)(1.0 - (double)beta2);
    return launch_adamw(p, g, m, v, n, beta1, beta2, eps, decay, a, c, o1, o2, (hipStream_t)stream);
}

// ---- single layer -----------------------------------------------------------------------------
namespace {
struct LinWs { size_t A16, B16, B16T, A16T, zs, ps, WT, ytmp, part, total; };
LinWs lin_ws(int T, int n_in, int n_out)
{
    LinWs w;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = al256(off + bytes); return o; };
    w.A16 = take(2 * 16 * (size_t)n_in);
    w.B16 = take(2 * (size_t)n_out * 32);
    w.B16T = take(2 * 16 * (size_t)n_out);
    w.A16T = take(2 * (size_t)n_in * 32);
    w.zs = take(2 * (size_t)T * 16);
    w.ps = take(2 * (size_t)T * 16);
    w.WT = take(2 * (size_t)n_in * n_out);
    w.ytmp = take(2 * (size_t)T * n_out);
    w.part = take(4 * lora_grad_partial_floats(T, n_in > n_out ? n_in : n_out));
    w.total = off;
    return w;
}
bool lin_args_ok(int dtype, int T, int n_in, int n_out, int r)
{
    if (dtype != SLORA_DTYPE_F32 && dtype != SLORA_DTYPE_BF16) return false;
    if (T <= 0 || n_in <= 0 || n_out <= 0 || r < 1 || r > SLORA_MAX_RANK) return false;
    if ((long long)T * (n_in > n_out ? n_in : n_out) > (1ll << 31) - 1) return false;
    if ((long long)n_in * n_out > (1ll << 31) - 1) return false;
    if (dtype == SLORA_DTYPE_BF16 && ((n_in % 64) || (n_out % 64))) return false;
    return true;
}
}  // namespace

size_t slora_lora_linear_ws_bytes(int dtype, int T, int n_in, int n_out, int r)
{
    if (!lin_args_ok(dtype, T, n_in, n_out, r)) return 0;
    if (dtype == SLORA_DTYPE_F32) return al256(2 * sizeof(float) * (size_t)T * r);
    return lin_ws(T, n_in, n_out).total;
}

int slora_lora_linear_fwd(int dtype, int T, int n_in, int n_out, int r, float alpha, const void *x, const void *W,
                          const void *bias, const float *A, const float *B, void *y, void *ws, size_t ws_bytes,
                          void *stream)
{
    if (!lin_args_ok(dtype, T, n_in, n_out, r) || !x || !W || !A || !B || !y || !ws) return SLORA_EINVAL;
    if (ws_bytes < slora_lora_linear_ws_bytes(dtype, T, n_in, n_out, r)) return SLORA_ENOSPC;
    if (((uintptr_t)ws) & 255) return SLORA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const float s = alpha / (float)r;
    if (dtype == SLORA_DTYPE_F32)
        return f32_lora_linear_fwd(T, n_in, n_out, r, s, (const float *)x, (const float *)W, (const float *)bias, A,
                                   B, (float *)y, (float *)ws, st);
    if ((((uintptr_t)x) | ((uintptr_t)W) | ((uintptr_t)y)) & 15) return SLORA_EINVAL;
    const LinWs w = lin_ws(T, n_in, n_out);
    char *base = (char *)ws;
    int rc;
    if ((rc = launch_cast_pad(A, r, n_in, (bf16 *)(base + w.A16), 16, n_in, 0, st))) return rc;
    if ((rc = launch_cast_pad(B, n_out, r, (bf16 *)(base + w.B16), n_out, 32, 0, st))) return rc;
    GemmArgs a = gemm_base((const bf16 *)x, n_in, (const bf16 *)W, T, n_out, n_in, (const bf16 *)bias, s);
    a.zmat[0] = (bf16 *)(base + w.A16); a.tmat[0] = (bf16 *)(base + w.B16); a.zspill[0] = (bf16 *)(base + w.zs);
    a.out0 = y;
    return launch_gemm(a, EPI_STORE, 16, st);
}

int slora_frozen_linear_bf16(int T, int n_in, int n_out, const void *x, const void *W, const void *bias, void *y,
                             void *stream)
{
    if (T <= 0 || n_in <= 0 || n_out <= 0 || (n_in % 64) || (n_out % 8) || !x || !W || !y) return SLORA_EINVAL;
    if ((long long)T * (n_in > n_out ? n_in : n_out) > (1ll << 31) - 1) return SLORA_EINVAL;
    if ((long long)n_in * n_out > (1ll << 31) - 1) return SLORA_EINVAL;
    if ((((uintptr_t)x) | ((uintptr_t)W) | ((uintptr_t)y)) & 15) return SLORA_EINVAL;
    GemmArgs a = gemm_base((const bf16 *)x, n_in, (const bf16 *)W, T, n_out, n_in, (const bf16 *)bias, 0.f);
    a.out0 = y;
    return launch_gemm(a, EPI_STORE, 0, (hipStream_t)stream);
}

int slora_lora_linear_bwd(int dtype, int T, int n_in, int n_out, int r, float alpha, const void *x, const void *dy,
                          const void *W, const float *A, const float *B, void *dx, float *dA, float *dB, void *ws,
                          size_t ws_bytes, void *stream)
{
    if (!lin_args_ok(dtype, T, n_in, n_out, r) || !x || !dy || !W || !A || !B || !dx || !dA || !dB || !ws)
        return SLORA_EINVAL;
    if (ws_bytes < slora_lora_linear_ws_bytes(dtype, T, n_in, n_out, r)) return SLORA_ENOSPC;
    if (((uintptr_t)ws) & 255) return SLORA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const float s = alpha / (float)r;
    if (dtype == SLORA_DTYPE_F32)
        return f32_lora_linear_bwd(T, n_in, n_out, r, s, (const float *)x, (const float *)dy, (const float *)W, A, B,
                                   (float *)dx, dA, dB, (float *)ws, st);
    if ((((uintptr_t)x) | ((uintptr_t)W) | ((uintptr_t)dy) | ((uintptr_t)dx)) & 15) return SLORA_EINVAL;
    const LinWs w = lin_ws(T, n_in, n_out);
    char *base = (char *)ws;
    int rc;
    // the forward's rank-space activations zs = s x A^T are needed by dB: rerun the fused forward
    if ((rc = slora_lora_linear_fwd(dtype, T, n_in, n_out, r, alpha, x, W, nullptr, A, B, base + w.ytmp, ws, ws_bytes,
                                    stream)))
        return rc;
    if ((rc = launch_cast_pad(B, n_out, r, (bf16 *)(base + w.B16T), 16, n_out, 1, st))) return rc;
    if ((rc = launch_cast_pad(A, r, n_in, (bf16 *)(base + w.A16T), n_in, 32, 1, st))) return rc;
    if ((rc = launch_transpose_bf16((const bf16 *)W, n_out, n_in, (bf16 *)(base + w.WT), st))) return rc;
    GemmArgs a = gemm_base((const bf16 *)dy, n_out, (bf16 *)(base + w.WT), T, n_in, n_out, nullptr, s);
    a.zmat[0] = (bf16 *)(base + w.B16T); a.tmat[0] = (bf16 *)(base + w.A16T); a.zspill[0] = (bf16 *)(base + w.ps);
    a.out0 = dx;
    if ((rc = launch_gemm(a, EPI_STORE, 16, st))) return rc;
    float *part = (float *)(base + w.part);
    if ((rc = launch_lora_grad((const bf16 *)x, n_in, n_in, (bf16 *)(base + w.ps), 16, r, T, part, dA, 1, st)))
        return rc;
    return launch_lora_grad((const bf16 *)dy, n_out, n_out, (bf16 *)(base + w.zs), 16, r, T, part, dB, 0, st);
}

// ---- the same backward for callers that cannot allocate ------------------------------------------
// The scratch of slora_lora_linear_bwd held by the library itself: one array per GPU (every device the
// code object is loaded on has its own copy at its own address), alive until the process ends.
static __device__ __align__(256) unsigned char scratch[SLORA_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each GPU, null until first use there

// `scratch` is a host-side stand-in in host code, not a device address: ask the runtime for the address
// on the current device once and use only that pointer afterwards.
int scratch_address(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_hip_error(e, "hipGetDevice"); return SLORA_EHIP; }
    if (dev < 0 || dev >= kMaxDevices) return SLORA_EINVAL;
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) { set_hip_error(e, "hipGetSymbolAddress(scratch)"); return SLORA_EHIP; }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SLORA_OK;
}
}  // namespace

int slora_lora_linear_bwd_noalloc(int T, int n_in, int n_out, int r, float alpha, const void *x, const void *dy,
                                  const void *W, const float *A, const float *B, void *dx, float *dA, float *dB,
                                  void *stream)
{
    if (!lin_args_ok(SLORA_DTYPE_BF16, T, n_in, n_out, r) || !x || !dy || !W || !A || !B || !dx || !dA || !dB)
        return SLORA_EINVAL;
    if (slora_lora_linear_ws_bytes(SLORA_DTYPE_BF16, T, n_in, n_out, r) > (size_t)SLORA_NOALLOC_SCRATCH_BYTES)
        return SLORA_ENOSPC;
    if ((((uintptr_t)x) | ((uintptr_t)W) | ((uintptr_t)dy) | ((uintptr_t)dx)) & 15) return SLORA_EINVAL;
    void *ptr = nullptr;
    int rc = scratch_address(&ptr);
    if (rc) return rc;
    // every region of the scratch that a kernel of this call reads is written earlier in the same call
    // (padded operand copies are written whole, zeros included), so nothing has to be cleared between calls
    return slora_lora_linear_bwd(SLORA_DTYPE_BF16, T, n_in, n_out, r, alpha, x, dy, W, A, B, dx, dA, dB, ptr,
                                 (size_t)SLORA_NOALLOC_SCRATCH_BYTES, stream);
}

}  // extern "C"
