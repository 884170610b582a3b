/* slora.h -- C ABI of the MI355X (gfx950) library for the server-side step of split
 * federated LoRA fine-tuning (SplitLoRA, arXiv 2407.00952).
 *
 * What the calls compute (paper passages):
 *   Sec. II-C       LoRA: a frozen weight W plus a trainable rank-r product.  Here
 *                   y = x W^T + b + s (x A^T) B^T with A [r,in], B [out,r], s = alpha/r.
 *   Sec. III-B a3   the central server concatenates the clients' cut-layer activations
 *                   S = [s_1; ...; s_N] and runs the server-side model forward (Eq. 3),
 *                   then back-propagates to obtain the gradients of the server adapters
 *                   only (frozen weights get none) and updates them by SGD (Eq. 4, 5).
 *   Sec. III-B a4   the activation gradient of each client's slice of S is returned.
 *   Sec. III-B b2   client adapters are averaged with weights |D_i|/|D| (Eq. 8, 9).
 * The server-side model is a stack of GPT-2 blocks (pre-LayerNorm, causal attention with
 * head size 64, tanh-GELU MLP, biases on every linear); the loss head is the caller's:
 * the backward call takes the gradient dY of the caller's loss w.r.t. the stack output.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name starts with h_ (then HOST).
 *   - The library never allocates or frees device memory, never synchronises the stream
 *     and never writes to stdout.  `stream` is a hipStream_t passed as void* (NULL = the
 *     default stream).  All work is queued on that stream; buffers must stay alive until
 *     it has run.  Outputs must not alias inputs.
 *   - Return value: 0 (SLORA_OK) or a negative SLORA_E* code.  All argument and state
 *     checks happen before the first kernel launch, so they work on a machine without a GPU.
 *   - A context is not thread-safe; use one per host thread / stream.
 *   - Matrices are row-major, dense.  "bf16" is the upper 16 bits of an IEEE binary32.
 */
#ifndef SLORA_H
#define SLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SLORA_OK        0
#define SLORA_EINVAL   -1   /* NULL pointer, size out of range, unsupported configuration     */
#define SLORA_ESTATE   -2   /* call order violated, or weights / adapters / workspace unbound */
#define SLORA_ENOSPC   -3   /* workspace smaller than slora_workspace_bytes()                 */
#define SLORA_EHIP     -4   /* a HIP call failed (text: slora_last_hip_error)                 */
#define SLORA_EZERO    -5   /* FedAvg: negative sample count or zero total                    */

/* projections that may carry an adapter; bit (1u << SLORA_PROJ_x) in lora_mask */
enum { SLORA_PROJ_Q = 0, SLORA_PROJ_K = 1, SLORA_PROJ_V = 2, SLORA_PROJ_O = 3,
       SLORA_PROJ_FC = 4, SLORA_PROJ_PR = 5, SLORA_NPROJ = 6 };

/* frozen tensors of one block, all bf16 */
enum { SLORA_LN1_G = 0, SLORA_LN1_B, SLORA_WQKV /* [3d,d]: rows q, then k, then v */, SLORA_BQKV /* [3d] */,
       SLORA_WO /* [d,d] */, SLORA_BO, SLORA_LN2_G, SLORA_LN2_B, SLORA_WFC /* [d_ff,d] */, SLORA_BFC,
       SLORA_WPR /* [d,d_ff] */, SLORA_BPR, SLORA_NFROZEN };

#define SLORA_DTYPE_F32  0
#define SLORA_DTYPE_BF16 1   /* bf16 storage, fp32 accumulation */
#define SLORA_DTYPE_MXFP8 2  /* contexts only: as BF16, but every frozen product runs in MXFP8 (Sec. V-B): the
                                frozen weights are packed once (both orientations), each product's activation
                                operand is converted by the kernel that produces it or right before the
                                product, adapters stay in bf16; d_model and
                                d_ff multiples of 128.  Same calls, same outputs (bf16), looser agreement
                                with the uncompressed model: a few percent per product */

#define SLORA_MAX_RANK    16
#define SLORA_MAX_CLIENTS 64

typedef struct slora_ctx slora_ctx;      /* opaque, host memory */

typedef struct {
    int32_t  d_model;      /* multiple of 64, at most 2048; head size d_model / n_head must be 64 */
    int32_t  n_head;
    int32_t  d_ff;         /* multiple of 64                                                   */
    int32_t  n_blocks;     /* server-side blocks only                                          */
    int32_t  lora_r;       /* 1 .. SLORA_MAX_RANK                                              */
    float    lora_alpha;   /* s = lora_alpha / lora_r                                          */
    uint32_t lora_mask;    /* which projections carry an adapter, same in every block          */
    int32_t  dtype;        /* SLORA_DTYPE_BF16 (the stack has no fp32 variant)                 */
    float    ln_eps;       /* e.g. 1e-5                                                        */
    int32_t  max_seqs;     /* upper bound on the number of sequences per round (sum of b_i)    */
    int32_t  seq_len;      /* S, multiple of 64, every sequence has exactly this length        */
} slora_config;
/* Further limits checked by slora_create (SLORA_EINVAL): n_blocks <= 1024; max_seqs * seq_len <= 2^24 tokens;
 * max_seqs * seq_len * max(3 * d_model, d_ff) < 2^31 elements (the kernels address a GEMM operand with 32-bit
 * byte offsets from its base). */

/* ---- context (host only) ---------------------------------------------------------------- */
int    slora_create(const slora_config *cfg, slora_ctx **out);
int    slora_destroy(slora_ctx *ctx);
/* bytes of caller-owned device memory the context needs: transposed copies of the frozen
 * weights, bf16 copies of the adapters, the activations saved between forward and backward,
 * and scratch.  0 if ctx is NULL. */
size_t slora_workspace_bytes(const slora_ctx *ctx);
/* ws must be 256-byte aligned and stay alive while the context is used. */
int    slora_bind_workspace(slora_ctx *ctx, void *ws, size_t bytes);
/* Borrow one frozen tensor (bf16, shapes above, 16-byte aligned) of block `block`; never written.  The
 * first forward call after any bind queues the one-off set-up kernels (transposed copies of the frozen weights
 * for the backward pass, the descriptor tables of the adapters); like every other call it only queues kernels,
 * so it neither blocks nor prevents stream capture (a captured first forward repeats the set-up on every
 * replay: run one round eagerly first if that matters). */
int    slora_bind_frozen(slora_ctx *ctx, int block, int which, const void *w);
/* Borrow the fp32 master adapter of projection `proj` in block `block`: A [r,in], B [out,r],
 * and the gradient buffers dA [r,in], dB [out,r].  A, B are changed only by
 * slora_adapter_step; dA, dB are overwritten by every slora_server_bwd. */
int    slora_bind_adapter(slora_ctx *ctx, int block, int proj, float *A, float *B, float *dA, float *dB);

/* ---- the round (Sec. III-B a3, a4): state machine  fwd -> bwd -> step ------------------------ */
/* Forward of the concatenated activations (Eq. 3).  h_x_clients: K device pointers, client i
 * holding [h_batch[i], S, d] bf16; y: [sum_i h_batch[i], S, d] bf16, clients in index order.
 * Uses the adapters as they are now (R_s^{t-1}). */
int slora_server_fwd(slora_ctx *ctx, int K, const void *const *h_x_clients, const int32_t *h_batch,
                     void *y, void *stream);
/* Backward of the forward just run.  dy: [sum b_i, S, d] bf16, gradient of the caller's loss
 * w.r.t. y (any normalisation or client weighting is already inside dy).  Writes client i's
 * activation gradient [b_i,S,d] bf16 to h_dx_clients[i] and, into every bound dA/dB, the sum
 * over all tokens of all clients.  Never forms a weight, bias or LayerNorm gradient. */
int slora_server_bwd(slora_ctx *ctx, const void *dy, void *const *h_dx_clients, void *stream);
/* Eq. (4),(5): p = fmaf(-lr, g, p) on every bound A, B; legal only after a backward. */
int slora_adapter_step(slora_ctx *ctx, float lr, void *stream);

/* ---- optimiser variant: AdamW on a flat parameter vector -------------------------------------------
 * The paper's updates (Eq. 4-7) are plain SGD = slora_adapter_step.  For callers that fine-tune with
 * Adam and decoupled weight decay instead, this applies one step to n fp32 parameters p with gradient g
 * and moment vectors m, v (all device pointers, caller-owned, m = v = 0 before step 1), in the order
 *   p *= 1 - lr*wd;  m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;
 *   p -= lr/(1-b1^step) * m / (sqrt(v)/sqrt(1-b2^step) + eps)
 * evaluated in fp32 with one fixed operation order (bit-reproducible).  When p is the memory bound to a
 * context as its adapters (after slora_server_bwd / slora_client_bwd), follow it with
 * slora_adapters_changed instead of slora_adapter_step.  step >= 1, 0 <= beta < 1, eps > 0. */
int slora_adamw(size_t n, float *p, const float *g, float *m, float *v, float lr, float beta1, float beta2,
                float eps, float weight_decay, int32_t step, void *stream);

/* ---- client-adapter aggregation (Sec. III-B b2, Eq. 8-9) -------------------------------------- */
/* out[j] = sum_i w_i x_i[j] over K flat fp32 vectors of n floats, with
 * w_i = (float)((double)n_i / (double)sum n) and the fixed evaluation order
 * acc = 0; for i = 0..K-1: acc = fmaf(w_i, x_i[j], acc)  -- bit-reproducible.
 * K <= SLORA_MAX_CLIENTS; SLORA_EZERO if a count is negative or the total is zero. */
int slora_fedavg(int K, const float *const *h_client_params, const int64_t *h_sample_counts,
                 size_t n, float *out, void *stream);

/* ---- one LoRA-adapted linear layer (Sec. II-C), used on its own -------------------------------- */
/* y [T,out] = x [T,in] W[out,in]^T + bias + (alpha/r) (x A^T) B^T.  dtype F32: every buffer fp32.
 * dtype BF16: x, W, bias, y bf16 and A, B fp32; `ws` is scratch of slora_lora_linear_ws_bytes().
 * bias may be NULL.  r in 1..SLORA_MAX_RANK.  BF16: in, out multiples of 64; x, W, y, dy, dx 16-byte aligned;
 * T * max(in, out) < 2^31 and in * out < 2^31 elements.  slora_lora_linear_ws_bytes returns 0 for sizes
 * outside these limits; the calls return SLORA_EINVAL. */
size_t slora_lora_linear_ws_bytes(int dtype, int T, int n_in, int n_out, int r);
int slora_lora_linear_fwd(int dtype, int T, int n_in, int n_out, int r, float alpha,
                          const void *x, const void *W, const void *bias, const float *A, const float *B,
                          void *y, void *ws, size_t ws_bytes, void *stream);
/* dx [T,in] = dy W + s (dy B) A;  dA [r,in] = s (dy B)^T x;  dB [out,r] = s dy^T (x A^T).
 * dtype as above (dx follows x's type, dA and dB are fp32). */
int slora_lora_linear_bwd(int dtype, int T, int n_in, int n_out, int r, float alpha,
                          const void *x, const void *dy, const void *W, const float *A, const float *B,
                          void *dx, float *dA, float *dB, void *ws, size_t ws_bytes, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): slora_lora_linear_bwd for dtype BF16 with the scratch held inside the
 * library, in one fixed array of SLORA_NOALLOC_SCRATCH_BYTES per GPU that stays allocated until the process
 * ends.  Same arguments (minus dtype and the workspace), same kernels, same results as
 * slora_lora_linear_bwd.  Calls nothing that allocates or frees.  SLORA_ENOSPC when
 * slora_lora_linear_ws_bytes(SLORA_DTYPE_BF16, T, n_in, n_out, r) exceeds SLORA_NOALLOC_SCRATCH_BYTES (e.g.
 * T = 4096 with n_in = n_out = 1024 needs 11.4 MiB, T = 16384 needs 39.2 MiB); SLORA_EINVAL / SLORA_EHIP as for slora_lora_linear_bwd.
 * All calls on one GPU share that GPU's array: two calls whose work overlaps in time on one GPU (different
 * streams, or different host threads) race; calls queued on one stream are safe.  Nothing in the array has
 * to be cleared between calls. */
#define SLORA_NOALLOC_SCRATCH_BYTES (32 << 20)
int slora_lora_linear_bwd_noalloc(int T, int n_in, int n_out, int r, float alpha,
                                  const void *x, const void *dy, const void *W, const float *A, const float *B,
                                  void *dx, float *dA, float *dB, void *stream);

/* The frozen product alone (Sec. II-C with no adapter): y [T,out] = x [T,in] W[out,in]^T + bias, all
 * bf16 with fp32 accumulation; bias may be NULL.  in a multiple of 64, out a multiple of 8; x, W, y 16-byte
 * aligned; T * max(in, out) < 2^31 and in * out < 2^31 elements (SLORA_EINVAL otherwise).  Runs the same GEMM
 * kernel as the stack and needs no scratch. */
int slora_frozen_linear_bf16(int T, int n_in, int n_out, const void *x, const void *W, const void *bias,
                             void *y, void *stream);

/* ---- client-side model (Sec. III-B a1, Eq. 2: client forward up to the cut layer; a5, Eq. 6-7:
 *      client backward from the returned activation gradients and SGD on the client adapters) ---------- */
/* A client's share of the model is a context of its own (slora_create with n_blocks = the number of
 * client-side blocks; frozen weights and adapters bound as for the server).  The input of its first block
 * is the embedding of the batch: row t = wte[tokens[t]] + wpe[t mod seq_len], summed in fp32 from the two
 * frozen bf16 tables (wte [vocab, d_model], wpe [>= seq_len, d_model]); token ids outside 0..vocab-1 are
 * clamped.  tokens: device int32 [batch * seq_len].  act [batch, seq_len, d_model] bf16 receives the
 * cut-layer activations that go to the server.  batch <= max_seqs. */
int slora_client_fwd(slora_ctx *ctx, int32_t batch, const int32_t *tokens, int32_t vocab, const void *wte,
                     const void *wpe, void *act, void *stream);
/* dact [batch, seq_len, d_model] bf16 = the activation gradient received from the server (step a4).
 * Overwrites dA, dB of every bound adapter; no gradient is produced for the embedding (frozen).
 * Same call order as the server: fwd -> bwd -> slora_adapter_step (Eq. 6-7 with the client rate). */
int slora_client_bwd(slora_ctx *ctx, const void *dact, void *stream);
/* Tell a context that the caller has overwritten its bound A / B buffers (the aggregated adapters
 * coming back in step b3): the bf16 operand copies are rebuilt at the next forward.  Not allowed
 * between a forward and its backward (SLORA_ESTATE). */
int slora_adapters_changed(slora_ctx *ctx);

/* ---- loss head of the server (Sec. III-B: labels arrive with the activations in step a2; step a3
 *      computes the loss from the predicted value and the labels and derives the gradients from it) --- */
/* GPT-2's head on the stack output y [T, d_model] (bf16): u = LayerNorm(y; lnf_g, lnf_b, eps),
 * logits = u Wv^T against the frozen token-embedding matrix Wv [vocab, d_model] (bf16, no bias),
 *   loss_tok[t] = logsumexp_v logits[t, v] - logits[t, labels[t]]      (0 where the token has no label)
 *   loss        = sum_t loss_tok[t] / n,  n = number of labeled tokens   (device float)
 *   dy [T, d_model] (bf16) = d loss / d y   -- the dy argument of slora_server_bwd.
 * labels [T] int32 on the device; a label outside 0..vocab-1 marks a token without label (context
 * tokens).  With no labeled token at all, loss is NaN and dy is all zeros.  Logits are rounded to bf16
 * before the softmax, probabilities are evaluated in fp32.  Nothing in the head is trainable.
 * d_model a multiple of 64, <= 2048; vocab <= 65536.  All pointers device pointers, 16-byte aligned;
 * ws 256-byte aligned, caller-owned, slora_loss_head_ws_bytes(max_tokens, ...) bytes; its first part
 * holds a zero-padded and a transposed copy of Wv written by slora_loss_head_prepare (call it once, and
 * again only if Wv changes); the rest is scratch.  T <= max_tokens.  Nothing synchronises the stream.
 * Returns SLORA_EINVAL / SLORA_ENOSPC / SLORA_EHIP like the other calls (0 bytes from _ws_bytes on
 * invalid sizes). */
size_t slora_loss_head_ws_bytes(int32_t max_tokens, int32_t d_model, int32_t vocab);
int slora_loss_head_prepare(int32_t d_model, int32_t vocab, const void *Wv, void *ws, size_t ws_bytes,
                            void *stream);
int slora_loss_head(int32_t T, int32_t d_model, int32_t vocab, const void *y, const void *lnf_g,
                    const void *lnf_b, float eps, const int32_t *labels, void *ws, size_t ws_bytes,
                    float *loss_tok, float *loss, void *dy, void *stream);

/* ---- compressed frozen weights and cut-layer traffic (Sec. V-B: quantisation as the route to a more
 *      storage-, communication- and computation-efficient framework; the paper fixes no format) -------
 * Format: MXFP8 of the OCP Microscaling Formats (MX) v1.0 specification.  A row of K elements (K a
 * multiple of 32) becomes K element codes (FP8 E4M3, one byte each) and K/32 scale codes (E8M0, one byte
 * per block of 32 consecutive elements, value 2^(code-127)).  Conversion (MX v1.0 Sec. 6.3):
 * scale code = max(E - 8, 0) with E the biased binary32 exponent of the block's largest magnitude;
 * element = value / scale rounded to nearest, ties to even, clamped at +-448; the sign of zero is kept.
 * Inputs must be finite.  All pointers are device pointers; nothing synchronises the stream; nothing is
 * allocated.
 *
 * slora_mx_quantize:   x bf16 [M, K] with row stride ldx (elements, multiple of 8, 16-byte aligned base)
 *                      -> codes u8 [M, K] (8-byte aligned), scales u8 [M, K/32], both dense.
 * slora_mx_dequantize: the inverse map to bf16 [M, K] with row stride ldy; exact whenever the value is in
 *                      bf16's range (an E4M3 value has 4 significant bits).
 * These two are also the codec for what crosses the cut (the activations of step a2 and their gradients
 * of step a4, Sec. III-B): 8.25 bits per element instead of 16.
 *
 * slora_frozen_linear_mxfp8: y[T, n_out] = deq(x)[T, n_in] . deq(W)[n_out, n_in]^T + bias on the fp8 matrix
 *                      cores (block scales applied by the hardware, fp32 accumulation, bf16 output, dense
 *                      row-major).  n_in a multiple of 128, n_out a multiple of 8, T * n_in and
 *                      n_out * n_in below 2^32; xq, wq, y (and bias, bf16 [n_out], may be NULL) 16-byte
 *                      aligned, xs and ws 4-byte aligned.  NaN codes (S.1111.111) must not occur.
 * Errors: SLORA_EINVAL for a NULL pointer, a size or alignment outside the above; SLORA_EHIP. */
int slora_mx_quantize(int64_t M, int32_t K, const void *x, int64_t ldx, void *codes, void *scales, void *stream);
int slora_mx_dequantize(int64_t M, int32_t K, const void *codes, const void *scales, void *y, int64_t ldy,
                        void *stream);
int slora_frozen_linear_mxfp8(int32_t T, int32_t n_in, int32_t n_out, const void *xq, const void *xs,
                              const void *wq, const void *ws, const void *bias, void *y, void *stream);

/* Frozen weights in 4 bits (MXFP4: FP4 E2M1 elements -- values 0, 0.5, 1, 1.5, 2, 3, 4, 6, no NaN -- under
 * the same E8M0 scale per 32 elements, 4.25 bits per weight; the paper's pointer for quantisation is a
 * 4-bit-weight fine-tuning method, Sec. V-B).  slora_mx_quantize_fp4 is slora_mx_quantize with E2M1 elements
 * (scale code = max(E - 2, 0), clamp at +-6); codes u8 [M, K/2], two per byte, the element with the even
 * index in the low nibble (4-byte aligned).  slora_frozen_linear_mxfp8_w4 is slora_frozen_linear_mxfp8 with
 * the weight given in that form (wq4 u8 [n_out, n_in/2], 16-byte aligned); activations stay MXFP8. */
int slora_mx_quantize_fp4(int64_t M, int32_t K, const void *x, int64_t ldx, void *codes, void *scales,
                          void *stream);
int slora_frozen_linear_mxfp8_w4(int32_t T, int32_t n_in, int32_t n_out, const void *xq, const void *xs,
                                 const void *wq4, const void *ws, const void *bias, void *y, void *stream);

/* One LoRA-adapted linear layer (Sec. II-C) with the frozen product in MXFP8 and the adapter kept in bf16
 * operands / fp32 parameters:
 *   fwd:  y  = deq(Q(x)) . deq(Q(W))^T + bias + s (x A^T) B^T            s = alpha / r
 *   bwd:  dx = deq(Q(dy)) . deq(Q(W^T))^T + s (dy B) A                   (straight-through; never dW)
 *         dA = s (dy B)^T x        dB = s dy^T (x A^T)                    from the unquantised x, dy
 * Q quantises along the contraction axis of the product it feeds: x and W along n_in, dy and W^T along
 * n_out (W^T is quantised on its own).  The frozen weight is packed once:
 * slora_mx_weight_bytes:  size of the packed form (both orientations plus packing scratch), 0 if the
 *                         shape is unsupported.
 * slora_mx_pack_weight:   W bf16 [n_out, n_in] dense (16-byte aligned) -> packed (256-byte aligned,
 *                         at least slora_mx_weight_bytes).  The packed buffer is read-only afterwards.
 * slora_mx_lora_linear_ws_bytes / _fwd / _bwd: x bf16 [T, n_in], dy bf16 [T, n_out], bias bf16 [n_out] or
 *                         NULL, A fp32 [r, n_in], B fp32 [n_out, r]; outputs y bf16 [T, n_out], dx bf16
 *                         [T, n_in], dA fp32 [r, n_in], dB fp32 [n_out, r] (overwritten); ws caller-owned,
 *                         256-byte aligned, holds the quantised activations and the rank-space
 *                         intermediates; bwd does not need a preceding fwd.
 * n_in and n_out multiples of 128, 1 <= r <= SLORA_MAX_RANK, T * max(n_in, n_out) and n_in * n_out below
 * 2^31.  Errors: SLORA_EINVAL, SLORA_ENOSPC (ws or packed buffer too small), SLORA_EHIP. */
/* The server's round with compressed cut-layer traffic: what the clients upload in step a2 and what goes
 * back to them in step a4 (Sec. III-B) is MXFP8 instead of bf16.  slora_server_fwd_mx is slora_server_fwd
 * with client i's activations given as element codes h_xq_clients[i] (u8 [b_i, S, d], 8-byte aligned) and
 * scale codes h_xs_clients[i] (u8 [b_i, S, d/32]), blocks along d; they are expanded on the fly by the
 * first LayerNorm (no bf16 copy is made), so the result equals slora_server_fwd on the dequantised
 * activations bit for bit.  slora_server_bwd_mx is slora_server_bwd with client i's activation gradient
 * written as codes and scales of the same shapes: Q(bf16(dx)), i.e. exactly slora_mx_quantize of what
 * slora_server_bwd would have written.  The two forms can be mixed within a round.  Same errors and state
 * machine as the bf16 calls; d_model is a multiple of 64 already, hence of 32. */
int slora_server_fwd_mx(slora_ctx *ctx, int K, const void *const *h_xq_clients, const void *const *h_xs_clients,
                        const int32_t *h_batch, void *y, void *stream);
int slora_server_bwd_mx(slora_ctx *ctx, const void *dy, void *const *h_dxq_clients, void *const *h_dxs_clients,
                        void *stream);

size_t slora_mx_weight_bytes(int32_t n_in, int32_t n_out);
int slora_mx_pack_weight(int32_t n_in, int32_t n_out, const void *W, void *packed, size_t bytes, void *stream);
size_t slora_mx_lora_linear_ws_bytes(int32_t T, int32_t n_in, int32_t n_out, int32_t r);
int slora_mx_lora_linear_fwd(int32_t T, int32_t n_in, int32_t n_out, int32_t r, float alpha, const void *x,
                             const void *packed_w, const void *bias, const float *A, const float *B, void *y,
                             void *ws, size_t ws_bytes, void *stream);
int slora_mx_lora_linear_bwd(int32_t T, int32_t n_in, int32_t n_out, int32_t r, float alpha, const void *x,
                             const void *dy, const void *packed_w, const float *A, const float *B, void *dx,
                             float *dA, float *dB, void *ws, size_t ws_bytes, void *stream);

/* ---- measurement hook (not part of the method) ---------------------------------------------------- */
/* Kernel launches of the kinds selected by slora_prof_enable (bit k of `kinds` = kind k; 0 = off; 1 = the
 * bf16 GEMM launches only) are bracketed by HIP events on their stream.  slora_prof_read_kind waits for the
 * recorded events (it BLOCKS the host) and returns, for one kind, the summed kernel time in milliseconds, the
 * summed algorithmic work of those launches and their number.  Work is in flop for the matrix-core kinds --
 * GEMM: 2*M*N*K of the frozen product (Sec. II-C); attention: 2*S*d per token forward, 4*S*d backward, lower
 * triangle only -- and in bytes for the HBM-bound kinds: each tensor the kernel must read or write, once.
 * At most 16384 launches are recorded between two calls of slora_prof_enable, which also clears the record.
 * slora_prof_read is slora_prof_read_kind(SLORA_PROF_GEMM, ...).  Process-wide, not thread-safe.
 * SLORA_EINVAL for an unknown kind, SLORA_EHIP if an event call fails. */
enum { SLORA_PROF_GEMM = 0,      /* frozen products with the fused low-rank branch (flop)                 */
       SLORA_PROF_LN_FWD,        /* LayerNorm forward (bytes)                                              */
       SLORA_PROF_LN_BWD,        /* LayerNorm backward + residual gradient (bytes)                         */
       SLORA_PROF_LORA_GRAD,     /* streaming pass of an adapter gradient dA or dB (bytes)                 */
       SLORA_PROF_SGD,           /* Eq. (4)-(5) over all adapters (bytes)                                  */
       SLORA_PROF_ATTN_FWD,      /* attention forward (flop)                                               */
       SLORA_PROF_ATTN_BWD,      /* attention backward (flop)                                              */
       SLORA_PROF_FEDAVG,        /* Eq. (8)-(9) (bytes)                                                    */
       SLORA_PROF_KINDS };
int slora_prof_enable(int kinds);
int slora_prof_read_kind(int kind, double *h_ms, double *h_work, int *h_launches);
int slora_prof_read(double *h_gemm_ms, double *h_gemm_flop, int *h_launches);
/* The shader clock the chip held during the recorded GEMM launches, in MHz (the datasheet peak assumes 2400):
 * while SLORA_PROF_GEMM is selected, the launches that run the 4-wave kernel store the shader-clock counter and
 * the 100 MHz reference counter at their start and end; this call synchronises the device (it BLOCKS), and
 * returns sum of shader ticks / sum of reference ticks x 100 over those launches and their number (0 MHz with no
 * sample).  Uses 512 KB of device memory of the library's own (a static array). */
int slora_prof_read_clock(double *h_mhz, int *h_samples);

const char *slora_strerror(int code);
const char *slora_last_hip_error(void);   /* text of the last failed HIP call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* SLORA_H */
