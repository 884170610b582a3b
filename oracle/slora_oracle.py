"""Plain fp64 CPU oracle for the server-side step of split federated LoRA fine-tuning.

THIS IS TEST INFRASTRUCTURE.  It is deliberately slow and plain; it exists only so
that tests, the smoke check and the benchmark's CPU-baseline leg have an
independent statement of what the GPU library must compute.  It shares no code
with the HIP path and must never be imported by the product package.

What it follows (SplitLoRA, arXiv 2407.00952):
  * LoRA parameterisation  W + dW with a rank-r product (Sec. II-C); the scale
    alpha/r and the orientation A:[r,in], B:[out,r] are the usual LoRA convention
    (the paper prints only the product of the two factors).
  * Step a3 of Sec. III-B: the central server concatenates the clients'
    activations S = [s_1; ...; s_N], runs the server-side model forward (Eq. 3),
    and back-propagates to get the gradients of the server adapters only; the
    frozen weights W_s get no gradient (Sec. III-A).
  * Eq. (4),(5): plain SGD on every server adapter matrix.
  * Step a4: the activation gradient of each client's slice of S is returned.
  * Step b2, Eq. (8),(9): client adapters are averaged with weights |D_i|/|D|,
    A and B separately (i.e. element-wise on the flat parameter vector).

The block internals are not in the paper; they are the public GPT-2 block:
pre-LayerNorm, causal multi-head attention with 1/sqrt(dh) scaling, tanh-GELU
MLP, biases on every linear, biased variance and eps inside the square root.

Everything is float64.  Contractions use numpy matmul; nothing is blocked, fused or
reordered beyond the definitions above.  Sequences are independent, so the stack
runs one sequence at a time.

Pinned by tests/test_oracle_*.py (B = 0 equality, merged-weight identity, torch
fp64 autograd of library ops, finite differences of an independent loop-only
forward, split-then-merge, causality, client structure, FedAvg identities).
"""
from __future__ import annotations

import math
import numpy as np

PROJ_NAMES = ("q", "k", "v", "o", "fc", "pr")
_GELU_C = math.sqrt(2.0 / math.pi)
_GELU_K = 0.044715


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


# ----------------------------------------------------------------------------------
# LoRA-adapted linear layer (Sec. II-C):  y = x W^T + b + s (x A^T) B^T,  s = alpha / r
# ----------------------------------------------------------------------------------
def lora_linear_fwd(x, W, b, A, B, s):
    """x [T,in], W [out,in], b [out] or None, A [r,in], B [out,r] (or both None).

    Returns (y [T,out], z [T,r] or None) with z = x A^T.
    """
    x, W, b, A, B = _f64(x), _f64(W), _f64(b), _f64(A), _f64(B)
    y = x @ W.T
    if b is not None:
        y = y + b
    z = None
    if A is not None:
        z = x @ A.T
        y = y + s * (z @ B.T)
    return y, z


def lora_linear_bwd(x, dy, W, A, B, s):
    """Gradients of <y, dy> w.r.t. x, A and B; none for W or the bias (frozen).

    Returns (dx [T,in], dA [r,in] or None, dB [out,r] or None).
    """
    x, dy, W, A, B = _f64(x), _f64(dy), _f64(W), _f64(A), _f64(B)
    dx = dy @ W
    if A is None:
        return dx, None, None
    z = x @ A.T                      # [T,r]
    p = dy @ B                       # [T,r]
    dx = dx + s * (p @ A)
    dA = s * (p.T @ x)
    dB = s * (dy.T @ z)
    return dx, dA, dB


# ----------------------------------------------------------------------------------
# LayerNorm, GELU, causal attention: forward and hand-written backward
# ----------------------------------------------------------------------------------
def layernorm_fwd(h, gamma, beta, eps):
    """Per row: mu = mean, var = biased variance, rho = (var+eps)^-1/2."""
    h = _f64(h)
    mu = h.mean(axis=-1, keepdims=True)
    var = ((h - mu) ** 2).mean(axis=-1, keepdims=True)
    rho = 1.0 / np.sqrt(var + eps)
    xhat = (h - mu) * rho
    return xhat * _f64(gamma) + _f64(beta), (xhat, rho)


def layernorm_bwd(du, gamma, saved):
    """Input gradient only (gamma, beta are frozen)."""
    xhat, rho = saved
    dxhat = _f64(du) * _f64(gamma)
    m1 = dxhat.mean(axis=-1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    return rho * (dxhat - m1 - xhat * m2)


def gelu_tanh(f):
    f = _f64(f)
    t = np.tanh(_GELU_C * (f + _GELU_K * f ** 3))
    return 0.5 * f * (1.0 + t)


def gelu_tanh_grad(f):
    f = _f64(f)
    t = np.tanh(_GELU_C * (f + _GELU_K * f ** 3))
    return 0.5 * (1.0 + t) + 0.5 * f * (1.0 - t * t) * _GELU_C * (1.0 + 3.0 * _GELU_K * f * f)


def attention_fwd(q, k, v, n_head):
    """Causal multi-head attention for ONE sequence.  q,k,v [S,d]; returns (o [S,d], P [H,S,S])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    S, d = q.shape
    dh = d // n_head
    scale = 1.0 / math.sqrt(dh)
    o = np.empty_like(q)
    P = np.empty((n_head, S, S))
    future = np.triu(np.ones((S, S), dtype=bool), k=1)      # j > i
    for a in range(n_head):
        c = slice(a * dh, (a + 1) * dh)
        sc = (q[:, c] @ k[:, c].T) * scale
        sc[future] = -np.inf
        sc = sc - sc.max(axis=-1, keepdims=True)
        e = np.exp(sc)
        P[a] = e / e.sum(axis=-1, keepdims=True)
        o[:, c] = P[a] @ v[:, c]
    return o, P


def attention_bwd(do, q, k, v, P, n_head):
    """Returns (dq, dk, dv), each [S,d]."""
    do, q, k, v = _f64(do), _f64(q), _f64(k), _f64(v)
    S, d = q.shape
    dh = d // n_head
    scale = 1.0 / math.sqrt(dh)
    dq = np.empty_like(q)
    dk = np.empty_like(q)
    dv = np.empty_like(q)
    for a in range(n_head):
        c = slice(a * dh, (a + 1) * dh)
        dv[:, c] = P[a].T @ do[:, c]
        dP = do[:, c] @ v[:, c].T
        dS = P[a] * (dP - (dP * P[a]).sum(axis=-1, keepdims=True))
        dq[:, c] = (dS @ k[:, c]) * scale
        dk[:, c] = (dS.T @ q[:, c]) * scale
    return dq, dk, dv


# ----------------------------------------------------------------------------------
# One GPT-2 block with LoRA on any subset of {q,k,v,o,fc,pr}; one sequence [S,d]
# ----------------------------------------------------------------------------------
def _split_qkv(blk, d):
    Wqkv, bqkv = _f64(blk["Wqkv"]), _f64(blk["bqkv"])
    return {
        "q": (Wqkv[0:d], bqkv[0:d]),
        "k": (Wqkv[d:2 * d], bqkv[d:2 * d]),
        "v": (Wqkv[2 * d:3 * d], bqkv[2 * d:3 * d]),
        "o": (_f64(blk["Wo"]), _f64(blk["bo"])),
        "fc": (_f64(blk["Wfc"]), _f64(blk["bfc"])),
        "pr": (_f64(blk["Wpr"]), _f64(blk["bpr"])),
    }


def _lin_fwd(x, lin, adapters, name, s):
    W, b = lin[name]
    A, B = adapters.get(name, (None, None))
    return lora_linear_fwd(x, W, b, A, B, s)[0]


def _lin_bwd(x, dy, lin, adapters, name, s, grads):
    W, _ = lin[name]
    A, B = adapters.get(name, (None, None))
    dx, dA, dB = lora_linear_bwd(x, dy, W, A, B, s)
    if A is not None:
        grads[name] = (dA, dB)
    return dx


def block_fwd(h, blk, adapters, n_head, s, eps, _lin_fwd=_lin_fwd):
    """h [S,d] -> (h_out [S,d], saved).  (`_lin_fwd`: how a linear layer is evaluated; oracle/mx.py passes the
    variant with the frozen product in MXFP8.)"""
    h = _f64(h)
    d = h.shape[1]
    lin = _split_qkv(blk, d)
    u, ln1 = layernorm_fwd(h, blk["ln1_g"], blk["ln1_b"], eps)
    q = _lin_fwd(u, lin, adapters, "q", s)
    k = _lin_fwd(u, lin, adapters, "k", s)
    v = _lin_fwd(u, lin, adapters, "v", s)
    o, P = attention_fwd(q, k, v, n_head)
    h1 = h + _lin_fwd(o, lin, adapters, "o", s)
    u2, ln2 = layernorm_fwd(h1, blk["ln2_g"], blk["ln2_b"], eps)
    f = _lin_fwd(u2, lin, adapters, "fc", s)
    g = gelu_tanh(f)
    h2 = h1 + _lin_fwd(g, lin, adapters, "pr", s)
    saved = dict(ln1=ln1, u=u, q=q, k=k, v=v, P=P, o=o, ln2=ln2, u2=u2, f=f, g=g)
    return h2, saved


def block_bwd(dh2, blk, adapters, n_head, s, saved, _lin_bwd=_lin_bwd):
    """dh2 [S,d] -> (dh [S,d], {proj: (dA, dB)})."""
    dh2 = _f64(dh2)
    d = dh2.shape[1]
    lin = _split_qkv(blk, d)
    grads = {}
    dg = _lin_bwd(saved["g"], dh2, lin, adapters, "pr", s, grads)
    df = dg * gelu_tanh_grad(saved["f"])
    du2 = _lin_bwd(saved["u2"], df, lin, adapters, "fc", s, grads)
    dh1 = dh2 + layernorm_bwd(du2, blk["ln2_g"], saved["ln2"])
    do = _lin_bwd(saved["o"], dh1, lin, adapters, "o", s, grads)
    dq, dk, dv = attention_bwd(do, saved["q"], saved["k"], saved["v"], saved["P"], n_head)
    du = _lin_bwd(saved["u"], dq, lin, adapters, "q", s, grads)
    du = du + _lin_bwd(saved["u"], dk, lin, adapters, "k", s, grads)
    du = du + _lin_bwd(saved["u"], dv, lin, adapters, "v", s, grads)
    dh = dh1 + layernorm_bwd(du, blk["ln1_g"], saved["ln1"])
    return dh, grads


# ----------------------------------------------------------------------------------
# The server (Sec. III-B step a3, a4; Eq. 3-5)
# ----------------------------------------------------------------------------------
class ServerOracle:
    """Server-side stack: frozen blocks + one adapter set R_s.

    blocks   : list (length L) of dicts with ln1_g, ln1_b, Wqkv [3d,d], bqkv, Wo, bo,
               ln2_g, ln2_b, Wfc [d_ff,d], bfc, Wpr [d,d_ff], bpr
    adapters : list (length L) of dicts {proj: (A [r,in], B [out,r])}, proj in PROJ_NAMES
    """

    # how a linear layer is evaluated forward and backward (a subclass may replace the pair)
    lin_fwd = staticmethod(_lin_fwd)
    lin_bwd = staticmethod(_lin_bwd)

    def __init__(self, blocks, adapters, n_head, lora_alpha, lora_r, eps=1e-5):
        self.blocks = blocks
        self.adapters = [{p: (_f64(A).copy(), _f64(B).copy()) for p, (A, B) in ad.items()}
                         for ad in adapters]
        self.n_head = int(n_head)
        self.s = float(lora_alpha) / float(lora_r)
        self.eps = float(eps)
        self._saved = None
        self._batch = None
        self.grads = None

    # -- one sequence at a time ------------------------------------------------------
    def fwd_sequence(self, h0):
        h = _f64(h0)
        saved = []
        for blk, ad in zip(self.blocks, self.adapters):
            h, sv = block_fwd(h, blk, ad, self.n_head, self.s, self.eps, self.lin_fwd)
            saved.append(sv)
        return h, saved

    def bwd_sequence(self, dy, saved):
        dh = _f64(dy)
        grads = [None] * len(self.blocks)
        for l in range(len(self.blocks) - 1, -1, -1):
            dh, grads[l] = block_bwd(dh, self.blocks[l], self.adapters[l], self.n_head,
                                     self.s, saved[l], self.lin_bwd)
        return dh, grads

    def fwd_bwd_sequence(self, h0, dy):
        """(y, dx, grads) for one sequence; nothing is kept."""
        y, saved = self.fwd_sequence(h0)
        dx, grads = self.bwd_sequence(dy, saved)
        return y, dx, grads

    # -- the round: concat, forward, backward, per-client gradients --------------------
    def fwd(self, clients):
        """clients: list of K arrays [b_i,S,d].  S^t is their concatenation in client order.

        Returns Y [sum b_i, S, d]."""
        self._batch = [int(c.shape[0]) for c in clients]
        S_all = np.concatenate([_f64(c) for c in clients], axis=0)
        Y = np.empty_like(S_all)
        self._saved = []
        for n in range(S_all.shape[0]):
            Y[n], sv = self.fwd_sequence(S_all[n])
            self._saved.append(sv)
        return Y

    def bwd(self, dY):
        """dY [sum b_i, S, d] -> list of K activation gradients [b_i,S,d]; fills self.grads
        with the sums over every token of every client."""
        if self._saved is None:
            raise RuntimeError("bwd before fwd")
        dY = _f64(dY)
        dX = np.empty_like(dY)
        total = [dict() for _ in self.blocks]
        for n in range(dY.shape[0]):
            dX[n], g = self.bwd_sequence(dY[n], self._saved[n])
            for l, gl in enumerate(g):
                for p, (dA, dB) in gl.items():
                    if p in total[l]:
                        total[l][p] = (total[l][p][0] + dA, total[l][p][1] + dB)
                    else:
                        total[l][p] = (dA, dB)
        self.grads = total
        self._saved = None
        out, at = [], 0
        for b in self._batch:
            out.append(dX[at:at + b])
            at += b
        return out

    def step(self, lr):
        """Eq. (4),(5): A <- A - lr G_A, B <- B - lr G_B for every server adapter."""
        if self.grads is None:
            raise RuntimeError("step before bwd")
        for l, ad in enumerate(self.adapters):
            for p in list(ad.keys()):
                A, B = ad[p]
                dA, dB = self.grads[l][p]
                ad[p] = (A - lr * dA, B - lr * dB)
        self.grads = None


# ----------------------------------------------------------------------------------
# Client-adapter aggregation (step b2, Eq. 8-9)
# ----------------------------------------------------------------------------------
def fedavg(client_params, sample_counts):
    """client_params: K flat vectors of equal length; sample_counts: K integers |D_i|.

    out = sum_i (|D_i| / |D|) x_i with |D| = sum_i |D_i|, clients taken in index order.
    """
    n = np.asarray(sample_counts, dtype=np.float64)
    if np.any(n < 0) or n.sum() <= 0:
        raise ValueError("sample counts must be non-negative with a positive sum")
    tot = n.sum()
    out = np.zeros_like(_f64(client_params[0]))
    for ni, x in zip(n, client_params):
        out = out + (ni / tot) * _f64(x)
    return out


# ----------------------------------------------------------------------------------
# Optimiser variant (not in the paper, whose Eq. 4-7 are plain SGD): Adam with decoupled
# weight decay (Loshchilov & Hutter), in the order torch.optim.AdamW applies it.
# ----------------------------------------------------------------------------------
def adamw_step(p, g, m, v, lr, beta1, beta2, eps, weight_decay, step):
    """One update of the flat vectors; step counts from 1.  Returns (p, m, v)."""
    p, g, m, v = _f64(p), _f64(g), _f64(m), _f64(v)
    p = p * (1.0 - lr * weight_decay)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    bc1 = 1.0 - beta1 ** step
    bc2 = 1.0 - beta2 ** step
    p = p - (lr / bc1) * m / (np.sqrt(v) / math.sqrt(bc2) + eps)
    return p, m, v
