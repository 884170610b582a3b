"""Seeded synthetic inputs shaped like the SplitLoRA server-side workloads.

This module holds input generation only (shapes, distributions, seeds, rounding of
INPUT values to bf16-representable numbers).  It contains none of the method's
arithmetic and is the one module both the CPU oracle's tests and the GPU path's
tests may import.

Shapes follow the paper's setup (Sec. IV-A: GPT-2 small / medium, sequences up to
512 tokens, a few client layers and the rest on the server, rank r in {1,2,4,8})
and the five workload descriptions this repository is measured on, which extend
them (more clients, GPT-2-large dimensions, rank 16, sequence 1024).  The E2E NLG
records and the pre-trained weights the paper uses are replaced by random tensors:
    activations, upstream gradient ~ N(0,1);  W ~ N(0, 0.02^2);
    biases, LayerNorm beta ~ N(0, 0.02^2);  LayerNorm gamma ~ 1 + N(0, 0.02^2);
    A ~ U(-1/sqrt(in), 1/sqrt(in));  B ~ N(0, 0.01^2);  sample counts ~ U{100..1000}.
Draw order for one stack (numpy Generator(PCG64(seed))): per block ln1_g, ln1_b,
Wqkv, bqkv, Wo, bo, ln2_g, ln2_b, Wfc, bfc, Wpr, bpr; then per block the adapters in
projection order (A then B); then client activations in client order; then dY.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 240700952
PROJ_NAMES = ("q", "k", "v", "o", "fc", "pr")


@dataclass(frozen=True)
class StackConfig:
    name: str
    d_model: int
    n_head: int
    d_ff: int
    n_blocks: int           # server-side blocks only
    lora_r: int
    lora_alpha: float
    lora_proj: tuple        # subset of PROJ_NAMES
    n_clients: int          # K
    batch: int              # b sequences per client
    seq_len: int            # S
    ln_eps: float = 1e-5
    seed: int = BASE_SEED

    @property
    def n_seq(self):
        return self.n_clients * self.batch

    @property
    def tokens(self):
        return self.n_seq * self.seq_len

    def proj_shape(self, p):
        """(in, out) of projection p."""
        d, f = self.d_model, self.d_ff
        return {"q": (d, d), "k": (d, d), "v": (d, d), "o": (d, d), "fc": (d, f), "pr": (f, d)}[p]


# Workloads 2-5 (workload 1 is the single fp32 layer, see make_single_layer).
CONFIGS = {
    2: StackConfig("gpt2-small-split3", 768, 12, 3072, 9, 4, 32.0, ("q", "v"), 5, 4, 512,
                   seed=BASE_SEED + 2),
    3: StackConfig("gpt2-medium-split6", 1024, 16, 4096, 18, 4, 32.0, ("q", "v"), 8, 8, 512,
                   seed=BASE_SEED + 3),
    4: StackConfig("gpt2-large-split6", 1280, 20, 5120, 30, 8, 32.0, ("q", "k", "v", "o"), 8, 4, 1024,
                   seed=BASE_SEED + 4),
    5: StackConfig("gpt2-medium-split6-r16-all", 1024, 16, 4096, 18, 16, 32.0, PROJ_NAMES, 16, 4, 1024,
                   seed=BASE_SEED + 5),
}
# FedAvg leg of workload 5: 16 client adapter sets, 6 client blocks, r = 16, all six projections.
FEDAVG_CLIENT_BLOCKS = 6


def tiny_config(**kw):
    """A small stack for CPU tests and quick GPU parity; override any field."""
    base = StackConfig("tiny", 128, 2, 256, 2, 4, 32.0, ("q", "v"), 2, 1, 128, seed=BASE_SEED + 100)
    return replace(base, **kw)


# ------------------------------------------------------------------------------------
# bf16 helpers for INPUT preparation (round-to-nearest-even, no NaN handling needed)
# ------------------------------------------------------------------------------------
def bf16_bits(a):
    """float32 array -> uint16 array of bf16 bit patterns (RNE)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    u = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(a):
    """float32 array -> float32 array whose values are exactly representable in bf16."""
    return bf16_bits_to_f32(bf16_bits(a)).reshape(np.shape(a))


def _normal(rng, shape, std=1.0, mean=0.0):
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return a


def make_block(rng, cfg, quant):
    d, f = cfg.d_model, cfg.d_ff
    q = round_bf16 if quant else (lambda a: a)
    blk = {}
    blk["ln1_g"] = q(_normal(rng, (d,), 0.02, 1.0))
    blk["ln1_b"] = q(_normal(rng, (d,), 0.02))
    blk["Wqkv"] = q(_normal(rng, (3 * d, d), 0.02))
    blk["bqkv"] = q(_normal(rng, (3 * d,), 0.02))
    blk["Wo"] = q(_normal(rng, (d, d), 0.02))
    blk["bo"] = q(_normal(rng, (d,), 0.02))
    blk["ln2_g"] = q(_normal(rng, (d,), 0.02, 1.0))
    blk["ln2_b"] = q(_normal(rng, (d,), 0.02))
    blk["Wfc"] = q(_normal(rng, (f, d), 0.02))
    blk["bfc"] = q(_normal(rng, (f,), 0.02))
    blk["Wpr"] = q(_normal(rng, (d, f), 0.02))
    blk["bpr"] = q(_normal(rng, (d,), 0.02))
    return blk


def make_adapter(rng, r, n_in, n_out, quant):
    lim = 1.0 / np.sqrt(n_in)
    A = rng.uniform(-lim, lim, size=(r, n_in)).astype(np.float32)
    B = _normal(rng, (n_out, r), 0.01)
    if quant:
        A, B = round_bf16(A), round_bf16(B)
    return A, B


def make_stack_inputs(cfg, quant=True, with_dy=True):
    """All inputs of one server round for `cfg`.

    Returns dict(blocks=[...], adapters=[{proj:(A,B)}...], clients=[K x [b,S,d] f32], dY=[K*b,S,d] f32).
    With quant=True every value is bf16-representable (stored as float32).
    """
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    blocks = [make_block(rng, cfg, quant) for _ in range(cfg.n_blocks)]
    adapters = []
    for _ in range(cfg.n_blocks):
        ad = {}
        for p in PROJ_NAMES:
            if p in cfg.lora_proj:
                n_in, n_out = cfg.proj_shape(p)
                ad[p] = make_adapter(rng, cfg.lora_r, n_in, n_out, quant)
        adapters.append(ad)
    q = round_bf16 if quant else (lambda a: a)
    clients = [q(_normal(rng, (cfg.batch, cfg.seq_len, cfg.d_model))) for _ in range(cfg.n_clients)]
    out = dict(blocks=blocks, adapters=adapters, clients=clients)
    if with_dy:
        out["dY"] = q(_normal(rng, (cfg.n_seq, cfg.seq_len, cfg.d_model)))
    return out


def make_single_layer(T=1024, n_in=768, n_out=768, r=4, alpha=32.0, seed=BASE_SEED + 1,
                      quant=False, bias=False):
    """Workload 1: one LoRA-adapted linear layer, fp32 unless quant."""
    rng = np.random.Generator(np.random.PCG64(seed))
    q = round_bf16 if quant else (lambda a: a)
    x = q(_normal(rng, (T, n_in)))
    W = q(_normal(rng, (n_out, n_in), 0.02))
    A, B = make_adapter(rng, r, n_in, n_out, quant)
    dy = q(_normal(rng, (T, n_out)))
    b = q(_normal(rng, (n_out,), 0.02)) if bias else None
    return dict(x=x, W=W, b=b, A=A, B=B, dy=dy, r=r, alpha=alpha)


def fedavg_param_count(cfg, n_blocks=FEDAVG_CLIENT_BLOCKS):
    """Floats in one client's adapter set: n_blocks x sum over adapted projections of r*(in+out)."""
    per_block = sum(cfg.lora_r * sum(cfg.proj_shape(p)) for p in cfg.lora_proj)
    return n_blocks * per_block


def make_fedavg_inputs(n_clients=16, n_params=None, seed=BASE_SEED + 5 + 1000, cfg=None):
    """K flat fp32 adapter vectors (A ~ U, B ~ N as above, flattened block by block) + sample counts."""
    cfg = cfg or CONFIGS[5]
    rng = np.random.Generator(np.random.PCG64(seed))
    if n_params is None:
        vecs = []
        for _ in range(n_clients):
            parts = []
            for _ in range(FEDAVG_CLIENT_BLOCKS):
                for p in cfg.lora_proj:
                    n_in, n_out = cfg.proj_shape(p)
                    A, B = make_adapter(rng, cfg.lora_r, n_in, n_out, False)
                    parts += [A.ravel(), B.ravel()]
            vecs.append(np.concatenate(parts))
    else:
        vecs = [_normal(rng, (n_params,), 0.02) for _ in range(n_clients)]
    counts = rng.integers(100, 1001, size=n_clients).astype(np.int64)
    return vecs, counts


GPT2_VOCAB = 50257


def make_loss_head_inputs(n_seq, seq_len, d_model, vocab=GPT2_VOCAB, seed=BASE_SEED + 3 + 2000, quant=True,
                          y_std=1.0):
    """Inputs of the server's loss head: final LayerNorm, vocabulary matrix, stack output, labels.

    Returns dict(lnf_g [d], lnf_b [d], Wv [V,d], y [n_seq*S, d], labels [n_seq*S] int32).
    Labels follow the shape of prompt-completion fine-tuning data: in every sequence a context of
    c ~ U[S/4, S/2) leading tokens carries no label (-1), the rest are uniform over the vocabulary.
    Draw order: lnf_g, lnf_b, Wv, y, then per sequence c and its labels.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    q = round_bf16 if quant else (lambda a: a)
    out = {}
    out["lnf_g"] = q(_normal(rng, (d_model,), 0.02, 1.0))
    out["lnf_b"] = q(_normal(rng, (d_model,), 0.02))
    out["Wv"] = q(_normal(rng, (vocab, d_model), 0.02))
    out["y"] = q(_normal(rng, (n_seq * seq_len, d_model), y_std))
    labels = np.empty((n_seq, seq_len), dtype=np.int32)
    for s in range(n_seq):
        c = int(rng.integers(max(seq_len // 4, 0), max(seq_len // 2, 1)))
        labels[s] = rng.integers(0, vocab, size=seq_len).astype(np.int32)
        labels[s, :c] = -1
    out["labels"] = labels.reshape(-1)
    return out


def make_mx_linear_inputs(M, K, N, seed=BASE_SEED + 4 + 3000, outliers=True):
    """Inputs of one frozen linear layer in compressed form, all bf16-representable.

    Returns dict(x [M,K], W [N,K], bias [N]).  x has the look of a LayerNorm output (unit normal) with,
    when `outliers`, a handful of feature columns 8..30 times larger (the channel outliers of transformer
    activations, which is what a per-block scale is for) and one all-zero block per 61 rows; W ~ N(0, 0.02^2)
    as in GPT-2's initialisation; bias ~ N(0, 0.02^2).  Draw order: x, column factors, W, bias.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    x = _normal(rng, (M, K), 1.0)
    if outliers:
        cols = rng.choice(K, size=max(K // 128, 1), replace=False)
        x[:, cols] *= rng.uniform(8.0, 30.0, size=len(cols)).astype(x.dtype)
        x[::61, :32] = 0.0
    W = _normal(rng, (N, K), 0.02)
    bias = _normal(rng, (N,), 0.02)
    return dict(x=round_bf16(x), W=round_bf16(W), bias=round_bf16(bias))
