"""Loop-only twin of the oracle's forward pass, for tiny shapes (S <= 8, d <= 16).

TEST INFRASTRUCTURE ONLY.  No matmul, no einsum, no broadcasting: every output
element is written as the explicit sum the definition gives, so that an index or
transposition slip in the vectorised oracle shows up as a mismatch.  Central
finite differences of the scalar <Y, G> computed with THIS forward pin the
oracle's hand-written backward.

Follows the same passages as slora_oracle.py: the LoRA product (Sec. II-C), the
server forward of Eq. (3) over the concatenated activations, and the GPT-2 block.
"""
from __future__ import annotations

import math

_C = math.sqrt(2.0 / math.pi)


def linear(x, W, b, A, B, s):
    """x [T][in] lists; y[t][o] = sum_i x[t][i] W[o][i] + b[o] + s sum_j (sum_i x[t][i] A[j][i]) B[o][j]."""
    T, n_in, n_out = len(x), len(x[0]), len(W)
    y = [[0.0] * n_out for _ in range(T)]
    for t in range(T):
        z = []
        if A is not None:
            for j in range(len(A)):
                acc = 0.0
                for i in range(n_in):
                    acc += x[t][i] * A[j][i]
                z.append(acc)
        for o in range(n_out):
            acc = 0.0
            for i in range(n_in):
                acc += x[t][i] * W[o][i]
            if b is not None:
                acc += b[o]
            if A is not None:
                lo = 0.0
                for j in range(len(A)):
                    lo += z[j] * B[o][j]
                acc += s * lo
            y[t][o] = acc
    return y


def layernorm(h, gamma, beta, eps):
    out = []
    for row in h:
        d = len(row)
        mu = sum(row) / d
        var = sum((v - mu) * (v - mu) for v in row) / d
        rho = 1.0 / math.sqrt(var + eps)
        out.append([(row[i] - mu) * rho * gamma[i] + beta[i] for i in range(d)])
    return out


def gelu(f):
    return 0.5 * f * (1.0 + math.tanh(_C * (f + 0.044715 * f * f * f)))


def attention(q, k, v, n_head):
    S, d = len(q), len(q[0])
    dh = d // n_head
    o = [[0.0] * d for _ in range(S)]
    for a in range(n_head):
        c0 = a * dh
        for i in range(S):
            sc = []
            for j in range(i + 1):                      # causal: keys 0..i only
                acc = 0.0
                for e in range(dh):
                    acc += q[i][c0 + e] * k[j][c0 + e]
                sc.append(acc / math.sqrt(dh))
            m = max(sc)
            w = [math.exp(v_ - m) for v_ in sc]
            tot = sum(w)
            for e in range(dh):
                acc = 0.0
                for j in range(i + 1):
                    acc += (w[j] / tot) * v[j][c0 + e]
                o[i][c0 + e] = acc
    return o


def _rows(M, r0, r1):
    return [list(map(float, M[r])) for r in range(r0, r1)]


def block(h, blk, adapters, n_head, s, eps):
    """h [S][d] list of lists; blk / adapters hold numpy arrays or nested lists."""
    d = len(h[0])

    def lin(x, name, W, b):
        A, B = adapters.get(name, (None, None))
        A = None if A is None else [list(map(float, r)) for r in A]
        B = None if B is None else [list(map(float, r)) for r in B]
        return linear(x, W, b, A, B, s)

    Wqkv, bqkv = blk["Wqkv"], [float(v) for v in blk["bqkv"]]
    u = layernorm(h, [float(v) for v in blk["ln1_g"]], [float(v) for v in blk["ln1_b"]], eps)
    q = lin(u, "q", _rows(Wqkv, 0, d), bqkv[0:d])
    k = lin(u, "k", _rows(Wqkv, d, 2 * d), bqkv[d:2 * d])
    v = lin(u, "v", _rows(Wqkv, 2 * d, 3 * d), bqkv[2 * d:3 * d])
    o = attention(q, k, v, n_head)
    ao = lin(o, "o", _rows(blk["Wo"], 0, d), [float(x) for x in blk["bo"]])
    h1 = [[h[t][i] + ao[t][i] for i in range(d)] for t in range(len(h))]
    u2 = layernorm(h1, [float(x) for x in blk["ln2_g"]], [float(x) for x in blk["ln2_b"]], eps)
    f = lin(u2, "fc", _rows(blk["Wfc"], 0, len(blk["Wfc"])), [float(x) for x in blk["bfc"]])
    g = [[gelu(x) for x in row] for row in f]
    mo = lin(g, "pr", _rows(blk["Wpr"], 0, d), [float(x) for x in blk["bpr"]])
    return [[h1[t][i] + mo[t][i] for i in range(d)] for t in range(len(h))]


def stack(h, blocks, adapters, n_head, s, eps):
    for blk, ad in zip(blocks, adapters):
        h = block(h, blk, ad, n_head, s, eps)
    return h


def fedavg(client_params, sample_counts):
    """out[j] = sum_i (n_i / sum n) x_i[j], written per element (Eq. 8-9)."""
    tot = float(sum(sample_counts))
    n = len(client_params[0])
    out = [0.0] * n
    for j in range(n):
        acc = 0.0
        for i in range(len(client_params)):
            acc += (float(sample_counts[i]) / tot) * float(client_params[i][j])
        out[j] = acc
    return out
