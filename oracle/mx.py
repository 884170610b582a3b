"""Plain CPU oracle for the compressed (microscaling fp8) frozen linear and cut-layer traffic.

THIS IS TEST INFRASTRUCTURE (see slora_oracle.py): slow, plain, independent of the
HIP path, never imported by the product package.

What it follows.  SplitLoRA (arXiv 2407.00952) names quantisation of the model as the way
to a more storage-, communication- and computation-efficient framework (Sec. V-B) and
fixes no format.  The format taken here is the published OCP Microscaling (MX) v1.0
"MXFP8" one: a block of 32 consecutive elements along the contraction axis shares one
power-of-two scale (E8M0: an 8-bit biased exponent, value 2^(code-127), code 255 = NaN),
elements are FP8 E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no
infinities; S.1111.111 = NaN; largest finite value 448; subnormals m * 2^-9).

Conversion of a block V_1..V_32 (MX v1.0, Sec. 6.3):
    shared_exp = floor(log2(max_i |V_i|)) - emax_elem,     emax_elem = 8 for E4M3
    X = 2^shared_exp  (clamped to what E8M0 can hold)
    P_i = V_i / X rounded to the nearest E4M3 value, ties to even, values beyond the
          largest normal clamped to it
Readings where the specification leaves a choice:
  * a block whose largest magnitude is zero or below 2^-119 gets the smallest scale
    (code 0): with E the biased binary32 exponent of the maximum, the rule is code = max(E - 8, 0);
  * inputs are finite (bf16 activations and weights); NaN/Inf are not supported.
The scale is a power of two, so V_i / X is exact: every decision below is exact integer or
exact binary arithmetic and does not depend on the working precision.

The linear layer is then the plain definition on the dequantised values, in float64:
    y = deq(x) . deq(W)^T + bias
"""
from __future__ import annotations

import numpy as np

BLOCK = 32
E4M3_MAX = 448.0


def _e4m3_table():
    """value of each of the 256 codes, from the format definition (NaN for S.1111.111)"""
    t = np.empty(256, dtype=np.float64)
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 15 and m == 7:
            v = np.nan
        elif e == 0:
            v = m * 2.0 ** -9                       # subnormal: 0.m * 2^(1-7)
        else:
            v = (1.0 + m / 8.0) * 2.0 ** (e - 7)
        t[c] = -v if s else v
    return t


E4M3 = _e4m3_table()
# the 127 non-negative finite values in increasing order: code c (0..126) <-> value E4M3[c]
_POS = E4M3[:127].copy()


def e4m3_decode(codes):
    return E4M3[np.asarray(codes, dtype=np.uint8)]


def e4m3_encode(v):
    """nearest E4M3 code of each value: ties to the even code, saturating at +-448, sign of zero kept"""
    v = np.asarray(v, dtype=np.float64)
    a = np.abs(v)
    a = np.minimum(a, E4M3_MAX)
    hi = np.searchsorted(_POS, a, side="left")              # first value >= a
    hi = np.minimum(hi, 126)
    lo = np.maximum(hi - 1, 0)
    dlo, dhi = a - _POS[lo], _POS[hi] - a
    # consecutive codes are consecutive values, so "even mantissa" is "even code"
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    code = np.where(np.signbit(v), code | 0x80, code).astype(np.uint8)
    return np.where(np.isnan(v), np.uint8(0x7F), code).astype(np.uint8)


def e8m0_decode(codes):
    return np.ldexp(1.0, np.asarray(codes, dtype=np.int64) - 127)


def mx_quantize(x):
    """x [..., K] (K a multiple of 32) -> (codes uint8 [..., K], scales uint8 [..., K/32])"""
    x = np.asarray(x, dtype=np.float64)
    K = x.shape[-1]
    if K % BLOCK:
        raise ValueError("K must be a multiple of 32")
    if not np.isfinite(x).all():
        raise ValueError("non-finite input")
    xb = x.reshape(x.shape[:-1] + (K // BLOCK, BLOCK))
    amax = np.abs(xb).max(axis=-1)
    # floor(log2 amax) from the binary exponent (amax = m 2^e, m in [0.5, 1)); code = biased exponent - 8,
    # held at the ends of what E8M0 stores (code 0 also for the zero block)
    _, e = np.frexp(amax)
    scode = np.where(amax > 0, np.clip(e.astype(np.int64) - 1 + 127 - 8, 0, 254), 0)
    scaled = np.ldexp(xb, (127 - scode)[..., None])          # exact: division by a power of two
    codes = e4m3_encode(scaled).reshape(x.shape)
    return codes, scode.astype(np.uint8)


def mx_dequantize(codes, scales):
    codes = np.asarray(codes, dtype=np.uint8)
    K = codes.shape[-1]
    v = e4m3_decode(codes).reshape(codes.shape[:-1] + (K // BLOCK, BLOCK))
    return (v * e8m0_decode(scales)[..., None]).reshape(codes.shape)


def mx_linear(xq, xs, wq, ws, bias=None):
    """y [M,N] = deq(x)[M,K] . deq(W)[N,K]^T + bias, float64"""
    y = mx_dequantize(xq, xs) @ mx_dequantize(wq, ws).T
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    return y


def mx_lora_linear_fwd(x, W, bias, A, B, s):
    """LoRA-adapted linear layer (Sec. II-C) with the frozen product in MXFP8 and the adapter exact:
        y = deq(Q(x)) . deq(Q(W))^T + bias + s (x A^T) B^T
    x [T,in] and W [out,in] are quantised along the contraction axis `in`; the low-rank branch sees the
    unquantised x ("LoRA kept in higher precision")."""
    x, W = np.asarray(x, dtype=np.float64), np.asarray(W, dtype=np.float64)
    A, B = np.asarray(A, dtype=np.float64), np.asarray(B, dtype=np.float64)
    y = mx_linear(*mx_quantize(x), *mx_quantize(W), bias)
    return y + s * ((x @ A.T) @ B.T)


def mx_lora_linear_bwd(x, dy, W, A, B, s):
    """The backward pass taken by the compressed layer (no weight gradient: W is frozen):
        dx = deq(Q(dy)) . deq(Q(W^T))^T + s (dy B) A        both operands quantised along `out`
        dA = s (dy B)^T x            dB = s dy^T (x A^T)    from the unquantised x and dy
    W^T is quantised on its own (its blocks run along the other axis), so dx is the straight-through
    input gradient, not the exact derivative of the quantised forward."""
    x, dy, W = (np.asarray(t, dtype=np.float64) for t in (x, dy, W))
    A, B = np.asarray(A, dtype=np.float64), np.asarray(B, dtype=np.float64)
    dx = mx_linear(*mx_quantize(dy), *mx_quantize(W.T.copy()), None) + s * ((dy @ B) @ A)
    dA = s * (dy @ B).T @ x
    dB = s * dy.T @ (x @ A.T)
    return dx, dA, dB


def bf16_round(x):
    """nearest bfloat16 (8 significant bits), ties to even, of float64 values in bf16's normal range"""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                       # x = m 2^e, |m| in [0.5, 1)
    return np.ldexp(np.rint(m * 256.0), e - 8)


def cut_compress(t):
    """What crosses the cut in compressed form (activations of step a2, activation gradients of step a4,
    Sec. III-B): the tensor as it would have been sent, i.e. rounded to bf16, then MXFP8 along the feature
    axis.  Returns (codes, scales)."""
    return mx_quantize(bf16_round(t))


# ---- MXFP4: FP4 E2M1 elements (1 sign, 2 exponent bits with bias 1, 1 mantissa bit; no NaN, no Inf;
#      values 0, 0.5, 1, 1.5, 2, 3, 4, 6) under the same E8M0 block scale; emax_elem = 2 (MX v1.0 Sec. 5.3.3, 6.3).
#      Used for the frozen weights only (4.25 bits per weight).

def _e2m1_table():
    t = np.empty(16, dtype=np.float64)
    for c in range(16):
        s, e, m = c >> 3, (c >> 1) & 3, c & 1
        v = m * 0.5 if e == 0 else (1.0 + m / 2.0) * 2.0 ** (e - 1)
        t[c] = -v if s else v
    return t


E2M1 = _e2m1_table()
_POS4 = E2M1[:8].copy()


def e2m1_decode(codes):
    return E2M1[np.asarray(codes, dtype=np.uint8) & 0xF]


def e2m1_encode(v):
    """nearest E2M1 code: ties to the even code, saturating at +-6, sign of zero kept"""
    v = np.asarray(v, dtype=np.float64)
    a = np.minimum(np.abs(v), 6.0)
    hi = np.minimum(np.searchsorted(_POS4, a, side="left"), 7)
    lo = np.maximum(hi - 1, 0)
    dlo, dhi = a - _POS4[lo], _POS4[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return np.where(np.signbit(v), code | 0x8, code).astype(np.uint8)


def mx_quantize_fp4(x):
    """x [..., K] -> (codes uint8 [..., K] one E2M1 code per element, scales uint8 [..., K/32])"""
    x = np.asarray(x, dtype=np.float64)
    K = x.shape[-1]
    if K % BLOCK:
        raise ValueError("K must be a multiple of 32")
    if not np.isfinite(x).all():
        raise ValueError("non-finite input")
    xb = x.reshape(x.shape[:-1] + (K // BLOCK, BLOCK))
    amax = np.abs(xb).max(axis=-1)
    _, e = np.frexp(amax)
    scode = np.where(amax > 0, np.clip(e.astype(np.int64) - 1 + 127 - 2, 0, 254), 0)
    codes = e2m1_encode(np.ldexp(xb, (127 - scode)[..., None])).reshape(x.shape)
    return codes, scode.astype(np.uint8)


def pack_fp4(codes):
    """two codes per byte, the element with the even index in the low nibble"""
    c = np.asarray(codes, dtype=np.uint8)
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_fp4(packed):
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = p & 0xF
    out[..., 1::2] = p >> 4
    return out


def mx_dequantize_fp4(codes, scales):
    codes = np.asarray(codes, dtype=np.uint8)
    K = codes.shape[-1]
    v = e2m1_decode(codes).reshape(codes.shape[:-1] + (K // BLOCK, BLOCK))
    return (v * e8m0_decode(scales)[..., None]).reshape(codes.shape)


def mx_linear_w4(xq, xs, wq4, ws, bias=None):
    """y = deq(x) . deq(W)^T + bias with MXFP8 activations and MXFP4 weights (codes unpacked), float64"""
    y = mx_dequantize(xq, xs) @ mx_dequantize_fp4(wq4, ws).T
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    return y


# ---- the server stack with every frozen product in MXFP8 (a context of type SLORA_DTYPE_MXFP8) --------------
# Each linear layer of a block (q, k, v, o, fc, proj; Sec. III-A) is the compressed LoRA layer above, applied
# to the operand as the bf16 tensor it is stored as: Q(bf16(x)) forward, Q(bf16(dy)) and Q(W^T) backward.
# LayerNorm, attention, GELU and the residual stream are the uncompressed model's.

_W_CACHE = {}


def _quantized_weight(W, transposed):
    """deq(Q(W)) or deq(Q(W^T)), remembered by content: a stack evaluates the same frozen matrices once per
    sequence, and converting a few million weights in numpy takes longer than the product"""
    import hashlib
    W = np.ascontiguousarray(np.asarray(W, dtype=np.float64))
    key = (W.shape, bool(transposed), hashlib.blake2b(W.tobytes(), digest_size=16).digest())
    if key not in _W_CACHE:
        if len(_W_CACHE) > 512:
            _W_CACHE.clear()
        M = np.ascontiguousarray(W.T) if transposed else W
        _W_CACHE[key] = mx_dequantize(*mx_quantize(M))
    return _W_CACHE[key]


def _mx_product(x, W, transposed):
    """deq(Q(bf16(x))) . deq(Q(W or W^T))^T"""
    return mx_dequantize(*mx_quantize(bf16_round(x))) @ _quantized_weight(W, transposed).T


def _mx_lin_fwd(x, lin, adapters, name, s):
    W, b = lin[name]
    A, B = adapters.get(name, (None, None))
    x = np.asarray(x, dtype=np.float64)
    y = _mx_product(x, W, False)
    if b is not None:
        y = y + np.asarray(b, dtype=np.float64)[None, :]
    if A is not None:
        y = y + s * ((x @ np.asarray(A, dtype=np.float64).T) @ np.asarray(B, dtype=np.float64).T)
    return y


def _mx_lin_bwd(x, dy, lin, adapters, name, s, grads):
    W, _ = lin[name]
    A, B = adapters.get(name, (None, None))
    x, dy = np.asarray(x, dtype=np.float64), np.asarray(dy, dtype=np.float64)
    dx = _mx_product(dy, W, True)
    if A is not None:
        A, B = np.asarray(A, dtype=np.float64), np.asarray(B, dtype=np.float64)
        p = dy @ B
        dx = dx + s * (p @ A)
        grads[name] = (s * (p.T @ x), s * (dy.T @ (x @ A.T)))
    return dx


def make_mx_server_oracle(blocks, adapters, n_head, lora_alpha, lora_r, eps=1e-5):
    """the stack oracle of slora_oracle.py with the two functions above in place of the exact linear layer"""
    from .slora_oracle import ServerOracle

    class MxServerOracle(ServerOracle):
        lin_fwd = staticmethod(_mx_lin_fwd)
        lin_bwd = staticmethod(_mx_lin_bwd)

    return MxServerOracle(blocks, adapters, n_head, lora_alpha, lora_r, eps)
