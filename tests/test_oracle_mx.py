"""Pins for oracle/mx.py (MXFP8 conversion and the quantised linear).

What fixes the oracle here: the format constants and hand-worked blocks of the OCP MX v1.0
specification (tests/golden/mx_examples.txt), torch's own float8_e4m3fn cast as an independent
round-to-nearest-even implementation, a brute-force nearest-value search over all codes, and
properties that follow from the definition (scale window, idempotence, exactness on representable
data, reduction of the linear layer to a plain matmul)."""
import os

import numpy as np
import pytest
import torch

from oracle import mx

GOLD = os.path.join(os.path.dirname(__file__), "golden", "mx_examples.txt")


def _gold():
    e4, e8, blocks = [], [], []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        kind, rest = line.split(None, 1)
        if kind == "E4M3":
            c, v = rest.split()
            e4.append((int(c, 16), float(v)))
        elif kind == "E8M0":
            c, v = rest.split()
            e8.append((int(c), int(v)))
        elif kind == "BLOCK":
            vals, sc, codes = [p.strip() for p in rest.split("|")]
            blocks.append(([float(t) for t in vals.split()], int(sc), [int(t, 16) for t in codes.split()]))
    return e4, e8, blocks


def test_format_constants_from_the_specification():
    e4, e8, _ = _gold()
    for c, v in e4:
        assert mx.e4m3_decode(np.uint8(c)) == v
    for c, lg in e8:
        assert mx.e8m0_decode(c) == 2.0 ** lg
    assert np.isnan(mx.e4m3_decode(np.uint8(0x7F))) and np.isnan(mx.e4m3_decode(np.uint8(0xFF)))
    assert np.signbit(mx.e4m3_decode(np.uint8(0x80))) and mx.e4m3_decode(np.uint8(0x80)) == 0.0
    # monotone over the positive codes, 126 distinct positive finite values
    pos = mx.e4m3_decode(np.arange(127, dtype=np.uint8))
    assert (np.diff(pos) > 0).all()


def test_hand_worked_blocks():
    _, _, blocks = _gold()
    for vals, sc, codes in blocks:
        x = np.zeros(32)
        x[:len(vals)] = vals
        q, s = mx.mx_quantize(x[None, :])
        assert int(s[0, 0]) == sc, (vals, s)
        want = np.zeros(32, dtype=np.uint8)
        want[:len(codes)] = codes
        np.testing.assert_array_equal(q[0], want)


def test_encode_inverts_decode_on_every_finite_code():
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    np.testing.assert_array_equal(mx.e4m3_encode(mx.e4m3_decode(codes)), codes)


def test_encode_matches_torch_float8_cast_in_range():
    rng = np.random.default_rng(0)
    v = np.concatenate([
        rng.uniform(-448, 448, 20000), rng.normal(0, 1, 20000), rng.normal(0, 0.01, 20000),
        # every midpoint between neighbouring values (the ties) and points just beside them
        (mx._POS[1:] + mx._POS[:-1]) / 2, -(mx._POS[1:] + mx._POS[:-1]) / 2,
        np.nextafter((mx._POS[1:] + mx._POS[:-1]) / 2, 1e9), np.nextafter((mx._POS[1:] + mx._POS[:-1]) / 2, -1e9),
    ]).astype(np.float32)
    ref = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = mx.e4m3_encode(v.astype(np.float64))
    np.testing.assert_array_equal(got, ref)


def test_encode_is_the_nearest_value_with_ties_to_even_and_saturation():
    rng = np.random.default_rng(1)
    v = np.concatenate([rng.uniform(-520, 520, 3000), rng.normal(0, 0.02, 3000)])
    finite = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    table = mx.e4m3_decode(finite)
    got = mx.e4m3_encode(v)
    for x, c in zip(v, got):
        d = np.abs(table - x)
        best = d.min()
        assert abs(mx.e4m3_decode(c) - x) == best
        cands = finite[d == best]
        if len(cands) > 1 and x != 0:           # a tie: the even code wins
            assert c % 2 == 0
    # beyond the largest normal: clamp, never NaN
    np.testing.assert_array_equal(mx.e4m3_encode(np.array([449.0, 464.0, 480.0, 511.9, -1e6])),
                                  np.array([0x7E, 0x7E, 0x7E, 0x7E, 0xFE], dtype=np.uint8))


def test_block_scale_window_and_error_bound():
    rng = np.random.default_rng(2)
    x = (rng.normal(0, 1, (64, 256)) * 10.0 ** rng.uniform(-6, 6, (64, 1))).astype(np.float32).astype(np.float64)
    q, s = mx.mx_quantize(x)
    X = mx.e8m0_decode(s)
    amax = np.abs(x.reshape(64, 8, 32)).max(axis=-1)
    # shared_exp = floor(log2 amax) - 8  <=>  amax / X in [256, 512)
    assert ((amax / X >= 256) & (amax / X < 512)).all()
    d = mx.mx_dequantize(q, s)
    err = np.abs(d - x).reshape(64, 8, 32)
    # elements below 448 X are rounded to nearest: half a spacing, spacing <= 2^-3 of the value's binade
    # (or 2^-9 X for subnormals); elements in (448 X, 512 X) are clamped: error < 64 X
    bound = np.maximum(np.abs(x).reshape(64, 8, 32) * 2.0 ** -4, X[..., None] * 2.0 ** -10)
    clamped = np.abs(x).reshape(64, 8, 32) > 448 * X[..., None]
    assert (err[~clamped] <= bound[~clamped]).all()
    assert (err[clamped] < 64 * np.broadcast_to(X[..., None], err.shape)[clamped]).all()


def test_quantise_is_idempotent_and_exact_on_representable_data():
    rng = np.random.default_rng(3)
    x = rng.normal(0, 3, (16, 128))
    q, s = mx.mx_quantize(x)
    d = mx.mx_dequantize(q, s)
    q2, s2 = mx.mx_quantize(d)
    np.testing.assert_array_equal(q2, q)
    np.testing.assert_array_equal(s2, s)
    # data that is already an E4M3 value times a power of two per block survives unchanged
    codes = rng.integers(0, 127, (16, 128)).astype(np.uint8)
    codes[:, ::32] = 0x7E                          # pin every block's maximum to 448
    sc = rng.integers(100, 150, (16, 4)).astype(np.uint8)
    y = mx.mx_dequantize(codes, sc)
    qy, sy = mx.mx_quantize(y)
    np.testing.assert_array_equal(qy, codes)
    np.testing.assert_array_equal(sy, sc)


def test_linear_reduces_to_a_plain_matmul():
    rng = np.random.default_rng(4)
    M, K, N = 5, 64, 7
    xq = rng.integers(0, 127, (M, K)).astype(np.uint8) | (rng.integers(0, 2, (M, K)).astype(np.uint8) << 7)
    wq = rng.integers(0, 127, (N, K)).astype(np.uint8) | (rng.integers(0, 2, (N, K)).astype(np.uint8) << 7)
    xs = rng.integers(120, 134, (M, K // 32)).astype(np.uint8)
    ws = rng.integers(120, 134, (N, K // 32)).astype(np.uint8)
    b = rng.normal(0, 1, N)
    y = mx.mx_linear(xq, xs, wq, ws, b)
    # the same by explicit loops over blocks and elements
    ref = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for kb in range(K // 32):
                sx, sw = 2.0 ** (int(xs[m, kb]) - 127), 2.0 ** (int(ws[n, kb]) - 127)
                for k in range(32):
                    acc += (mx.E4M3[xq[m, kb * 32 + k]] * sx) * (mx.E4M3[wq[n, kb * 32 + k]] * sw)
            ref[m, n] = acc + b[n]
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)
    # all-ones data with unit scales: every output is K
    one = np.full((M, K), 0x38, dtype=np.uint8)
    u = np.full((M, K // 32), 127, dtype=np.uint8)
    np.testing.assert_array_equal(mx.mx_linear(one, u, one[:3], u[:3]), np.full((M, 3), float(K)))


def test_rejects_bad_input():
    with pytest.raises(ValueError):
        mx.mx_quantize(np.zeros((2, 48)))
    with pytest.raises(ValueError):
        mx.mx_quantize(np.array([[np.inf] + [0.0] * 31]))


def _representable(rng, shape):
    """values that MXFP8 stores exactly: E4M3 codes times a per-block power of two, every block's largest
    magnitude 448 so that quantising returns the same codes"""
    codes = rng.integers(0, 127, shape).astype(np.uint8) | (rng.integers(0, 2, shape).astype(np.uint8) << 7)
    codes[..., ::32] = 0x7E
    sc = rng.integers(115, 125, shape[:-1] + (shape[-1] // 32,)).astype(np.uint8)
    return mx.mx_dequantize(codes, sc)


def test_lora_linear_equals_the_exact_layer_on_representable_data():
    """where nothing is lost to quantisation the compressed layer IS the exact LoRA layer (pinned on its
    own in test_oracle_linear.py): catches a wrong transpose, a dropped term or a misplaced s"""
    from oracle import slora_oracle as so
    rng = np.random.default_rng(6)
    T, n_in, n_out, r, s = 24, 64, 96, 3, 32.0 / 3
    x = _representable(rng, (T, n_in))
    dy = _representable(rng, (T, n_out))
    # W must be representable along BOTH axes (it is quantised as W and as W^T): a power of two per
    # 32 x 32 tile times E4M3 values, every row and column of a tile reaching 448
    Wc = rng.integers(1, 127, (n_out, n_in)).astype(np.uint8)
    W = mx.e4m3_decode(Wc)
    for i in range(0, n_out, 32):
        for j in range(0, n_in, 32):
            tile = W[i:i + 32, j:j + 32]
            np.fill_diagonal(tile, 448.0)
            tile *= 2.0 ** rng.integers(-12, -6)
    b = rng.normal(0, 1, n_out)
    A = rng.normal(0, 0.1, (r, n_in)); B = rng.normal(0, 0.1, (n_out, r))
    y = mx.mx_lora_linear_fwd(x, W, b, A, B, s)
    y_ref, _ = so.lora_linear_fwd(x, W, b, A, B, s)
    np.testing.assert_allclose(y, y_ref, rtol=1e-12, atol=1e-12)
    dx, dA, dB = mx.mx_lora_linear_bwd(x, dy, W, A, B, s)
    dx_ref, dA_ref, dB_ref = so.lora_linear_bwd(x, dy, W, A, B, s)
    np.testing.assert_allclose(dx, dx_ref, rtol=1e-12, atol=1e-9)
    np.testing.assert_allclose(dA, dA_ref, rtol=1e-12, atol=1e-9)
    np.testing.assert_allclose(dB, dB_ref, rtol=1e-12, atol=1e-9)


def test_lora_linear_noise_budget_and_reductions():
    from oracle import slora_oracle as so
    from paper_2407_00952_amd import synth
    c = synth.make_single_layer(T=128, n_in=256, n_out=128, r=4, quant=True, bias=True)
    s = c["alpha"] / c["r"]
    y = mx.mx_lora_linear_fwd(c["x"], c["W"], c["b"], c["A"], c["B"], s)
    y_ref, _ = so.lora_linear_fwd(c["x"], c["W"], c["b"], c["A"], c["B"], s)
    dx, dA, dB = mx.mx_lora_linear_bwd(c["x"], c["dy"], c["W"], c["A"], c["B"], s)
    dx_ref, dA_ref, dB_ref = so.lora_linear_bwd(c["x"], c["dy"], c["W"], c["A"], c["B"], s)
    rms = lambda a, b: np.sqrt(((a - b) ** 2).mean() / (b ** 2).mean())
    # two operands with 2^-4/sqrt(3) relative element noise each: about 5 % of the product's rms
    assert 0.01 < rms(y, y_ref) < 0.07 and 0.01 < rms(dx, dx_ref) < 0.07
    # the adapter gradients never see the quantised operands
    np.testing.assert_allclose(dA, dA_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dB, dB_ref, rtol=1e-12, atol=1e-12)
    # without an adapter the layer is the quantised linear
    Z = np.zeros_like(c["B"])
    np.testing.assert_array_equal(mx.mx_lora_linear_fwd(c["x"], c["W"], c["b"], c["A"], Z, s),
                                  mx.mx_linear(*mx.mx_quantize(c["x"]), *mx.mx_quantize(c["W"]), c["b"]))


def test_bf16_round_matches_torch_and_cut_compress_composes():
    rng = np.random.default_rng(8)
    x = np.concatenate([rng.normal(0, 1, 5000), rng.normal(0, 1e-3, 5000), rng.normal(0, 1e3, 5000)])
    # exact ties between neighbouring bf16 values
    b = torch.from_numpy(x[:2000].astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    ties = b + np.ldexp(1.0, np.frexp(b)[1] - 9)
    x = np.concatenate([x, ties])
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(mx.bf16_round(x), ref)
    t = rng.normal(0, 2, (6, 64))
    q, s = mx.cut_compress(t)
    q2, s2 = mx.mx_quantize(ref_bf := torch.from_numpy(t).to(torch.bfloat16).to(torch.float64).numpy())
    np.testing.assert_array_equal(q, q2); np.testing.assert_array_equal(s, s2)
    # what the receiver sees differs from the tensor by the bf16 rounding plus one element step
    err = np.abs(mx.mx_dequantize(q, s) - t).max() / np.abs(t).max()
    assert err < 2.0 ** -4 + 2.0 ** -8


def _gold4():
    e2, blocks = [], []
    for line in open(GOLD):
        line = line.strip()
        if line.startswith("E2M1 "):
            _, c, v = line.split()
            e2.append((int(c, 16), float(v)))
        elif line.startswith("BLOCK4 "):
            vals, sc, codes = [p.strip() for p in line[len("BLOCK4 "):].split("|")]
            blocks.append(([float(t) for t in vals.split()], int(sc), [int(t, 16) for t in codes.split()]))
    return e2, blocks


def test_fp4_constants_worked_blocks_and_nearest():
    e2, blocks = _gold4()
    assert len(e2) == 8 and len(blocks) == 2
    for c, v in e2:
        assert mx.e2m1_decode(np.uint8(c)) == v
    for vals, sc, codes in blocks:
        x = np.zeros(32); x[:len(vals)] = vals
        q, s = mx.mx_quantize_fp4(x[None, :])
        assert int(s[0, 0]) == sc
        want = np.zeros(32, dtype=np.uint8); want[:len(codes)] = codes
        np.testing.assert_array_equal(q[0], want)
    # encode inverts decode on all 16 codes; brute-force nearest with the even code on ties; clamp at 6
    allc = np.arange(16, dtype=np.uint8)
    np.testing.assert_array_equal(mx.e2m1_encode(mx.e2m1_decode(allc)), allc)
    rng = np.random.default_rng(10)
    v = np.concatenate([rng.uniform(-8, 8, 4000), (mx._POS4[1:] + mx._POS4[:-1]) / 2, -(mx._POS4[1:] + mx._POS4[:-1]) / 2])
    got = mx.e2m1_encode(v)
    for x, c in zip(v, got):
        d = np.abs(mx.E2M1 - x)
        assert abs(mx.E2M1[c] - x) == d.min()
        if (d == d.min()).sum() > 1 and x != 0:
            assert c % 2 == 0
    # block window: max / scale in [4, 8); packing round trip; exactness on representable data
    x = (rng.normal(0, 1, (16, 128)) * 10.0 ** rng.uniform(-4, 4, (16, 1)))
    q, s = mx.mx_quantize_fp4(x)
    amax = np.abs(x.reshape(16, 4, 32)).max(axis=-1)
    r = amax / mx.e8m0_decode(s)
    assert ((r >= 4) & (r < 8)).all()
    np.testing.assert_array_equal(mx.unpack_fp4(mx.pack_fp4(q)), q)
    assert mx.pack_fp4(np.array([[0x1, 0xF, 0x7, 0x0]], dtype=np.uint8)).tolist() == [[0xF1, 0x07]]
    codes = rng.integers(0, 16, (8, 64)).astype(np.uint8); codes[:, ::32] = 0x7
    sc = rng.integers(110, 140, (8, 2)).astype(np.uint8)
    q2, s2 = mx.mx_quantize_fp4(mx.mx_dequantize_fp4(codes, sc))
    np.testing.assert_array_equal(q2 & 7, codes & 7)          # magnitudes (the sign of a zero element may differ)
    np.testing.assert_array_equal(s2, sc)
    # the linear with 4-bit weights against explicit loops
    xq = rng.integers(0, 127, (3, 64)).astype(np.uint8); xs = rng.integers(120, 130, (3, 2)).astype(np.uint8)
    y = mx.mx_linear_w4(xq, xs, codes, sc)
    ref = np.array([[sum(mx.E4M3[xq[m, k]] * 2.0 ** (int(xs[m, k // 32]) - 127) * mx.E2M1[codes[n, k]] * 2.0 ** (int(sc[n, k // 32]) - 127)
                         for k in range(64)) for n in range(8)] for m in range(3)])
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)


def test_mx_stack_oracle_reduces_to_the_exact_stack_and_stays_close():
    """(a) with operands MXFP8 stores exactly the compressed block IS the exact block; (b) on ordinary data
    the compressed stack stays within the noise budget of the exact one and its adapter gradients are the
    exact formulas applied to its own activations (checked by finite differences of the exact-adapter part)."""
    from oracle import slora_oracle as so
    from paper_2407_00952_amd import synth
    cfg = synth.tiny_config(d_model=128, n_head=2, d_ff=256, n_blocks=2, lora_r=4, lora_proj=("q", "v", "fc"),
                            n_clients=2, batch=1, seq_len=64)
    inp = synth.make_stack_inputs(cfg)
    exact = so.ServerOracle(inp["blocks"], inp["adapters"], cfg.n_head, cfg.lora_alpha, cfg.lora_r, cfg.ln_eps)
    comp = mx.make_mx_server_oracle(inp["blocks"], inp["adapters"], cfg.n_head, cfg.lora_alpha, cfg.lora_r, cfg.ln_eps)
    Ye, Yc = exact.fwd(inp["clients"]), comp.fwd(inp["clients"])
    dXe, dXc = exact.bwd(inp["dY"]), comp.bwd(inp["dY"])
    rel = lambda a, b: np.abs(a - b).max() / np.abs(b).max()
    assert 1e-4 < rel(Yc, Ye) < 0.1
    for a, b in zip(dXc, dXe):
        assert 1e-4 < rel(a, b) < 0.25
    for gl_c, gl_e in zip(comp.grads, exact.grads):
        for p in gl_e:
            assert rel(gl_c[p][0], gl_e[p][0]) < 0.3 and rel(gl_c[p][1], gl_e[p][1]) < 0.3
    # the linear-layer pair itself against the exact pair on representable operands
    rng = np.random.default_rng(12)
    x, dy = _representable(rng, (16, 64)), _representable(rng, (16, 96))
    Wc = mx.e4m3_decode(rng.integers(1, 127, (96, 64)).astype(np.uint8))
    for i in range(0, 96, 32):
        for j in range(0, 64, 32):
            t = Wc[i:i + 32, j:j + 32]; np.fill_diagonal(t, 448.0); t *= 2.0 ** -10
    A, B = rng.normal(0, 0.1, (3, 64)), rng.normal(0, 0.1, (96, 3))
    lin, ad = {"fc": (Wc, rng.normal(0, 1, 96))}, {"fc": (A, B)}
    np.testing.assert_allclose(mx._mx_lin_fwd(x, lin, ad, "fc", 2.5), so._lin_fwd(x, lin, ad, "fc", 2.5), rtol=1e-12, atol=1e-12)
    g1, g2 = {}, {}
    np.testing.assert_allclose(mx._mx_lin_bwd(x, dy, lin, ad, "fc", 2.5, g1), so._lin_bwd(x, dy, lin, ad, "fc", 2.5, g2),
                               rtol=1e-12, atol=1e-9)
    for k in (0, 1):
        np.testing.assert_allclose(g1["fc"][k], g2["fc"][k], rtol=1e-12, atol=1e-9)
