"""Pins for the oracle's client-adapter aggregation (SplitLoRA step b2, Eq. 8-9) and SGD (Eq. 4-5)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import brute, cref
from oracle import slora_oracle as so
from paper_2407_00952_amd import synth


def test_matches_numpy_average_and_loops():
    vecs, counts = synth.make_fedavg_inputs(n_clients=7, n_params=513)
    out = so.fedavg(vecs, counts)
    ref = np.average(np.stack([v.astype(np.float64) for v in vecs]), axis=0, weights=counts.astype(np.float64))
    assert np.allclose(out, ref, rtol=1e-13, atol=1e-16)
    assert np.allclose(out[:40], brute.fedavg([v[:40] for v in vecs], counts.tolist()), rtol=1e-13, atol=1e-16)


def test_identities():
    vecs, counts = synth.make_fedavg_inputs(n_clients=5, n_params=300)
    x = vecs[0].astype(np.float64)
    # identical adapters come back unchanged, up to K roundings of the weights
    out = so.fedavg([x] * 5, counts)
    assert np.all(np.abs(out - x) <= 5 * 2.0 ** -52 * np.abs(x))
    # exact when K is a power of two with equal counts
    assert np.array_equal(so.fedavg([x] * 4, [10, 10, 10, 10]), x)
    # K = 1, and counts (n,0,...,0)
    assert np.array_equal(so.fedavg([x], [17]), x)
    assert np.array_equal(so.fedavg(vecs, [9, 0, 0, 0, 0]), x)
    # permutation invariance to rounding
    perm = [3, 1, 4, 0, 2]
    out1 = so.fedavg(vecs, counts)
    out2 = so.fedavg([vecs[i] for i in perm], counts[perm])
    assert np.allclose(out1, out2, rtol=0, atol=1e-15)
    # A and B are aggregated separately == element-wise on the flat vector: the result is NOT the
    # average of the products (checks we did not average dW)
    rng = np.random.default_rng(0)
    As = [rng.standard_normal((2, 6)) for _ in range(3)]; Bs = [rng.standard_normal((5, 2)) for _ in range(3)]
    n = [1, 2, 3]
    A, B = so.fedavg(As, n), so.fedavg(Bs, n)
    prod_avg = so.fedavg([b @ a for a, b in zip(As, Bs)], n)
    assert np.abs(B @ A - prod_avg).max() > 1e-2


def test_bad_counts():
    for bad in ([0, 0], [3, -1]):
        with pytest.raises(ValueError):
            so.fedavg([np.ones(3), np.ones(3)], bad)
        with pytest.raises(ValueError):
            cref.fedavg_weights_f32(bad)


def _nearest_f32_check(got, exact):
    """got (np.float32) is a correctly rounded value of the rational `exact`."""
    g = Fraction(float(got))
    lo = Fraction(float(np.nextafter(got, np.float32(-np.inf))))
    hi = Fraction(float(np.nextafter(got, np.float32(np.inf))))
    return abs(g - exact) <= abs(lo - exact) and abs(g - exact) <= abs(hi - exact)


def test_fixed_order_f32_is_a_chain_of_correctly_rounded_fmas():
    vecs, counts = synth.make_fedavg_inputs(n_clients=6, n_params=64)
    w = cref.fedavg_weights_f32(counts)
    # weights: float(double(n_i)/double(sum))
    tot = float(counts.sum())
    assert np.array_equal(w, np.array([np.float32(float(c) / tot) for c in counts]))
    out = cref.fedavg_f32(vecs, counts)
    for j in range(64):
        acc = np.float32(0.0)
        for i in range(6):
            exact = Fraction(float(w[i])) * Fraction(float(vecs[i][j])) + Fraction(float(acc))
            # exact rational value of this step, rounded once to fp32
            cand = np.float32(float(exact))
            if not _nearest_f32_check(cand, exact):     # double rounding through float64: fix up
                for c in (np.nextafter(cand, np.float32(-np.inf)), np.nextafter(cand, np.float32(np.inf))):
                    if _nearest_f32_check(c, exact):
                        cand = c
            assert _nearest_f32_check(cand, exact)
            acc = cand
        assert out[j] == acc, (j, out[j], acc)


def test_fixed_order_f32_close_to_fp64_and_identities():
    vecs, counts = synth.make_fedavg_inputs(n_clients=16, n_params=4096)
    out32 = cref.fedavg_f32(vecs, counts)
    out64 = so.fedavg(vecs, counts)
    scale = np.abs(out64).max()
    assert np.abs(out32 - out64).max() <= 1e-6 * scale
    x = vecs[0]
    assert np.array_equal(cref.fedavg_f32([x], [5]), x)
    assert np.array_equal(cref.fedavg_f32([x, x, x, x], [3, 3, 3, 3]), x)
    assert np.array_equal(cref.fedavg_f32(vecs[:3], [7, 0, 0]), x)
    same = cref.fedavg_f32([x] * 16, counts)
    assert np.all(np.abs(same - x) <= 16 * 2.0 ** -23 * np.abs(x))


def test_sgd_f32_is_one_fma_per_element():
    rng = np.random.default_rng(3)
    p = rng.standard_normal(200).astype(np.float32); g = rng.standard_normal(200).astype(np.float32)
    lr = np.float32(2e-4)
    out = cref.sgd_f32(p, g, float(lr))
    for j in range(200):
        exact = Fraction(float(p[j])) - Fraction(float(lr)) * Fraction(float(g[j]))
        assert _nearest_f32_check(out[j], exact)
    assert np.abs(out - (p.astype(np.float64) - 2e-4 * g.astype(np.float64))).max() < 1e-6


def test_workload5_adapter_vector_size():
    # 6 client blocks, r = 16, six projections of GPT-2-medium: 294 912 floats per block
    assert synth.fedavg_param_count(synth.CONFIGS[5]) == 6 * 294912 == 1769472


# ---- AdamW variant of the adapter step (beyond the paper's plain SGD) ------------------------------
def test_adamw_oracle_matches_torch_optimizer():
    import torch
    rng = np.random.default_rng(11)
    p0 = rng.standard_normal(257)
    hp = dict(lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1)
    tp = torch.tensor(p0.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tp], **hp)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    for step in range(1, 6):
        g = rng.standard_normal(257) * (0.1 if step % 2 else 3.0)
        tp.grad = torch.tensor(g.copy(), dtype=torch.float64)
        opt.step()
        p, m, v = so.adamw_step(p, g, m, v, hp["lr"], hp["betas"][0], hp["betas"][1], hp["eps"],
                                hp["weight_decay"], step)
        assert np.allclose(p, tp.detach().numpy(), rtol=1e-12, atol=1e-14), step


def test_adamw_fixed_order_f32_close_to_oracle_and_first_step_closed_form():
    rng = np.random.default_rng(12)
    n = 1000
    p0 = rng.standard_normal(n).astype(np.float32)
    g = rng.standard_normal(n).astype(np.float32)
    z = np.zeros(n, dtype=np.float32)
    p1, m1, v1 = cref.adamw_f32(p0, g, z, z, 1e-2, 0.9, 0.999, 1e-8, 0.0, 1)
    # first step, no decay: m/(1-b1) = g, v/(1-b2) = g^2, so p moves by lr * sign(g) (up to eps)
    assert np.allclose(p1, p0 - 1e-2 * np.sign(g), rtol=0, atol=2e-7)
    p, m, v = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    pf, mf, vf = p0, z, z
    for step in range(1, 5):
        gs = (rng.standard_normal(n) * 0.5).astype(np.float32)
        p, m, v = so.adamw_step(p, gs, m, v, 2e-3, 0.9, 0.98, 1e-6, 0.05, step)
        pf, mf, vf = cref.adamw_f32(pf, gs, mf, vf, 2e-3, 0.9, 0.98, 1e-6, 0.05, step)
    assert np.abs(pf - p).max() <= 2e-6 * np.abs(p).max()
    assert np.abs(mf - m).max() <= 2e-6 * np.abs(m).max()
    assert np.abs(vf - v).max() <= 2e-6 * np.abs(v).max()
