"""Pins of the loss-head oracle against things it does not define itself."""
import math

import numpy as np
import pytest

from oracle.loss_head import loss_head_fwd_bwd
from paper_2407_00952_amd import synth


def loop_loss(y, gamma, beta, eps, Wv, labels):
    """Independent loop-only statement of the loss (no numpy reductions, no backward)."""
    T, d = y.shape
    V = Wv.shape[0]
    total, n = 0.0, 0
    for t in range(T):
        if labels[t] < 0:
            continue
        mu = sum(float(y[t, i]) for i in range(d)) / d
        var = sum((float(y[t, i]) - mu) ** 2 for i in range(d)) / d
        rho = 1.0 / math.sqrt(var + eps)
        u = [(float(y[t, i]) - mu) * rho * float(gamma[i]) + float(beta[i]) for i in range(d)]
        logit = [sum(u[i] * float(Wv[v, i]) for i in range(d)) for v in range(V)]
        mx = max(logit)
        lse = mx + math.log(sum(math.exp(l - mx) for l in logit))
        total += lse - logit[labels[t]]
        n += 1
    return total / n


def small(seed=0, n_seq=2, S=6, d=8, V=11):
    inp = synth.make_loss_head_inputs(n_seq, S, d, vocab=V, seed=seed, quant=False)
    inp["Wv"] = inp["Wv"] * 25.0          # logits of order 1 so that the softmax is far from uniform
    return {k: (np.asarray(v, dtype=np.float64) if k != "labels" else v) for k, v in inp.items()}


def test_loss_matches_loop_twin():
    p = small(1)
    loss, loss_tok, _ = loss_head_fwd_bwd(p["y"], p["lnf_g"], p["lnf_b"], 1e-5, p["Wv"], p["labels"])
    ref = loop_loss(p["y"], p["lnf_g"], p["lnf_b"], 1e-5, p["Wv"], p["labels"])
    assert abs(loss - ref) < 1e-12 * max(1.0, abs(ref))
    assert np.all(loss_tok[p["labels"] < 0] == 0.0)
    assert abs(loss_tok.sum() / (p["labels"] >= 0).sum() - ref) < 1e-12


def test_gradient_matches_finite_differences_of_loop_twin():
    p = small(2, n_seq=1, S=5, d=6, V=7)
    _, _, dy = loss_head_fwd_bwd(p["y"], p["lnf_g"], p["lnf_b"], 1e-5, p["Wv"], p["labels"])
    h = 1e-6
    num = np.zeros_like(dy)
    for t in range(dy.shape[0]):
        for i in range(dy.shape[1]):
            yp, ym = p["y"].copy(), p["y"].copy()
            yp[t, i] += h
            ym[t, i] -= h
            num[t, i] = (loop_loss(yp, p["lnf_g"], p["lnf_b"], 1e-5, p["Wv"], p["labels"]) -
                         loop_loss(ym, p["lnf_g"], p["lnf_b"], 1e-5, p["Wv"], p["labels"])) / (2 * h)
    assert np.abs(dy - num).max() < 1e-8 * max(1.0, np.abs(num).max())
    assert np.abs(num).max() > 1e-3       # the check is not vacuous
    # unlabeled rows get no gradient at all
    assert np.all(dy[p["labels"] < 0] == 0.0)


def test_zero_vocabulary_matrix_gives_log_V():
    p = small(3)
    V = p["Wv"].shape[0]
    loss, loss_tok, dy = loss_head_fwd_bwd(p["y"], p["lnf_g"], p["lnf_b"], 1e-5, np.zeros_like(p["Wv"]), p["labels"])
    assert abs(loss - math.log(V)) < 1e-14
    assert np.allclose(loss_tok[p["labels"] >= 0], math.log(V), rtol=0, atol=1e-14)
    assert np.all(dy == 0.0)


def test_same_shift_of_every_vocabulary_row_changes_nothing():
    # adding one vector w to every row of Wv adds u.w to all logits of a token: softmax unchanged
    p = small(4)
    rng = np.random.default_rng(0)
    w = rng.standard_normal(p["Wv"].shape[1])
    a = loss_head_fwd_bwd(p["y"], p["lnf_g"], p["lnf_b"], 1e-5, p["Wv"], p["labels"])
    b = loss_head_fwd_bwd(p["y"], p["lnf_g"], p["lnf_b"], 1e-5, p["Wv"] + w[None, :], p["labels"])
    assert abs(a[0] - b[0]) < 1e-12
    assert np.abs(a[2] - b[2]).max() < 1e-12


def test_gradient_rows_sum_to_zero_and_scale_with_label_count():
    p = small(5, n_seq=3)
    _, _, dy = loss_head_fwd_bwd(p["y"], p["lnf_g"], p["lnf_b"], 1e-5, p["Wv"], p["labels"])
    # LayerNorm removes the row mean on the way back, for any eps
    assert np.abs(dy.sum(axis=1)).max() < 1e-12
    # dropping the labels of the last sequence rescales the other rows by n_old / n_new
    S = 6
    lab2 = p["labels"].copy()
    lab2[-S:] = -1
    _, _, dy2 = loss_head_fwd_bwd(p["y"], p["lnf_g"], p["lnf_b"], 1e-5, p["Wv"], lab2)
    n1, n2 = (p["labels"] >= 0).sum(), (lab2 >= 0).sum()
    assert n2 < n1
    assert np.abs(dy2[:-S] * n2 - dy[:-S] * n1).max() < 1e-12
    assert np.all(dy2[-S:] == 0.0)


def test_single_token_closed_form():
    # d = 2: LayerNorm (eps = 0) maps any row with y0 > y1 to (+1, -1); with gamma = 1, beta = 0 and
    # Wv = [[a, 0], [0, a]] the logits are (a, -a): loss = log(1 + exp(-2a)) for label 0
    a = 0.7
    y = np.array([[3.0, 1.0]])
    loss, _, dy = loss_head_fwd_bwd(y, np.ones(2), np.zeros(2), 0.0, np.array([[a, 0.0], [0.0, a]]), np.array([0]))
    assert abs(loss - math.log1p(math.exp(-2 * a))) < 1e-14
    # the normalised row does not move under small changes of y, so the gradient is zero
    assert np.abs(dy).max() < 1e-12


def test_all_unlabeled_is_an_error():
    p = small(6)
    with pytest.raises(ValueError):
        loss_head_fwd_bwd(p["y"], p["lnf_g"], p["lnf_b"], 1e-5, p["Wv"], -np.ones_like(p["labels"]))


def test_generator_label_structure():
    inp = synth.make_loss_head_inputs(4, 64, 16, vocab=101, seed=9)
    lab = inp["labels"].reshape(4, 64)
    for s in range(4):
        c = int((lab[s] < 0).sum())
        assert 16 <= c < 32
        assert np.all(lab[s, :c] == -1) and np.all(lab[s, c:] >= 0) and np.all(lab[s, c:] < 101)
    again = synth.make_loss_head_inputs(4, 64, 16, vocab=101, seed=9)
    assert all(np.array_equal(inp[k], again[k]) for k in inp)
