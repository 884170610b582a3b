"""GPU loss head (SplitLoRA Sec. III-B step a3: loss from the predicted value and the labels, and the
gradient the server's backward pass starts from) against the fp64 oracle.

Tolerances: dy and the vector of per-token losses, each as one tensor in the max-norm relative sense,
<= 2e-2 (bf16 operands and bf16 logits, fp32 accumulation and softmax).  In absolute terms a loss term
carries the rounding error of two bf16 logits (the largest one, through the log-sum-exp, and the labeled
one), each at most 2^-9 |logit| from the store plus about as much from the bf16 LayerNorm output:
|error| <= 2^-7 max|logit| is asserted as well.  The mean loss: 2e-3 relative.
"""
import numpy as np
import pytest

from oracle.loss_head import loss_head_fwd_bwd
from oracle.slora_oracle import layernorm_fwd
from paper_2407_00952_amd import binding as B
from paper_2407_00952_amd import synth
from gpu_util import relerr, say, BF16_TOL

pytestmark = pytest.mark.gpu

EPS = 1e-5


def gpu_loss_head(inp, d, V, max_tokens=None):
    import torch
    T = inp["y"].shape[0]
    nbytes = B.slora_loss_head_ws_bytes(max_tokens or T, d, V)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    Wv = B.to_device_bf16(inp["Wv"])
    B.slora_loss_head_prepare(d, V, Wv, ws, nbytes)
    y = B.to_device_bf16(inp["y"])
    g, b = B.to_device_bf16(inp["lnf_g"]), B.to_device_bf16(inp["lnf_b"])
    labels = torch.from_numpy(inp["labels"].astype(np.int32)).cuda()
    loss_tok = torch.full((T,), float("nan"), dtype=torch.float32, device="cuda")
    loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    dy = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    B.slora_loss_head(T, d, V, y, g, b, EPS, labels, ws, nbytes, loss_tok, loss, dy)
    torch.cuda.synchronize()
    return float(loss.cpu().numpy()[0]), loss_tok.cpu().numpy(), B.from_device_bf16(dy)


def logit_bound(y, inp):
    u, _ = layernorm_fwd(y, inp["lnf_g"], inp["lnf_b"], EPS)
    return 2.0 ** -7 * max(4.0, float(np.abs(u @ np.asarray(inp["Wv"], dtype=np.float64).T).max()))


def check_full(inp, d, V, label):
    loss, loss_tok, dy = gpu_loss_head(inp, d, V)
    lo, lto, dyo = loss_head_fwd_bwd(inp["y"], inp["lnf_g"], inp["lnf_b"], EPS, inp["Wv"], inp["labels"])
    e_dy = relerr(dy, dyo)
    e_tok = float(np.abs(loss_tok - lto).max())
    e_loss = abs(loss - lo) / abs(lo)
    say("   %s: dy %.2e, loss_tok abs %.2e, loss %.6f vs %.6f (rel %.1e)" % (label, e_dy, e_tok, loss, lo, e_loss))
    assert e_dy <= BF16_TOL
    assert relerr(loss_tok, lto) <= BF16_TOL
    assert e_tok <= logit_bound(inp["y"], inp)
    assert e_loss <= 2e-3
    assert np.all(loss_tok[inp["labels"] < 0] == 0.0)
    assert np.all(dy[inp["labels"] < 0] == 0.0)
    n = int((inp["labels"] >= 0).sum())
    assert abs(loss - loss_tok.astype(np.float64).sum() / n) <= 1e-6 * abs(lo)


@pytest.mark.parametrize("n_seq,S,d,V,scale", [(2, 96, 128, 1003, 1.0), (3, 64, 64, 50, 20.0), (1, 320, 256, 4099, 5.0)])
def test_loss_head_small(n_seq, S, d, V, scale):
    """Ragged vocabulary sizes (padding columns), several row tiles, peaked and flat softmax."""
    say("loss head n_seq=%d S=%d d=%d V=%d scale=%g" % (n_seq, S, d, V, scale))
    inp = synth.make_loss_head_inputs(n_seq, S, d, vocab=V, seed=synth.BASE_SEED + 77)
    inp["Wv"] = synth.round_bf16(inp["Wv"] * np.float32(scale))
    check_full(inp, d, V, "small")


def test_loss_head_spans_two_token_chunks():
    """More tokens than one pass holds (16384): the second chunk has a ragged row tile."""
    n_seq, S, d, V = 33, 512, 64, 520
    say("loss head two chunks T=%d" % (n_seq * S))
    inp = synth.make_loss_head_inputs(n_seq, S, d, vocab=V, seed=synth.BASE_SEED + 78)
    inp["Wv"] = synth.round_bf16(inp["Wv"] * np.float32(8.0))
    check_full(inp, d, V, "two chunks")


def test_loss_head_without_labels():
    inp = synth.make_loss_head_inputs(2, 64, 64, vocab=200, seed=5)
    inp["labels"][:] = -1
    inp["labels"][3] = 200          # out of range counts as "no label" too
    loss, loss_tok, dy = gpu_loss_head(inp, 64, 200)
    assert np.isnan(loss)
    assert np.all(loss_tok == 0.0) and np.all(dy == 0.0)


def test_loss_head_workload3_sampled_rows():
    """Workload 3's shape: 64 x 512 tokens, d = 1024, GPT-2's vocabulary of 50257.  The oracle runs on a
    sample of rows; a row's loss term does not depend on the other rows and its gradient only through the
    number of labeled tokens, so the oracle's result on the sample is rescaled by n_sample / n_all."""
    cfg = synth.CONFIGS[3]
    d, V = cfg.d_model, synth.GPT2_VOCAB
    say("loss head workload 3: T=%d d=%d V=%d" % (cfg.n_seq * cfg.seq_len, d, V))
    inp = synth.make_loss_head_inputs(cfg.n_seq, cfg.seq_len, d, vocab=V)
    loss, loss_tok, dy = gpu_loss_head(inp, d, V)
    T = inp["y"].shape[0]
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([rng.integers(0, T, size=40), [0, 1, 255, 256, 16383, 16384, T - 1]]))
    lab = inp["labels"][rows]
    assert (lab >= 0).any() and (lab < 0).any()
    _, lto, dyo = loss_head_fwd_bwd(inp["y"][rows], inp["lnf_g"], inp["lnf_b"], EPS, inp["Wv"], lab)
    n_all, n_s = int((inp["labels"] >= 0).sum()), int((lab >= 0).sum())
    dyo = dyo * (n_s / n_all)
    e_dy = relerr(dy[rows], dyo)
    e_tok = float(np.abs(loss_tok[rows] - lto).max())
    say("   sampled %d rows: dy %.2e, loss_tok abs %.2e, loss %.5f" % (rows.size, e_dy, e_tok, loss))
    assert e_dy <= BF16_TOL and relerr(loss_tok[rows], lto) <= BF16_TOL
    assert e_tok <= logit_bound(inp["y"][rows], inp)
    assert np.all(dy[inp["labels"] < 0] == 0.0) and np.all(loss_tok[inp["labels"] < 0] == 0.0)
    assert abs(loss - loss_tok.astype(np.float64).sum() / n_all) <= 1e-5 * abs(loss)
    # with N(0, 0.02^2) vocabulary rows the softmax is nearly flat: the loss sits just above log V
    assert abs(loss - np.log(V)) < 0.5
