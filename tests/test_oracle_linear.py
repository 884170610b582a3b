"""Pins for the oracle's LoRA-adapted linear layer (SplitLoRA Sec. II-C: W + dW, rank-r product)."""
import numpy as np
import torch

from oracle import slora_oracle as so
from paper_2407_00952_amd import synth


def _case(T=37, n_in=24, n_out=40, r=3, seed=0, bias=True):
    c = synth.make_single_layer(T, n_in, n_out, r, 32.0, seed=seed, bias=bias)
    return {k: (None if v is None else np.asarray(v, dtype=np.float64) if isinstance(v, np.ndarray) else v)
            for k, v in c.items()}


def test_zero_B_equals_base_output_bitwise():
    c = _case()
    s = c["alpha"] / c["r"]
    y0, _ = so.lora_linear_fwd(c["x"], c["W"], c["b"], None, None, s)
    y1, z = so.lora_linear_fwd(c["x"], c["W"], c["b"], c["A"], np.zeros_like(c["B"]), s)
    assert z is not None and np.abs(z).max() > 0
    assert np.array_equal(y0, y1)
    # and the input gradient too; dA must vanish, dB must not
    dx0, _, _ = so.lora_linear_bwd(c["x"], c["dy"], c["W"], None, None, s)
    dx1, dA, dB = so.lora_linear_bwd(c["x"], c["dy"], c["W"], c["A"], np.zeros_like(c["B"]), s)
    assert np.array_equal(dx0, dx1)
    assert np.all(dA == 0.0) and np.abs(dB).max() > 0


def test_merged_weight_identity():
    """y = x (W + s B A)^T + b, and the adapter gradients are the chain rule through the dense dW."""
    c = _case(seed=1)
    s = c["alpha"] / c["r"]
    y, _ = so.lora_linear_fwd(c["x"], c["W"], c["b"], c["A"], c["B"], s)
    Wm = c["W"] + s * c["B"] @ c["A"]
    assert np.allclose(y, c["x"] @ Wm.T + c["b"], rtol=0, atol=1e-12)
    dx, dA, dB = so.lora_linear_bwd(c["x"], c["dy"], c["W"], c["A"], c["B"], s)
    dW = c["dy"].T @ c["x"]                       # dense weight gradient, test only
    assert np.allclose(dx, c["dy"] @ Wm, rtol=0, atol=1e-12)
    assert np.allclose(dA, s * c["B"].T @ dW, rtol=0, atol=1e-10)
    assert np.allclose(dB, s * dW @ c["A"].T, rtol=0, atol=1e-10)


def test_against_torch_autograd():
    c = _case(seed=2)
    s = c["alpha"] / c["r"]
    t = {k: torch.tensor(c[k], dtype=torch.float64, requires_grad=k in ("x", "A", "B"))
         for k in ("x", "W", "b", "A", "B", "dy")}
    y = torch.nn.functional.linear(t["x"], t["W"], t["b"]) + s * torch.nn.functional.linear(
        torch.nn.functional.linear(t["x"], t["A"]), t["B"])
    (y * t["dy"]).sum().backward()
    yo, _ = so.lora_linear_fwd(c["x"], c["W"], c["b"], c["A"], c["B"], s)
    dx, dA, dB = so.lora_linear_bwd(c["x"], c["dy"], c["W"], c["A"], c["B"], s)
    assert np.allclose(yo, y.detach().numpy(), rtol=0, atol=1e-12)
    assert np.allclose(dx, t["x"].grad.numpy(), rtol=0, atol=1e-12)
    assert np.allclose(dA, t["A"].grad.numpy(), rtol=0, atol=1e-10)
    assert np.allclose(dB, t["B"].grad.numpy(), rtol=0, atol=1e-10)


def test_no_bias_and_rank_one():
    c = _case(r=1, bias=False, seed=3)
    s = c["alpha"] / c["r"]
    y, z = so.lora_linear_fwd(c["x"], c["W"], None, c["A"], c["B"], s)
    assert z.shape == (37, 1)
    # rank one: the low-rank term is an outer product per token
    lo = s * np.outer(c["x"] @ c["A"][0], c["B"][:, 0])
    assert np.allclose(y, c["x"] @ c["W"].T + lo, rtol=0, atol=1e-12)


def test_planted_mistakes_are_caught():
    """The pins above must fail for plausible slips: wrong scale, transposed factor, dropped term."""
    c = _case(seed=4, n_in=24, n_out=24)
    s = c["alpha"] / c["r"]
    y, _ = so.lora_linear_fwd(c["x"], c["W"], c["b"], c["A"], c["B"], s)
    Wm = c["W"] + s * c["B"] @ c["A"]
    good = c["x"] @ Wm.T + c["b"]
    wrong_scale = c["x"] @ (c["W"] + c["alpha"] * c["B"] @ c["A"]).T + c["b"]
    transposed = c["x"] @ (c["W"] + s * (c["B"] @ c["A"]).T).T + c["b"]
    no_bias = c["x"] @ Wm.T
    for bad in (wrong_scale, transposed, no_bias):
        assert np.abs(bad - good).max() > 1e-3
    assert np.abs(y - good).max() < 1e-12
