"""GPU parity of the single LoRA-adapted linear layer (SplitLoRA Sec. II-C) through the C ABI."""
import numpy as np
import pytest

from oracle import slora_oracle as so
from paper_2407_00952_amd import binding as B
from paper_2407_00952_amd import synth
from gpu_util import BF16_TOL, F32_TOL, relerr, say

pytestmark = pytest.mark.gpu


def _run_f32(c):
    import torch
    T, n_in = c["x"].shape
    n_out, r = c["W"].shape[0], c["r"]
    dev = {k: torch.from_numpy(np.ascontiguousarray(c[k], dtype=np.float32)).cuda()
           for k in ("x", "W", "A", "B", "dy")}
    bias = None if c["b"] is None else torch.from_numpy(c["b"]).cuda()
    nws = B.slora_lora_linear_ws_bytes(B.DTYPE_F32, T, n_in, n_out, r)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    y = torch.empty((T, n_out), dtype=torch.float32, device="cuda")
    dx = torch.empty((T, n_in), dtype=torch.float32, device="cuda")
    dA = torch.empty((r, n_in), dtype=torch.float32, device="cuda")
    dB = torch.empty((n_out, r), dtype=torch.float32, device="cuda")
    B.slora_lora_linear_fwd(B.DTYPE_F32, T, n_in, n_out, r, c["alpha"], dev["x"], dev["W"], bias, dev["A"],
                            dev["B"], y, ws, nws)
    B.slora_lora_linear_bwd(B.DTYPE_F32, T, n_in, n_out, r, c["alpha"], dev["x"], dev["dy"], dev["W"], dev["A"],
                            dev["B"], dx, dA, dB, ws, nws)
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in (y, dx, dA, dB)]


def _run_bf16(c):
    import torch
    T, n_in = c["x"].shape
    n_out, r = c["W"].shape[0], c["r"]
    x, W, dy = (B.to_device_bf16(c[k]) for k in ("x", "W", "dy"))
    bias = None if c["b"] is None else B.to_device_bf16(c["b"])
    A = torch.from_numpy(c["A"]).cuda()
    Bm = torch.from_numpy(c["B"]).cuda()
    nws = B.slora_lora_linear_ws_bytes(B.DTYPE_BF16, T, n_in, n_out, r)
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    y = torch.empty((T, n_out), dtype=torch.bfloat16, device="cuda")
    dx = torch.empty((T, n_in), dtype=torch.bfloat16, device="cuda")
    dA = torch.empty((r, n_in), dtype=torch.float32, device="cuda")
    dB = torch.empty((n_out, r), dtype=torch.float32, device="cuda")
    B.slora_lora_linear_fwd(B.DTYPE_BF16, T, n_in, n_out, r, c["alpha"], x, W, bias, A, Bm, y, ws, nws)
    torch.cuda.synchronize()
    B.slora_lora_linear_bwd(B.DTYPE_BF16, T, n_in, n_out, r, c["alpha"], x, dy, W, A, Bm, dx, dA, dB, ws, nws)
    torch.cuda.synchronize()
    return [B.from_device_bf16(y), B.from_device_bf16(dx), dA.cpu().numpy(), dB.cpu().numpy()]


def _oracle(c):
    s = c["alpha"] / c["r"]
    y, _ = so.lora_linear_fwd(c["x"], c["W"], c["b"], c["A"], c["B"], s)
    dx, dA, dB = so.lora_linear_bwd(c["x"], c["dy"], c["W"], c["A"], c["B"], s)
    return [y, dx, dA, dB]


def test_workload1_fp32():
    """x [1024,768], W [768,768], r = 4, alpha = 32: y, dx, dA, dB within 1e-4 of the fp64 oracle."""
    c = synth.make_single_layer()
    say("fp32 single layer 1024x768x768 r=4")
    got, ref = _run_f32(c), _oracle(c)
    for name, g, r in zip(("y", "dx", "dA", "dB"), got, ref):
        e = relerr(g, r)
        say("   %s rel err %.2e" % (name, e))
        assert e <= F32_TOL, (name, e)


@pytest.mark.parametrize("T,n_in,n_out,r,bias", [(100, 72, 40, 1, True), (257, 64, 200, 16, False)])
def test_fp32_ragged_shapes(T, n_in, n_out, r, bias):
    c = synth.make_single_layer(T, n_in, n_out, r, seed=7 + T, bias=bias)
    say("fp32 single layer", T, n_in, n_out, r)
    for name, g, ref in zip(("y", "dx", "dA", "dB"), _run_f32(c), _oracle(c)):
        assert relerr(g, ref) <= F32_TOL, name


def test_fp32_zero_B_is_bitwise_base():
    import torch
    c = synth.make_single_layer(300, 128, 192, 4, seed=11)
    c0 = dict(c); c0["B"] = np.zeros_like(c["B"])
    y_lora = _run_f32(c0)[0]
    # base layer: W only, expressed through the same call with A = 0 as well
    c1 = dict(c0); c1["A"] = np.zeros_like(c["A"])
    y_base = _run_f32(c1)[0]
    assert np.array_equal(y_lora, y_base)
    assert relerr(y_base, c["x"].astype(np.float64) @ c["W"].astype(np.float64).T) <= F32_TOL


@pytest.mark.parametrize("T,n_in,n_out,r,bias", [
    (1024, 768, 768, 4, False),      # workload 1 shapes, bf16 path
    (700, 320, 448, 3, True),        # ragged row tile, column tile and rank
    (256, 64, 64, 16, True),         # one tile, full rank
    (1300, 1024, 3072, 8, True),     # several column tiles
    (64, 128, 128, 1, False),
    (512, 768, 768, 2, True),        # the remaining ranks of the paper's sweep r in {1, 2, 4, 8} (Sec. IV)
    (512, 768, 2304, 8, False),
    # 34 chunks of 512 tokens, the last one ragged: each wavefront of the adapter-gradient reduction sums
    # nine chunks (the body with eight loads in flight plus its tail), the last wavefront seven (tail only)
    (16960, 256, 64, 4, True),
    (16960, 64, 256, 16, False),
])
def test_bf16_layer(T, n_in, n_out, r, bias):
    c = synth.make_single_layer(T, n_in, n_out, r, seed=100 + T + r, quant=True, bias=bias)
    c["B"] = synth.round_bf16(c["B"] * 10)       # make the low-rank term visible next to x W^T
    say("bf16 single layer", T, n_in, n_out, r)
    got, ref = _run_bf16(c), _oracle(c)
    for name, g, rf in zip(("y", "dx", "dA", "dB"), got, ref):
        e = relerr(g, rf)
        say("   %s rel err %.2e" % (name, e))
        assert e <= BF16_TOL, (name, e)


def test_bf16_zero_B_is_bitwise_base():
    c = synth.make_single_layer(512, 256, 320, 4, seed=21, quant=True, bias=True)
    c0 = dict(c); c0["B"] = np.zeros_like(c["B"])
    c1 = dict(c0); c1["A"] = np.zeros_like(c["A"])
    y_lora, dx_lora = _run_bf16(c0)[:2]
    y_base, dx_base = _run_bf16(c1)[:2]
    assert np.array_equal(y_lora, y_base) and np.array_equal(dx_lora, dx_base)


# The frozen product on its own (Sec. II-C without the adapter): this is the launch shape of the stack's
# products that have no rank-space branch, i.e. the 4-wave GEMM kernel with the plain-store epilogue.  One
# k-slab, an odd number of slabs, ragged row and column tiles, a single row, with and without bias.
@pytest.mark.parametrize("T,n_in,n_out,bias", [
    (700, 320, 448, True),
    (1, 64, 8, True),
    (257, 64, 264, False),
    (300, 704, 320, True),
    (1300, 1024, 3072, False),
    (4096, 4096, 1024, True),
])
def test_frozen_linear_bf16(T, n_in, n_out, bias):
    import torch
    c = synth.make_single_layer(T, n_in, n_out, 1, seed=300 + T + n_in, quant=True, bias=bias)
    x, W = B.to_device_bf16(c["x"]), B.to_device_bf16(c["W"])
    b = None if c["b"] is None else B.to_device_bf16(c["b"])
    y = torch.empty((T, n_out), dtype=torch.bfloat16, device="cuda")
    B.slora_frozen_linear_bf16(T, n_in, n_out, x, W, b, y)
    torch.cuda.synchronize()
    ref, _ = so.lora_linear_fwd(c["x"], c["W"], c["b"], np.zeros_like(c["A"]), np.zeros_like(c["B"]), 1.0)
    e = relerr(B.from_device_bf16(y), ref)
    say("frozen linear", T, n_in, n_out, "rel err %.2e" % e)
    # fp32 accumulation and one rounding to bf16: half a bf16 ulp of the largest output
    assert e <= 2.0 ** -8
