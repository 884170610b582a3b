"""The allocation-free variant of the single layer's backward (for callers that cannot allocate device
memory) against the entry point it is a variant of: same kernels, so the outputs must agree bit for bit
(and thereby to the 2e-2 bar of the bf16 path).  Two calls in a row on the library's own scratch array, the
second with a smaller input, so that whatever the first call left there is in the way of the second."""
import numpy as np
import pytest

from paper_2407_00952_amd import binding as B
from paper_2407_00952_amd import synth
from gpu_util import BF16_TOL, relerr, say

pytestmark = pytest.mark.gpu


def _both(T, n_in, n_out, r, seed):
    import torch
    c = synth.make_single_layer(T, n_in, n_out, r, seed=seed, quant=True)
    c["B"] = synth.round_bf16(c["B"] * 10)
    x, W, dy = (B.to_device_bf16(c[k]) for k in ("x", "W", "dy"))
    A = torch.from_numpy(c["A"]).cuda()
    Bm = torch.from_numpy(c["B"]).cuda()

    def outputs():
        return (torch.full((T, n_in), float("nan"), dtype=torch.bfloat16, device="cuda"),
                torch.full((r, n_in), float("nan"), dtype=torch.float32, device="cuda"),
                torch.full((n_out, r), float("nan"), dtype=torch.float32, device="cuda"))

    nws = B.slora_lora_linear_ws_bytes(B.DTYPE_BF16, T, n_in, n_out, r)
    assert 0 < nws <= B.NOALLOC_SCRATCH_BYTES
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    ref = outputs()
    B.slora_lora_linear_bwd(B.DTYPE_BF16, T, n_in, n_out, r, c["alpha"], x, dy, W, A, Bm, *ref, ws, nws)
    got = outputs()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.slora_lora_linear_bwd_noalloc(T, n_in, n_out, r, c["alpha"], x, dy, W, A, Bm, *got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for name, g, rf in zip(("dx", "dA", "dB"), got, ref):
        g, rf = g.float().cpu().numpy(), rf.float().cpu().numpy()
        assert np.all(np.isfinite(g)), name
        e = relerr(g, rf)
        say("   T=%d %s: rel diff %.1e, bitwise equal %s" % (T, name, e, np.array_equal(g, rf)))
        assert e <= BF16_TOL and np.array_equal(g, rf), name


def test_noalloc_backward_equals_the_workspace_backward():
    say("allocation-free single-layer backward, two calls in a row")
    _both(2048, 512, 768, 8, seed=901)
    _both(700, 320, 448, 3, seed=902)          # smaller, ragged tiles, lower rank


def test_noalloc_rejects_sizes_beyond_its_scratch():
    import torch
    t = torch.zeros(64, dtype=torch.float32, device="cuda")
    T, n = 65536, 4096
    assert B.slora_lora_linear_ws_bytes(B.DTYPE_BF16, T, n, n, 4) > B.NOALLOC_SCRATCH_BYTES
    with pytest.raises(B.SloraError) as e:
        B.slora_lora_linear_bwd_noalloc(T, n, n, 4, 32.0, t, t, t, t, t, t, t, t)
    assert e.value.code == B.SLORA_ENOSPC
