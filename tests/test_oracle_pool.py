"""The worker-pool wrapper used by the full-size GPU parity test gives what the plain oracle gives."""
import numpy as np

from oracle import slora_oracle as so
from oracle_pool import oracle_round
from paper_2407_00952_amd import synth


def test_pool_equals_serial_round():
    cfg = synth.tiny_config(d_model=64, n_head=1, d_ff=128, n_blocks=2, lora_r=2, lora_proj=("q", "v", "pr"),
                            n_clients=2, batch=2, seq_len=64)
    inp = synth.make_stack_inputs(cfg)
    orc = so.ServerOracle(inp["blocks"], inp["adapters"], cfg.n_head, cfg.lora_alpha, cfg.lora_r, cfg.ln_eps)
    Y = orc.fwd(inp["clients"])
    dX = np.concatenate(orc.bwd(inp["dY"]), axis=0)
    seen = {}
    tot = oracle_round(cfg, workers=2, on_result=lambda n, y, dx: seen.__setitem__(n, (y, dx)))
    assert sorted(seen) == list(range(cfg.n_seq))
    for n, (y, dx) in seen.items():
        assert np.array_equal(y, Y[n]) and np.array_equal(dx, dX[n])
    for l, gl in enumerate(orc.grads):
        for p, (dA, dB) in gl.items():
            assert np.allclose(tot[l][p][0], dA, rtol=1e-13, atol=0) and np.allclose(tot[l][p][1], dB, rtol=1e-13, atol=0)
    # a subset: gradients are the sum over exactly those sequences
    sub = oracle_round(cfg, seqs=[1, 3], workers=1)
    ref = None
    X = np.concatenate(inp["clients"], axis=0)
    for n in (1, 3):
        _, _, g = orc.fwd_bwd_sequence(X[n], inp["dY"][n])
        ref = g if ref is None else [{p: (a[p][0] + b[p][0], a[p][1] + b[p][1]) for p in a} for a, b in zip(ref, g)]
    for l in range(cfg.n_blocks):
        for p in cfg.lora_proj:
            assert np.array_equal(sub[l][p][0], ref[l][p][0]) and np.array_equal(sub[l][p][1], ref[l][p][1])
