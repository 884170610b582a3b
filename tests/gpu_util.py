"""Helpers shared by the GPU parity tests: run the library on seeded inputs, run the oracle on the
same inputs, compare per tensor in the max-norm relative sense."""
import sys

import numpy as np

from oracle import slora_oracle as so
from paper_2407_00952_amd import binding as B
from paper_2407_00952_amd import synth

BF16_TOL = 2e-2      # bf16 storage, fp32 accumulation
F32_TOL = 1e-4


def relerr(got, ref):
    """max |got - ref| / max |ref|  (max-norm relative error of one tensor)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def oracle_of(cfg, inp, n_blocks=None):
    blocks = inp["blocks"][:n_blocks] if n_blocks else inp["blocks"]
    adapters = inp["adapters"][:n_blocks] if n_blocks else inp["adapters"]
    return so.ServerOracle(blocks, adapters, cfg.n_head, cfg.lora_alpha, cfg.lora_r, cfg.ln_eps)


def gpu_round(cfg, inp, clients=None, dY=None, server=None):
    """One forward + backward on the GPU.  Returns (server, Y [n_seq,S,d] f32, [dx_i], grads)."""
    import torch
    clients = inp["clients"] if clients is None else clients
    dY = inp["dY"] if dY is None else dY
    n_seq = sum(c.shape[0] for c in clients)
    srv = server or B.Server(cfg, inp["blocks"], inp["adapters"], max_seqs=max(n_seq, 1))
    xs = [B.to_device_bf16(c) for c in clients]
    y = torch.empty((n_seq, cfg.seq_len, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    dy = B.to_device_bf16(dY)
    dxs = [torch.empty_like(x) for x in xs]
    srv.fwd(xs, y)
    srv.bwd(dy, dxs)
    torch.cuda.synchronize()
    grads = [{p: (t[2].cpu().numpy().copy(), t[3].cpu().numpy().copy()) for p, t in ad.items()}
             for ad in srv.adapters]
    return srv, B.from_device_bf16(y), [B.from_device_bf16(t) for t in dxs], grads


def compare_round(cfg, inp, Y, dX, grads, tol=BF16_TOL, label=""):
    """Full oracle round on the same inputs; asserts every tensor within tol.  Returns the worst error."""
    orc = oracle_of(cfg, inp)
    Yo = orc.fwd(inp["clients"])
    dXo = orc.bwd(inp["dY"])
    worst = {}
    worst["Y"] = relerr(Y, Yo)
    for i, (a, b) in enumerate(zip(dX, dXo)):
        worst["dx%d" % i] = relerr(a, b)
    for l, gl in enumerate(orc.grads):
        for p, (dA, dB) in gl.items():
            worst["dA[%d,%s]" % (l, p)] = relerr(grads[l][p][0], dA)
            worst["dB[%d,%s]" % (l, p)] = relerr(grads[l][p][1], dB)
    bad = {k: v for k, v in worst.items() if not v <= tol}
    top = sorted(worst.items(), key=lambda kv: -kv[1])[:4]
    say("   %s worst errors: %s" % (label, ", ".join("%s=%.2e" % kv for kv in top)))
    assert not bad, bad
    return max(worst.values())
