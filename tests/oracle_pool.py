"""Run the fp64 stack oracle on many sequences at once (test harness only).

Sequences are independent in Y and in dx, and the adapter gradients of a round are the sum of the
per-sequence gradients (SplitLoRA Sec. III-B a3: one concatenated batch), so a full-size round of the
oracle is `fwd_bwd_sequence` on every sequence.  The oracle itself stays as plain as it is; this module
only spreads its calls over worker processes.  Workers are started with the "spawn" method (fresh
interpreters that never touch the GPU), rebuild the seeded inputs themselves and split the host's cores
between them.
"""
from __future__ import annotations

import multiprocessing as mp
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

_state = {}


def _init(cfg, threads):
    if ROOT not in sys.path:
        sys.path.insert(0, ROOT)
    from threadpoolctl import threadpool_limits
    from oracle import slora_oracle as so
    from paper_2407_00952_amd import synth
    _state["limit"] = threadpool_limits(limits=threads)
    inp = synth.make_stack_inputs(cfg)
    _state["orc"] = so.ServerOracle(inp["blocks"], inp["adapters"], cfg.n_head, cfg.lora_alpha, cfg.lora_r,
                                    cfg.ln_eps)
    _state["x"] = np.concatenate(inp["clients"], axis=0)
    _state["dY"] = inp["dY"]


def _one(n):
    y, dx, g = _state["orc"].fwd_bwd_sequence(_state["x"][n], _state["dY"][n])
    return n, y, dx, g


def oracle_round(cfg, seqs=None, workers=None, on_result=None):
    """fwd + bwd of the oracle on the sequences `seqs` (default: all) of synth.make_stack_inputs(cfg).

    Calls on_result(n, y [S,d], dx [S,d]) for each finished sequence (any order) and returns the adapter
    gradients summed over the sequences in index order: [{proj: (dA, dB)}] per block.
    """
    seqs = list(range(cfg.n_seq)) if seqs is None else list(seqs)
    cores = len(os.sched_getaffinity(0))
    if workers is None:
        workers = max(1, min(len(seqs), cores // 4, 8))
    threads = max(1, cores // workers)
    per_seq = {}
    ctx = mp.get_context("spawn")
    with ctx.Pool(workers, initializer=_init, initargs=(cfg, threads)) as pool:
        for n, y, dx, g in pool.imap_unordered(_one, seqs):
            per_seq[n] = g
            if on_result is not None:
                on_result(n, y, dx)
    total = None
    for n in seqs:
        g = per_seq[n]
        if total is None:
            total = [{p: (a[p][0].copy(), a[p][1].copy()) for p in a} for a in g]
        else:
            total = [{p: (a[p][0] + b[p][0], a[p][1] + b[p][1]) for p in a} for a, b in zip(total, g)]
    return total
