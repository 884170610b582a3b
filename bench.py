#!/usr/bin/env python3
"""Benchmark of the server-side SplitLoRA round on one MI355X.

A step is one pass of the whole hot path over one synthetic batch: server forward over the
concatenated client activations, backward to the per-client activation gradients and the adapter
gradients, the SGD adapter step, and the FedAvg of the clients' adapter sets -- all through the C
ABI of libslora.so.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0          # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E peak


def model_flops_per_token(cfg):
    """Algorithmic work per token over the whole stack: frozen GEMMs forward + input-gradient (no
    weight gradient), causal attention forward + backward (lower triangle only), LoRA products."""
    d, f, S, L, r = cfg.d_model, cfg.d_ff, cfg.seq_len, cfg.n_blocks, cfg.lora_r
    gemm = 2 * 2 * (4 * d * d + 2 * d * f)
    attn = 6 * S * d
    lora = 6 * r * sum(sum(cfg.proj_shape(p)) for p in cfg.lora_proj)
    return L * gemm, L * attn, L * lora


def cpu_baseline(cfg, inp, budget_s=20.0):
    """The fp64 oracle, as it stands, timed on whole sequences of the same workload."""
    from oracle import slora_oracle as so
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    orc = so.ServerOracle(inp["blocks"], inp["adapters"], cfg.n_head, cfg.lora_alpha, cfg.lora_r, cfg.ln_eps)
    x = np.concatenate(inp["clients"][:1], axis=0)
    n, t0 = 0, time.perf_counter()
    while True:
        orc.fwd_bwd_sequence(x[n % x.shape[0]], inp["dY"][n % x.shape[0]])
        n += 1
        el = time.perf_counter() - t0
        if el > budget_s or n >= 4:
            break
    return {"value": n * cfg.seq_len / el, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d whole sequence(s) of %d tokens, forward+backward through all %d blocks, numpy fp64"
                      % (n, cfg.seq_len, cfg.n_blocks)}


def kernel_rooflines(step_fn, n_steps=3):
    """Per-kernel rates of the step's other kernels from HIP events around every launch (a separate pass after
    the timed region: bracketing ~370 launches per step with events would slow the timed step itself).
    HBM-bound kinds: algorithmic bytes / time against the HBM peak; attention: algorithmic flop / time against
    the bf16 MFMA peak."""
    import torch
    from paper_2407_00952_amd import binding as B
    kinds = {"ln_fwd_kernel": (B.PROF_LN_FWD, "hbm"), "ln_bwd_kernel": (B.PROF_LN_BWD, "hbm"),
             "lora_grad_partial_kernel": (B.PROF_LORA_GRAD, "hbm"), "sgd_table_kernel": (B.PROF_SGD, "hbm"),
             "attn_fwd_kernel": (B.PROF_ATTN_FWD, "mfma"), "attn_bwd_kernel(s)": (B.PROF_ATTN_BWD, "mfma")}
    mask = 0
    for k, _ in kinds.values():
        mask |= 1 << k
    B.slora_prof_enable(mask)
    for _ in range(n_steps):
        step_fn()
    torch.cuda.synchronize()
    hbm, mfma = {}, {}
    for name, (k, bound) in kinds.items():
        ms, work, n = B.slora_prof_read_kind(k)
        if n == 0 or ms <= 0:
            continue
        if bound == "hbm":
            gbs = work / (ms * 1e-3) / 1e9
            hbm[name] = {"achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                         "bytes_per_launch": work / n, "avg_launch_us": ms / n * 1e3, "launches_per_step": n // n_steps}
        else:
            tf = work / (ms * 1e-3) / 1e12
            mfma[name] = {"achieved": tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": tf / PEAK_BF16_TFLOPS,
                          "flop_per_launch": work / n, "avg_launch_us": ms / n * 1e3, "launches_per_step": n // n_steps}
    B.slora_prof_enable(0)
    return hbm, mfma


def fedavg_hbm_rate(stream, n_sets=4, reps=10):
    """Eq. (8)-(9) at workload 5's size (16 client adapter sets of 6 blocks, r = 16, all six projections:
    16 x 1 769 472 floats in, one set out = 120.3 MB per call) over `n_sets` DISTINCT buffer sets used in
    rotation, 481 MB in all, which no cache level holds: an HBM rate.  The same call repeated on one set
    (whose 120 MB stay in the last-level cache) is reported beside it."""
    import torch
    from paper_2407_00952_amd import binding as B
    from paper_2407_00952_amd import synth
    cfg5 = synth.CONFIGS[5]
    n, K = synth.fedavg_param_count(cfg5), cfg5.n_clients
    rng = np.random.Generator(np.random.PCG64(cfg5.seed + 1000))
    counts = rng.integers(100, 1001, size=K).astype(np.int64)
    g = torch.Generator(device="cuda")
    g.manual_seed(cfg5.seed + 1001)
    sets = [[torch.randn(n, device="cuda", generator=g) * 0.02 for _ in range(K)] for _ in range(n_sets)]
    outs = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(n_sets)]
    nbytes = 4.0 * (K + 1) * n

    def run(rotate):
        for i in range(n_sets):
            B.slora_fedavg(sets[i], counts, n, outs[i], stream)
        torch.cuda.synchronize()
        B.slora_prof_enable(1 << B.PROF_FEDAVG)
        for rep in range(reps):
            for i in range(n_sets):
                j = i if rotate else 0
                B.slora_fedavg(sets[j], counts, n, outs[j], stream)
        torch.cuda.synchronize()
        ms, work, cnt = B.slora_prof_read_kind(B.PROF_FEDAVG)
        B.slora_prof_enable(0)
        return work / (ms * 1e-3) / 1e9, ms / cnt * 1e3

    gbs, us = run(True)
    gbs_same, us_same = run(False)
    return {"kernel": "fedavg_kernel", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
            "bytes_per_launch": nbytes, "avg_launch_us": us, "clients": K, "params": n,
            "buffer_sets_rotated": n_sets, "working_set_bytes": nbytes * n_sets,
            "same_buffers_gb_s": gbs_same, "same_buffers_us": us_same,
            "what": "workload 5's aggregation; rotated over distinct buffer sets so that no cache holds them"}


def other_workload(w, lr, steps=5, warmup=2):
    """tokens/s and GEMM rate of another workload's step (forward + backward + adapter step), same protocol."""
    import torch
    from paper_2407_00952_amd import binding as B
    from paper_2407_00952_amd import synth
    cfg = synth.CONFIGS[w]
    inp = synth.make_stack_inputs(cfg)
    srv = B.Server(cfg, inp["blocks"], inp["adapters"])
    xs = [B.to_device_bf16(c) for c in inp["clients"]]
    y = torch.empty((cfg.n_seq, cfg.seq_len, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    dy = B.to_device_bf16(inp["dY"])
    dxs = [torch.empty_like(x) for x in xs]
    del inp
    stream = torch.cuda.current_stream().cuda_stream

    def step():
        srv.fwd(xs, y, stream)
        srv.bwd(dy, dxs, stream)
        srv.step(lr, stream)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    B.slora_prof_enable(1 << B.PROF_GEMM)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    el = (time.perf_counter() - t0) / steps
    gemm_ms, gemm_flop, launches = B.slora_prof_read()
    B.slora_prof_enable(0)
    srv.close()
    ach = gemm_flop / (gemm_ms * 1e-3) / 1e12
    fg, fa, fl = model_flops_per_token(cfg)
    return {"workload": "%s: %d blocks, d=%d, d_ff=%d, r=%d on %s, %d x %d x %d tokens" % (
                cfg.name, cfg.n_blocks, cfg.d_model, cfg.d_ff, cfg.lora_r, ",".join(cfg.lora_proj), cfg.n_clients,
                cfg.batch, cfg.seq_len),
            "tokens_per_step": cfg.tokens, "ms_per_step": el * 1e3, "tokens_per_s": cfg.tokens / el,
            "model_tflops": (fg + fa + fl) * cfg.tokens / el / 1e12,
            "gemm_tflops": ach, "gemm_frac_of_bf16_peak": ach / PEAK_BF16_TFLOPS, "steps": steps}


def recorded_gemm_traffic():
    """HBM bytes per GEMM launch from the committed rocprofv3 counter summary, or None when the GEMM
    source has changed since the counters were taken."""
    import hashlib
    import re
    path = os.path.join(ROOT, "profiles", "gemm_kernel_workload3_hbm_traffic.md")
    csrc = os.path.join(ROOT, "paper_2407_00952_amd", "csrc")
    try:
        text = open(path).read()
        # the kernel's source: main loop and launcher, and the epilogue it shares with the fp8 kernel
        h = hashlib.sha256()
        for name in ("gemm.hip", "gemm_epilogue.h"):
            h.update(open(os.path.join(csrc, name), "rb").read())
        sha = h.hexdigest()
        m_sha = re.search(r"gemm_source_sha256:\s*([0-9a-f]{64})", text)
        m_b = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text)
        if m_sha and m_b and m_sha.group(1) == sha:
            return float(m_b.group(1))
    except OSError:
        pass
    return None


PEAK_FP8_TFLOPS = 5000.0


def mxfp8_leg(cfg, stream):
    """The four frozen linears of a block's forward pass in MXFP8 (fp8 matrix cores, block scales), timed one
    by one on the workload's token count, next to the bf16 kernel on the same shapes; plus the conversion of
    one [T, d] activation tensor.  Separate from the metric's step, which stays bf16."""
    import torch
    from paper_2407_00952_amd import binding as B
    T, d, dff = cfg.tokens, cfg.d_model, cfg.d_ff
    g = torch.Generator(device="cuda")
    g.manual_seed(cfg.seed + 9000)

    def timed(fn, reps=10):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t_ = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t_) / reps * 1e3

    shapes, flop, ms_mx, ms_bf, ms_w4 = [], 0.0, 0.0, 0.0, 0.0
    quant = None
    for name, K, N in (("qkv", d, 3 * d), ("o", d, d), ("fc", d, dff), ("proj", dff, d)):
        x = torch.randn((T, K), device="cuda", generator=g).to(torch.bfloat16)
        W = (torch.randn((N, K), device="cuda", generator=g) * 0.02).to(torch.bfloat16)
        xq = torch.empty((T, K), dtype=torch.uint8, device="cuda")
        xs = torch.empty((T, K // 32), dtype=torch.uint8, device="cuda")
        wq = torch.empty((N, K), dtype=torch.uint8, device="cuda")
        ws = torch.empty((N, K // 32), dtype=torch.uint8, device="cuda")
        y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
        B.slora_mx_quantize(N, K, W, K, wq, ws, stream)
        tq = timed(lambda: B.slora_mx_quantize(T, K, x, K, xq, xs, stream))
        if name == "qkv":
            nbytes = T * K * (2 + 1) + T * K // 32
            quant = {"ms": tq, "bytes": nbytes, "gb_s": nbytes / (tq * 1e-3) / 1e9}
        t_mx = timed(lambda: B.slora_frozen_linear_mxfp8(T, K, N, xq, xs, wq, ws, None, y, stream))
        t_bf = timed(lambda: B.slora_frozen_linear_bf16(T, K, N, x, W, None, y, stream))
        wq4 = torch.empty((N, K // 2), dtype=torch.uint8, device="cuda")
        B.slora_mx_quantize_fp4(N, K, W, K, wq4, ws, stream)
        t_w4 = timed(lambda: B.slora_frozen_linear_mxfp8_w4(T, K, N, xq, xs, wq4, ws, None, y, stream))
        f = 2.0 * T * K * N
        shapes.append({"name": name, "K": K, "N": N, "mxfp8_us": t_mx * 1e3, "bf16_us": t_bf * 1e3,
                       "mxfp8_tflops": f / (t_mx * 1e-3) / 1e12, "w4_us": t_w4 * 1e3,
                       "w4_tflops": f / (t_w4 * 1e-3) / 1e12})
        ms_w4 += t_w4
        flop += f
        ms_mx += t_mx
        ms_bf += t_bf
        del x, W, xq, xs, wq, ws, y, wq4
    # the whole compressed LoRA layer (conversion of the activations, rank-space branch, fp8 product with the
    # bf16 low-rank tail; backward with the adapter gradients) on the qkv-sized and the FC-sized projection
    layer = []
    for name, K, N in (("q (d -> d)", d, d), ("fc (d -> d_ff)", d, dff)):
        r, alpha = cfg.lora_r, cfg.lora_alpha
        x = torch.randn((T, K), device="cuda", generator=g).to(torch.bfloat16)
        dyv = torch.randn((T, N), device="cuda", generator=g).to(torch.bfloat16)
        W = (torch.randn((N, K), device="cuda", generator=g) * 0.02).to(torch.bfloat16)
        A = torch.randn((r, K), device="cuda", generator=g) * 0.02
        Bm = torch.randn((N, r), device="cuda", generator=g) * 0.02
        nw, nws = B.slora_mx_weight_bytes(K, N), B.slora_mx_lora_linear_ws_bytes(T, K, N, r)
        packed = torch.empty(nw, dtype=torch.uint8, device="cuda")
        ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
        y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
        dx = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
        dA = torch.empty((r, K), dtype=torch.float32, device="cuda")
        dB = torch.empty((N, r), dtype=torch.float32, device="cuda")
        B.slora_mx_pack_weight(K, N, W, packed, nw, stream)
        t_f = timed(lambda: B.slora_mx_lora_linear_fwd(T, K, N, r, alpha, x, packed, None, A, Bm, y, ws, nws, stream))
        t_b = timed(lambda: B.slora_mx_lora_linear_bwd(T, K, N, r, alpha, x, dyv, packed, A, Bm, dx, dA, dB, ws, nws,
                                                       stream))
        f = 2.0 * T * K * N
        layer.append({"name": name, "fwd_us": t_f * 1e3, "bwd_us": t_b * 1e3,
                      "fwd_tflops": f / (t_f * 1e-3) / 1e12, "bwd_tflops": f / (t_b * 1e-3) / 1e12})
        del x, dyv, W, packed, ws, y, dx
    ach = flop / (ms_mx * 1e-3) / 1e12
    return {"lora_layer": layer, "what": "y = deq(x) deq(W)^T, MXFP8 operands (E4M3 + E8M0 per 32), bf16 out, T=%d" % T,
            "shapes": shapes, "tflops": ach, "peak": PEAK_FP8_TFLOPS, "frac": ach / PEAK_FP8_TFLOPS,
            "speedup_over_bf16_kernel": ms_bf / ms_mx, "quantize_activation": quant,
            "w4_tflops": flop / (ms_w4 * 1e-3) / 1e12,
            "w4_what": "the same products with MXFP4 (E2M1) weights, MXFP8 activations"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=3, help="2..5 (3 = GPT-2-medium split, the metric's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--loss-head", action="store_true",
                    help="put the loss head (final LayerNorm, vocabulary logits, cross-entropy -> dY) between "
                         "forward and backward inside the timed step; without it the step takes dY as given and "
                         "the loss head is timed on its own after the timed region")
    ap.add_argument("--no-legs", action="store_true",
                    help="skip the separately timed loss-head and client-side legs (profiles of the metric's step)")
    ap.add_argument("--no-workloads", action="store_true",
                    help="skip the other workloads (2, 4, 5) that are timed after the metric's own")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed steps, run a plain copy of known size (FedAvg with one client, "
                         "256 MiB in, 256 MiB out) so that HBM byte counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2407_00952_amd import binding as B
    from paper_2407_00952_amd import synth

    cfg = synth.CONFIGS[args.workload]
    torch.cuda.set_device(0)
    inp = synth.make_stack_inputs(cfg)
    srv = B.Server(cfg, inp["blocks"], inp["adapters"])
    xs = [B.to_device_bf16(c) for c in inp["clients"]]
    y = torch.empty((cfg.n_seq, cfg.seq_len, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    dy = B.to_device_bf16(inp["dY"])
    dxs = [torch.empty_like(x) for x in xs]
    # FedAvg leg: the K clients' adapter sets (client-side blocks, same rank and projections), fp32
    n_fed = synth.fedavg_param_count(cfg)
    fed_vecs, fed_counts = synth.make_fedavg_inputs(cfg.n_clients, n_params=None, cfg=cfg)
    fed_dev = [torch.from_numpy(v).cuda() for v in fed_vecs]
    fed_out = torch.empty(n_fed, dtype=torch.float32, device="cuda")
    lr = 2e-4
    stream = torch.cuda.current_stream().cuda_stream
    # loss head: GPT-2's vocabulary, labels with a context part that carries no label
    V = synth.GPT2_VOCAB
    if not args.no_legs or args.loss_head:
        lh = synth.make_loss_head_inputs(cfg.n_seq, cfg.seq_len, cfg.d_model, vocab=V)
        lh_bytes = B.slora_loss_head_ws_bytes(cfg.tokens, cfg.d_model, V)
        lh_ws = torch.empty(lh_bytes, dtype=torch.uint8, device="cuda")
        lh_Wv = B.to_device_bf16(lh["Wv"])
        B.slora_loss_head_prepare(cfg.d_model, V, lh_Wv, lh_ws, lh_bytes, stream)
        lh_g, lh_b = B.to_device_bf16(lh["lnf_g"]), B.to_device_bf16(lh["lnf_b"])
        lh_labels = torch.from_numpy(lh["labels"]).cuda()
        lh_tok = torch.empty(cfg.tokens, dtype=torch.float32, device="cuda")
        lh_loss = torch.empty(1, dtype=torch.float32, device="cuda")
        lh_dy = torch.empty_like(dy)
        del lh

    def loss_head():
        B.slora_loss_head(cfg.tokens, cfg.d_model, V, y, lh_g, lh_b, cfg.ln_eps, lh_labels, lh_ws, lh_bytes, lh_tok,
                          lh_loss, lh_dy, stream)

    def step():
        srv.fwd(xs, y, stream)
        if args.loss_head:
            loss_head()
            srv.bwd(lh_dy, dxs, stream)
        else:
            srv.bwd(dy, dxs, stream)
        srv.step(lr, stream)
        B.slora_fedavg(fed_dev, fed_counts, n_fed, fed_out, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.slora_prof_enable(1 << B.PROF_GEMM)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    gemm_ms, gemm_flop, launches = B.slora_prof_read()
    clock_mhz, clock_samples = B.slora_prof_read_clock()
    B.slora_prof_enable(0)
    hbm_kernels = attn_kernels = None
    if not args.no_legs:
        hbm_kernels, attn_kernels = kernel_rooflines(step)

    # the four calls of the step on their own (after the timed region, outside the GEMM statistics)
    phases = None
    if not args.no_legs:
        def timed(fn, reps=5):
            fn()
            torch.cuda.synchronize()
            t_ = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t_) / reps * 1e3

        phases = {"fwd_ms": timed(lambda: srv.fwd(xs, y, stream))}
        phases["fwd_bwd_ms"] = timed(lambda: (srv.fwd(xs, y, stream), srv.bwd(dy, dxs, stream)))
        phases["bwd_ms"] = phases["fwd_bwd_ms"] - phases["fwd_ms"]
        phases["fwd_bwd_step_ms"] = timed(lambda: (srv.fwd(xs, y, stream), srv.bwd(dy, dxs, stream), srv.step(lr, stream)))
        phases["adapter_step_ms"] = phases["fwd_bwd_step_ms"] - phases["fwd_bwd_ms"]
        phases["fedavg_ms"] = timed(lambda: B.slora_fedavg(fed_dev, fed_counts, n_fed, fed_out, stream), reps=20)
        phases["fedavg_bytes"] = 4 * n_fed * (cfg.n_clients + 1)

    # the loss head on its own (outside the timed region and outside the GEMM statistics above)
    legs = not args.no_legs
    lh_ms = cl_ms = float("nan")
    if legs:
        for _ in range(2):
            loss_head()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(5):
            loss_head()
        torch.cuda.synchronize()
        lh_ms = (time.perf_counter() - t1) / 5 * 1e3
    lh_flop = 4.0 * cfg.tokens * cfg.d_model * V

    # one client's share of a round (embedding + client-side blocks forward, backward, SGD step), on its own
    n_cb = synth.FEDAVG_CLIENT_BLOCKS
    if legs:
        import dataclasses
        c_cfg = dataclasses.replace(cfg, n_blocks=n_cb)
        c_inp = synth.make_stack_inputs(dataclasses.replace(c_cfg, n_clients=1, seed=cfg.seed + 7000), with_dy=False)
        cl = B.Client(c_cfg, c_inp["blocks"], c_inp["adapters"], max_seqs=cfg.batch)
        rng = np.random.Generator(np.random.PCG64(cfg.seed + 7001))
        cl_tok = torch.from_numpy(rng.integers(0, V, size=(cfg.batch, cfg.seq_len)).astype(np.int32)).cuda()
        cl_wpe = B.to_device_bf16(synth.round_bf16(rng.standard_normal((cfg.seq_len, cfg.d_model), dtype=np.float32)
                                                   * np.float32(0.02)))
        cl_act = torch.empty((cfg.batch, cfg.seq_len, cfg.d_model), dtype=torch.bfloat16, device="cuda")
        cl_dact = dy[:cfg.batch].contiguous()

        def client_round():
            cl.fwd(cl_tok, V, lh_Wv, cl_wpe, cl_act, stream)
            cl.bwd(cl_dact, stream)
            cl.step(lr, stream)

        for _ in range(2):
            client_round()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(10):
            client_round()
        torch.cuda.synchronize()
        cl_ms = (time.perf_counter() - t2) / 10 * 1e3
        del cl

    mx_leg = mxfp8_leg(cfg, stream) if legs else None
    if legs:
        # the metric's step once more with every frozen product in MXFP8 (a context of the compressed type);
        # reported beside the metric, never as the metric
        del srv
        torch.cuda.empty_cache()
        srv_mx = B.Server(cfg, inp["blocks"], inp["adapters"], dtype=B.DTYPE_MXFP8)

        def mx_step():
            srv_mx.fwd(xs, y, stream)
            srv_mx.bwd(dy, dxs, stream)
            srv_mx.step(lr, stream)

        for _ in range(2):
            mx_step()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for _ in range(5):
            mx_step()
        torch.cuda.synchronize()
        mx_ms = (time.perf_counter() - t3) / 5 * 1e3
        mx_leg["stack"] = {"ms_per_step": mx_ms, "tokens_per_s": cfg.tokens / (mx_ms * 1e-3),
                           "what": "forward + backward + adapter step of the same workload with the frozen "
                                   "products in MXFP8 (activation operands converted by the kernel that produces them or "
                                   "right before the product)"}
        del srv_mx
        srv = None

    fed5 = others = None
    if legs:
        fed5 = fedavg_hbm_rate(stream)
    if legs and not args.no_workloads and args.workload == 3:
        xs = y = dy = dxs = None
        torch.cuda.empty_cache()
        others = {}
        for w in (2, 4, 5):
            others[str(w)] = other_workload(w, lr)
            torch.cuda.empty_cache()

    if args.copy_calibration:
        n_cal = 64 * 1024 * 1024
        src = torch.ones(n_cal, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            B.slora_fedavg([src], [1], n_cal, dst, stream)
        torch.cuda.synchronize()

    ms = el / args.steps * 1e3
    tok_s = cfg.tokens / (el / args.steps)
    fg, fa, fl = model_flops_per_token(cfg)
    model_tflops = (fg + fa + fl) * cfg.tokens / (el / args.steps) / 1e12
    achieved = gemm_flop / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    out = {
        "metric": "server fwd+bwd tokens/sec on 1 MI355X + % bf16 MFMA peak (GPT-2-medium split)",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %d server blocks, d=%d, H=%d, d_ff=%d, LoRA r=%d on %s, K=%d clients x %d x %d "
                               "tokens (T=%d), bf16 activations; step = fwd + %sbwd + SGD adapter step + FedAvg of "
                               "the K client adapter sets" % (cfg.name, cfg.n_blocks, cfg.d_model, cfg.n_head,
                                                             cfg.d_ff, cfg.lora_r, ",".join(cfg.lora_proj),
                                                             cfg.n_clients, cfg.batch, cfg.seq_len, cfg.tokens,
                                                             "loss head (V=%d) + " % V if args.loss_head else ""),
                   "tokens_per_step": cfg.tokens},
        "model_tflops": model_tflops, "model_frac_of_bf16_peak": model_tflops / PEAK_BF16_TFLOPS,
        "roofline": {"bound": "mfma", "kernel": "gemm_kernel (bf16 MFMA GEMM + fused LoRA branch, all shapes)",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": recorded_gemm_traffic(),
                     "launches_timed": launches, "avg_launch_ms": gemm_ms / max(launches, 1),
                     # the clock the chip held under this load (the datasheet peak is at 2400 MHz), from the
                     # shader-clock and reference counters read by the 4-wave GEMM launches themselves
                     "shader_clock_mhz": clock_mhz, "clock_samples": clock_samples,
                     "frac_of_peak_at_observed_clock": (achieved / (PEAK_BF16_TFLOPS * clock_mhz / 2400.0)
                                                        if clock_mhz > 0 else None),
                     "gemm_share_of_step": gemm_ms / max(launches, 1) * (launches / args.steps) / ms},
    }
    if hbm_kernels is not None:
        if fed5 is not None:
            hbm_kernels["fedavg_kernel (workload 5)"] = fed5
        out["hbm_kernels"] = hbm_kernels
        out["attention_kernels"] = attn_kernels
    if others is not None:
        out["workloads"] = others
    if phases is not None:
        out["phases"] = phases
    if legs:
        out["client_side"] = {"ms": cl_ms, "client_blocks": n_cb, "tokens": cfg.batch * cfg.seq_len,
                              "tokens_per_s": cfg.batch * cfg.seq_len / (cl_ms * 1e-3),
                              "what": "one client: embedding + client blocks forward, backward, SGD step"}
        out["mxfp8_linear"] = mx_leg
        out["loss_head"] = {"ms": lh_ms, "vocab": V, "tflops": lh_flop / (lh_ms * 1e-3) / 1e12,
                            "in_timed_step": bool(args.loss_head)}
    if not args.no_cpu_baseline:
        srv = None
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(cfg, inp)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
