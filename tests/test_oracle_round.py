"""Pins of the whole-round oracle (Algorithm 1): the split pipeline against a monolithic model built
from torch library ops with autograd, and the aggregation schedule."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle.round_oracle import RoundOracle, flatten_adapters, unflatten_adapters
from paper_2407_00952_amd import synth
from test_oracle_stack import _torch_stack

torch.set_default_dtype(torch.float64)


def make_round(seed=0, n_clients=3, batches=(2, 1, 3), n_cb=2, n_sb=2, proj=("q", "v"), V=37, S=9):
    cfg = synth.tiny_config(d_model=16, n_head=2, d_ff=24, n_blocks=n_cb + n_sb, lora_r=2, lora_proj=proj,
                            n_clients=n_clients, batch=1, seq_len=S)
    rng = np.random.Generator(np.random.PCG64(seed))
    f = lambda a: np.asarray(a, dtype=np.float64)
    blocks = [{k: f(v) for k, v in synth.make_block(rng, cfg, False).items()} for _ in range(n_cb + n_sb)]

    def adapters(n):
        out = []
        for _ in range(n):
            ad = {}
            for p in synth.PROJ_NAMES:
                if p in proj:
                    n_in, n_out = cfg.proj_shape(p)
                    A, B = synth.make_adapter(rng, cfg.lora_r, n_in, n_out, False)
                    ad[p] = (f(A), f(B) * 30.0)         # B large enough for the adapters to matter
            out.append(ad)
        return out
    cads = [adapters(n_cb) for _ in range(n_clients)]
    sads = adapters(n_sb)
    wte = f(rng.standard_normal((V, cfg.d_model))) * 0.5
    wpe = f(rng.standard_normal((S, cfg.d_model))) * 0.1
    lnf_g = 1.0 + 0.1 * f(rng.standard_normal(cfg.d_model))
    lnf_b = 0.1 * f(rng.standard_normal(cfg.d_model))
    tokens = [rng.integers(0, V, size=(b, S)) for b in batches]
    labels = [rng.integers(0, V, size=(b, S)) for b in batches]
    for l in labels:
        l[:, :3] = -1
    orc = RoundOracle(wte, wpe, blocks[:n_cb], blocks[n_cb:], cads, sads, lnf_g, lnf_b, cfg.n_head, cfg.lora_alpha,
                      cfg.lora_r, cfg.ln_eps)
    return cfg, orc, blocks, cads, sads, wte, wpe, lnf_g, lnf_b, tokens, labels


def torch_monolithic_loss(cfg, blocks, n_cb, cads, sads, wte, wpe, lnf_g, lnf_b, tokens, labels):
    """Every client's sequences through [its client blocks] + [the shared server blocks] + head; one mean
    cross-entropy over all labeled tokens.  Returns (loss, per-client adapter leaves, server adapter leaves)."""
    S = tokens[0].shape[1]
    t_wte, t_wpe = torch.tensor(wte), torch.tensor(wpe)
    s = cfg.lora_alpha / cfg.lora_r
    # server adapter leaves are shared by all clients' sequences
    srv_leaves = None
    hs, cl_leaves = [], []
    for i, tok in enumerate(tokens):
        h0 = t_wte[torch.tensor(tok)] + t_wpe[:S][None]
        _, h, leaves = _torch_stack(cfg, blocks[:n_cb], cads[i], h0.numpy())
        cl_leaves.append(leaves)
        hs.append(h)
    hcat = torch.cat(hs, dim=0)
    # server part with ONE set of leaves: rebuild the stack by hand on the concatenation
    srv_leaves = [{p: (torch.tensor(A, requires_grad=True), torch.tensor(B, requires_grad=True))
                   for p, (A, B) in ad.items()} for ad in sads]
    d, H = cfg.d_model, cfg.n_head
    h = hcat
    for blk, ad in zip(blocks[n_cb:], srv_leaves):
        tb = {k: torch.tensor(v) for k, v in blk.items()}

        def lin(x, name, W, b):
            y = F.linear(x, W, b)
            if name in ad:
                y = y + s * F.linear(F.linear(x, ad[name][0]), ad[name][1])
            return y
        u = F.layer_norm(h, (d,), tb["ln1_g"], tb["ln1_b"], cfg.ln_eps)
        q = lin(u, "q", tb["Wqkv"][:d], tb["bqkv"][:d])
        k = lin(u, "k", tb["Wqkv"][d:2 * d], tb["bqkv"][d:2 * d])
        v = lin(u, "v", tb["Wqkv"][2 * d:], tb["bqkv"][2 * d:])
        N = h.shape[0]
        sp = lambda a: a.reshape(N, S, H, d // H).transpose(1, 2)
        o = F.scaled_dot_product_attention(sp(q), sp(k), sp(v), is_causal=True).transpose(1, 2).reshape(N, S, d)
        h = h + lin(o, "o", tb["Wo"], tb["bo"])
        u2 = F.layer_norm(h, (d,), tb["ln2_g"], tb["ln2_b"], cfg.ln_eps)
        h = h + lin(F.gelu(lin(u2, "fc", tb["Wfc"], tb["bfc"]), approximate="tanh"), "pr", tb["Wpr"], tb["bpr"])
    u = F.layer_norm(h, (d,), torch.tensor(lnf_g), torch.tensor(lnf_b), cfg.ln_eps)
    logits = F.linear(u, t_wte)
    lab = torch.tensor(np.concatenate([l.reshape(-1) for l in labels]))
    loss = F.cross_entropy(logits.reshape(-1, logits.shape[-1]), lab, ignore_index=-1, reduction="mean")
    return loss, cl_leaves, srv_leaves


@pytest.mark.parametrize("proj", [("q", "v"), synth.PROJ_NAMES])
def test_round_gradients_match_monolithic_torch_autograd(proj):
    cfg, orc, blocks, cads, sads, wte, wpe, lnf_g, lnf_b, tokens, labels = make_round(1, proj=proj)
    loss = orc.round(tokens, labels, lr_client=0.0, lr_server=0.0)
    tl, cl, sl = torch_monolithic_loss(cfg, blocks, 2, cads, sads, wte, wpe, lnf_g, lnf_b, tokens, labels)
    # the client-side leaves were built from numpy h0 inside _torch_stack (detached from the embedding,
    # which is frozen anyway); gradients flow from the loss through the server part into them
    tl.backward()
    assert abs(loss - tl.item()) < 1e-12
    for l, ad in enumerate(sl):
        for p, (A, B) in ad.items():
            assert np.allclose(orc.server_grads[l][p][0], A.grad.numpy(), atol=1e-11, rtol=1e-9)
            assert np.allclose(orc.server_grads[l][p][1], B.grad.numpy(), atol=1e-11, rtol=1e-9)
    big = 0.0
    for i, leaves in enumerate(cl):
        for l, ad in enumerate(leaves):
            for p, (A, B) in ad.items():
                assert np.allclose(orc.client_grads[i][l][p][0], A.grad.numpy(), atol=1e-11, rtol=1e-9)
                assert np.allclose(orc.client_grads[i][l][p][1], B.grad.numpy(), atol=1e-11, rtol=1e-9)
                big = max(big, np.abs(A.grad.numpy()).max())
    assert big > 1e-6         # client gradients are not trivially zero


def test_sgd_uses_the_two_rates_and_aggregation_averages_clients():
    cfg, orc, blocks, cads, sads, wte, wpe, lnf_g, lnf_b, tokens, labels = make_round(2)
    before_c = [flatten_adapters(c.adapters) for c in orc.clients]
    before_s = flatten_adapters(orc.server.adapters)
    orc.round(tokens, labels, lr_client=0.5, lr_server=0.25)
    gs = flatten_adapters([{p: g for p, g in gl.items()} for gl in orc.server_grads])
    assert np.allclose(flatten_adapters(orc.server.adapters), before_s - 0.25 * gs, atol=1e-15)
    for i, c in enumerate(orc.clients):
        gc = flatten_adapters([{p: g for p, g in gl.items()} for gl in orc.client_grads[i]])
        assert np.allclose(flatten_adapters(c.adapters), before_c[i] - 0.5 * gc, atol=1e-15)
    flat = [flatten_adapters(c.adapters) for c in orc.clients]
    counts = [10, 30, 60]
    avg = orc.aggregate(counts)
    assert np.allclose(avg, 0.1 * flat[0] + 0.3 * flat[1] + 0.6 * flat[2], atol=1e-15)
    for c in orc.clients:
        assert np.array_equal(flatten_adapters(c.adapters), avg)
    # server adapters are not part of the aggregation
    assert np.allclose(flatten_adapters(orc.server.adapters), before_s - 0.25 * gs, atol=1e-15)


def test_flatten_roundtrip_and_order():
    cfg, orc, *_ = make_round(3, proj=("q", "o", "pr"))
    ads = orc.clients[0].adapters
    v = flatten_adapters(ads)
    back = unflatten_adapters(v, ads)
    for a, b in zip(ads, back):
        for p in a:
            assert np.array_equal(a[p][0], b[p][0]) and np.array_equal(a[p][1], b[p][1])
    A0 = ads[0]["q"][0]
    assert np.array_equal(v[:A0.size], A0.ravel())


def test_identical_clients_stay_identical_and_loss_decreases():
    # same adapters, same data on every client: aggregation is a no-op and plain SGD lowers the loss
    cfg, orc, blocks, cads, sads, wte, wpe, lnf_g, lnf_b, tokens, labels = make_round(4, batches=(2, 2, 2))
    same = RoundOracle(wte, wpe, blocks[:2], blocks[2:], [cads[0]] * 3, sads, lnf_g, lnf_b, cfg.n_head,
                       cfg.lora_alpha, cfg.lora_r, cfg.ln_eps)
    tok, lab = [tokens[0]] * 3, [labels[0]] * 3
    l0 = same.round(tok, lab, 0.05, 0.05)
    f0 = [flatten_adapters(c.adapters) for c in same.clients]
    assert np.array_equal(f0[0], f0[1]) and np.array_equal(f0[0], f0[2])
    avg = same.aggregate([5, 5, 5])
    assert np.allclose(avg, f0[0], atol=1e-16)
    l1 = same.round(tok, lab, 0.05, 0.05)
    assert l1 < l0
