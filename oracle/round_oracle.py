"""Plain fp64 CPU oracle for whole training rounds of SplitLoRA (Algorithm 1) on one machine.

THIS IS TEST INFRASTRUCTURE (see slora_oracle.py): slow, plain, independent of the HIP path.

What it follows (SplitLoRA, arXiv 2407.00952, Sec. III-B and Algorithm 1), one round t:
  a1  every client i runs its client-side model forward on its mini-batch (Eq. 2): token + position
      embedding, then the client blocks with that client's adapters R_{c,i};
  a2  activations and labels go to the server;
  a3  the server runs its blocks on the concatenation S = [s_1; ...; s_N] (Eq. 3), computes the loss
      from the prediction and the labels, back-propagates, and updates its adapters (Eq. 4-5);
  a4  each client gets the gradient of its own slice of S;
  a5  each client back-propagates through its blocks and updates its adapters (Eq. 6-7);
  b1-b3, every I rounds: the client adapters are averaged with weights |D_i|/|D| (Eq. 8-9) and the
      average replaces every client's adapters.
Readings: the loss is the token cross-entropy of loss_head.py (one mean over all labeled tokens of all
clients in the round); embeddings are frozen; clients share the frozen weights and differ in adapters.
"""
from __future__ import annotations

import numpy as np

from .slora_oracle import ServerOracle, fedavg, _f64, PROJ_NAMES
from .loss_head import loss_head_fwd_bwd


def flatten_adapters(adapters):
    """Block by block, projections in PROJ_NAMES order, A then B, each row-major."""
    parts = []
    for ad in adapters:
        for p in PROJ_NAMES:
            if p in ad:
                parts += [np.asarray(ad[p][0]).ravel(), np.asarray(ad[p][1]).ravel()]
    return np.concatenate(parts)


def unflatten_adapters(vec, like):
    out, at = [], 0
    for ad in like:
        new = {}
        for p in PROJ_NAMES:
            if p in ad:
                A, B = ad[p]
                a = vec[at:at + A.size].reshape(A.shape); at += A.size
                b = vec[at:at + B.size].reshape(B.shape); at += B.size
                new[p] = (a.copy(), b.copy())
        out.append(new)
    assert at == vec.size
    return out


class RoundOracle:
    def __init__(self, wte, wpe, client_blocks, server_blocks, client_adapters, server_adapters, lnf_g, lnf_b,
                 n_head, lora_alpha, lora_r, eps=1e-5):
        """client_adapters: one adapter list (per client block) per client."""
        self.wte, self.wpe = _f64(wte), _f64(wpe)
        self.lnf_g, self.lnf_b, self.eps = _f64(lnf_g), _f64(lnf_b), float(eps)
        self.clients = [ServerOracle(client_blocks, ad, n_head, lora_alpha, lora_r, eps) for ad in client_adapters]
        self.server = ServerOracle(server_blocks, server_adapters, n_head, lora_alpha, lora_r, eps)

    def embed(self, tokens):
        tokens = np.asarray(tokens)
        S = tokens.shape[1]
        return self.wte[tokens] + self.wpe[np.arange(S)][None, :, :]

    def round(self, tokens, labels, lr_client, lr_server):
        """tokens, labels: per client integer arrays [b_i, S].  Returns the round's loss."""
        acts = [c.fwd([self.embed(t)]) for c, t in zip(self.clients, tokens)]           # a1
        Y = self.server.fwd(acts)                                                       # a3 forward
        lab = np.concatenate([np.asarray(l).reshape(-1) for l in labels])
        d = Y.shape[-1]
        loss, _, dY = loss_head_fwd_bwd(Y.reshape(-1, d), self.lnf_g, self.lnf_b, self.eps, self.wte, lab)
        dacts = self.server.bwd(dY.reshape(Y.shape))                                    # a3 backward, a4
        self.server_grads = self.server.grads
        self.server.step(lr_server)                                                     # Eq. 4-5
        self.client_grads = []
        for c, da in zip(self.clients, dacts):                                          # a5
            c.bwd(da)
            self.client_grads.append(c.grads)
            c.step(lr_client)                                                           # Eq. 6-7
        return loss

    def aggregate(self, sample_counts):
        """Eq. 8-9 on the flat adapter vectors; every client continues from the average."""
        flat = [flatten_adapters(c.adapters) for c in self.clients]
        avg = fedavg(flat, sample_counts)
        for c in self.clients:
            c.adapters = unflatten_adapters(avg, c.adapters)
        return avg
