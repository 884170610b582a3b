"""Driver of whole SplitLoRA training rounds (Algorithm 1) on one GPU: call sequencing only.

Every arithmetic step is a call into libslora (client forward, server forward, loss head, server
backward, SGD steps, client backward, FedAvg); this module owns device buffers through PyTorch and
decides the order, nothing else.  On a real deployment the clients are different machines; here their
contexts sit on the same device and run one after the other, which is what the parity test needs.
"""
from __future__ import annotations

import dataclasses

import numpy as np

from . import binding as B


class SplitRound:
    def __init__(self, cfg, n_client_blocks, blocks, client_adapters, server_adapters, wte, wpe, lnf_g, lnf_b,
                 batches):
        """cfg: synth.StackConfig of the whole model (n_blocks = client + server blocks).
        blocks: all frozen blocks; client_adapters: one adapter list per client; batches: b_i per client."""
        import torch
        self.cfg = cfg
        self.vocab = int(wte.shape[0])
        self.batches = [int(b) for b in batches]
        c_cfg = dataclasses.replace(cfg, n_blocks=n_client_blocks)
        s_cfg = dataclasses.replace(cfg, n_blocks=cfg.n_blocks - n_client_blocks)
        self.clients = [B.Client(c_cfg, blocks[:n_client_blocks], ad, max_seqs=b)
                        for ad, b in zip(client_adapters, self.batches)]
        n_seq = sum(self.batches)
        self.server = B.Server(s_cfg, blocks[n_client_blocks:], server_adapters, max_seqs=n_seq)
        self.wte, self.wpe = B.to_device_bf16(wte), B.to_device_bf16(wpe)
        self.lnf_g, self.lnf_b = B.to_device_bf16(lnf_g), B.to_device_bf16(lnf_b)
        S, d = cfg.seq_len, cfg.d_model
        self.T = n_seq * S
        bf = torch.bfloat16
        self.acts = [torch.empty((b, S, d), dtype=bf, device="cuda") for b in self.batches]
        self.dacts = [torch.empty((b, S, d), dtype=bf, device="cuda") for b in self.batches]
        self.y = torch.empty((n_seq, S, d), dtype=bf, device="cuda")
        self.dy = torch.empty((n_seq, S, d), dtype=bf, device="cuda")
        self.loss_tok = torch.empty(self.T, dtype=torch.float32, device="cuda")
        self.loss = torch.empty(1, dtype=torch.float32, device="cuda")
        self.lh_bytes = B.slora_loss_head_ws_bytes(self.T, d, self.vocab)
        if self.lh_bytes == 0:
            raise ValueError("loss head does not support these sizes")
        self.lh_ws = torch.empty(self.lh_bytes, dtype=torch.uint8, device="cuda")
        B.slora_loss_head_prepare(d, self.vocab, self.wte, self.lh_ws, self.lh_bytes)
        self.avg = torch.empty_like(self.clients[0].flat)

    def round(self, tokens, labels, lr_client, lr_server, stream=None):
        """tokens: per client device int32 [b_i, S]; labels: device int32 [sum b_i * S] in client order.
        Leaves the round's loss in self.loss (device) and returns that tensor."""
        cfg = self.cfg
        for c, t, a in zip(self.clients, tokens, self.acts):                       # a1
            c.fwd(t, self.vocab, self.wte, self.wpe, a, stream)
        self.server.fwd(self.acts, self.y, stream)                                 # a2, a3
        B.slora_loss_head(self.T, cfg.d_model, self.vocab, self.y, self.lnf_g, self.lnf_b, cfg.ln_eps, labels,
                          self.lh_ws, self.lh_bytes, self.loss_tok, self.loss, self.dy, stream)
        self.server.bwd(self.dy, self.dacts, stream)                               # a3, a4
        self.server.step(lr_server, stream)                                        # Eq. (4)-(5)
        for c, da in zip(self.clients, self.dacts):                                # a5
            c.bwd(da, stream)
            c.step(lr_client, stream)                                              # Eq. (6)-(7)
        return self.loss

    def aggregate(self, sample_counts, stream=None):
        """b1-b3: average the clients' flat adapter vectors (Eq. 8-9) and hand the result back to all."""
        import torch
        if stream is not None and stream != torch.cuda.current_stream().cuda_stream:
            raise ValueError("aggregate: the download copies run on torch's current stream; pass that one")
        n = self.clients[0].n_params
        B.slora_fedavg([c.flat for c in self.clients], np.asarray(sample_counts, dtype=np.int64), n, self.avg,
                       stream)
        for c in self.clients:
            c.flat.copy_(self.avg)                 # the download (plain copy)
            c.adapters_changed()
