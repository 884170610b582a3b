"""Plain fp64 CPU oracle for the server's loss head.

THIS IS TEST INFRASTRUCTURE (see slora_oracle.py): slow, plain, independent of the
HIP path, never imported by the product package.

What it follows (SplitLoRA, arXiv 2407.00952, Sec. III-B): in step a2 the clients
send their labels along with the activations; in step a3 the server turns its
predicted value and the labels into the loss and derives the gradients from it.
The paper does not spell the head out.  Readings taken here:
  * the head is GPT-2's (the paper's model, Sec. IV-A): a final LayerNorm followed
    by logits against the token-embedding matrix Wv [V, d] (tied, frozen like every
    pre-trained weight, Sec. III-A), no bias;
  * the loss is the token-level cross-entropy of the softmax over the vocabulary,
    averaged over the tokens that carry a label (label < 0 = "no label": context
    tokens of a prompt do not count), which is the usual language-model fine-tuning
    objective and matches Eq. (1)'s per-sample loss up to how samples are weighted;
  * nothing in the head is trainable, so the only gradient is the one w.r.t. the
    server stack's output, which is what the stack's backward pass takes as dY.

Everything is float64; one token row at a time would do, numpy does all rows at once.

Pinned by tests/test_oracle_loss_head.py (finite differences of an independent
loop-only loss, zero-logit closed form log V, shift invariance of the softmax,
row sums of the gradient, unlabeled tokens, one-token closed form).
"""
from __future__ import annotations

import numpy as np

from .slora_oracle import layernorm_fwd, layernorm_bwd, _f64


def loss_head_fwd_bwd(y, gamma, beta, eps, Wv, labels):
    """y [T,d] server output, gamma/beta [d] final LayerNorm, Wv [V,d], labels [T] int (<0: none).

    Returns (loss, loss_tok [T], dy [T,d]):
      loss_tok[t] = logsumexp_v(logits[t,:]) - logits[t, labels[t]]   (0 where unlabeled)
      loss        = sum_t loss_tok[t] / n_labeled
      dy          = d loss / d y
    """
    y, Wv = _f64(y), _f64(Wv)
    labels = np.asarray(labels, dtype=np.int64)
    T = y.shape[0]
    valid = labels >= 0
    n = int(valid.sum())
    if n == 0:
        raise ValueError("no labeled token")
    u, saved = layernorm_fwd(y, gamma, beta, eps)
    logits = u @ Wv.T                                        # [T,V]
    m = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - m)
    se = e.sum(axis=1, keepdims=True)
    lse = (m + np.log(se))[:, 0]
    rows = np.arange(T)
    picked = logits[rows, np.where(valid, labels, 0)]
    loss_tok = np.where(valid, lse - picked, 0.0)
    loss = loss_tok.sum() / n
    # d loss / d logits = (softmax - onehot) / n on labeled rows, 0 elsewhere
    dlogits = e / se
    dlogits[rows[valid], labels[valid]] -= 1.0
    dlogits *= (valid[:, None] / n)
    du = dlogits @ Wv                                        # [T,d]
    dy = layernorm_bwd(du, gamma, saved)
    return loss, loss_tok, dy
