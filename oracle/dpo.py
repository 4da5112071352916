"""Reference of the preference-learning step (DPO) on packed trajectories.

TEST INFRASTRUCTURE ONLY (see oracle/model.py).

The paper under study names the paradigm without formulas (Sections 1 and 3.2: the pipeline
trains with supervised fine-tuning and with preference learning such as DPO).  The loss is the
one of the public DPO description (Rafailov et al. 2023, the objective with a frozen reference
policy), written out:

  pi_s      = sum over the targets t of segment s of log p(token_{t+1} | tokens of s up to t)
              (the same targets as the supervised loss: next token in the same segment, mask 1)
  z_p       = beta * [(pi_c - ref_c) - (pi_r - ref_r)]        for a pair p = (chosen c, rejected r)
  loss      = mean over pairs of  -log sigmoid(z_p)  =  mean of log(1 + exp(-z_p))
  dloss/dpi_c = -beta * sigmoid(-z_p) / P,   dloss/dpi_r = +beta * sigmoid(-z_p) / P

``ref`` are the same sums under the frozen reference policy; they are an input here (with LoRA the
reference is the base model with the adapters switched off, with full fine-tuning a second set of
weights: either way one forward pass of oracle/model.py).  The reported statistics follow common
practice: margin = mean z_p, accuracy = fraction of pairs with z_p > 0.

Readings fixed here: a segment may appear in several pairs (its derivative is the sum) or in none
(derivative 0); a segment without targets has pi = 0.
"""
import numpy as np

from . import model as om


def sequence_logps(fwd, cu_seqlens):
    """pi_s for every segment, from a forward pass of oracle/model.py."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    per_token = fwd["per_token_loss"]                    # -log p at targets, 0 elsewhere
    return np.array([-per_token[cu[s]:cu[s + 1]].sum() for s in range(len(cu) - 1)])


def _log1pexp(x):
    """log(1 + exp(x)) without overflow."""
    return np.where(x > 0, x + np.log1p(np.exp(-np.abs(x))), np.log1p(np.exp(-np.abs(x))))


def dpo_loss(logp, ref_logp, pairs, beta):
    """Returns dict(loss, z [P], dlogp [S], margin, accuracy)."""
    logp, ref = np.asarray(logp, dtype=np.float64), np.asarray(ref_logp, dtype=np.float64)
    pairs = np.asarray(pairs, dtype=np.int64).reshape(-1, 2)
    P = len(pairs)
    dlogp = np.zeros_like(logp)
    if P == 0:
        return dict(loss=0.0, z=np.zeros(0), dlogp=dlogp, margin=0.0, accuracy=0.0)
    c, r = pairs[:, 0], pairs[:, 1]
    z = beta * ((logp[c] - ref[c]) - (logp[r] - ref[r]))
    loss = float(_log1pexp(-z).mean())
    with np.errstate(over="ignore"):
        sig_neg = 1.0 / (1.0 + np.exp(z))                # sigmoid(-z); exp overflow gives exactly 0
    np.add.at(dlogp, c, -beta * sig_neg / P)
    np.add.at(dlogp, r, +beta * sig_neg / P)
    return dict(loss=loss, z=z, dlogp=dlogp, margin=float(z.mean()), accuracy=float((z > 0).mean()))


def dpo_step(cfg, params, lora, tokens, cu_seqlens, loss_mask, pairs, ref_logp, beta):
    """Forward, loss and gradients.  Returns (dict(loss, logp, z, margin, accuracy), grads as oracle/model.backward)."""
    fwd = om.forward(cfg, params, lora, tokens, cu_seqlens, loss_mask)
    logp = sequence_logps(fwd, cu_seqlens)
    out = dpo_loss(logp, ref_logp, pairs, beta)
    # per_token_loss = -log p, so d loss / d per_token_loss[t] = -dlogp[segment of t]
    seg = om.segment_ids(np.asarray(cu_seqlens, dtype=np.int64), len(tokens))
    w = -out["dlogp"][seg[fwd["cache"]["tgt"]]]
    grads = om.backward(cfg, params, lora, fwd, target_weights=w)
    out["logp"] = logp
    return out, grads
