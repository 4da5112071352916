"""The pins must bite: plausible mistakes planted in the reference (on the
CPU, in a patched copy of its functions) have to be caught by at least one
cheap check below.  Each check is a reduced version of a pin in
test_oracle_model.py."""
import numpy as np
import pytest
import torch

from oracle import model as om
import oracle
import synth
from helpers import small_shape, random_trajs, packed, grad_norm_err
from test_oracle_model import _torch_model_loss, _to_torch


def _library_check():
    """Loss and LoRA/weight gradients against the torch library model."""
    sh = small_shape(n_layers=1, n_q_heads=4, n_kv_heads=2, head_dim=8, d_model=32, ffn=40, vocab=64,
                     lora_targets=synth.DENSE_TARGETS7, row_len=64)
    cfg = oracle.config_from_shape(sh)
    P = synth.weights(sh, 5, std=0.3, gain_jitter=0.1)
    Lo = synth.lora_weights(sh, 5, std=0.3)
    pk = packed(random_trajs(5, 3, sh.vocab), 64, 1)
    f, g = om.train_step(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    Pt, Lt = _to_torch(P, Lo)
    cu = pk["cu_seqlens"]
    total, count = 0.0, 0
    for s in range(len(cu) - 1):
        ls, c = _torch_model_loss(sh, Pt, Lt, pk["tokens"][cu[s]:cu[s + 1]], pk["loss_mask"][cu[s]:cu[s + 1]])
        total, count = total + ls, count + c
    (total / count).backward()
    ok = abs(float((total / count).detach()) - f["loss"]) < 1e-10 and count == f["count"]
    for k_, v in Pt["layers"][0].items():
        ok = ok and grad_norm_err(g["weights"]["layers"][0][k_], v.grad.numpy()) < 1e-9
    for k_, (A, B) in Lt[0].items():
        ok = ok and grad_norm_err(g["lora"][0][k_][0], A.grad.numpy()) < 1e-9
        ok = ok and grad_norm_err(g["lora"][0][k_][1], B.grad.numpy()) < 1e-9
    ok = ok and grad_norm_err(g["weights"]["embed"], Pt["embed"].grad.numpy()) < 1e-9
    ok = ok and grad_norm_err(g["weights"]["head"], Pt["head"].grad.numpy()) < 1e-9
    return bool(ok)


def test_unmutated_reference_passes():
    assert _library_check()


def _mut_rope_sign(x, cos, sin, inverse=False):
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    if inverse:
        s = -s
    return np.concatenate([x1 * c + x2 * s, -x1 * s + x2 * c], axis=-1)     # rotates the other way


def _mut_rope_interleaved(x, cos, sin, inverse=False):
    c, s = np.repeat(cos, 2, axis=1)[:, None, :], np.repeat(sin, 2, axis=1)[:, None, :]
    if inverse:
        s = -s
    xr = np.empty_like(x)
    xr[..., 0::2], xr[..., 1::2] = -x[..., 1::2], x[..., 0::2]              # pairs (2i, 2i+1) instead
    return x * c + xr * s


def _mut_rms_bwd_drop_term(dy, x, g, rho):
    return rho[:, None] * dy * g[None, :], np.sum(dy * x * rho[:, None], axis=0)


def _mut_linear_bwd_no_scale(dy, x, W, ab, scale, u):
    dx, dW = dy @ W, dy.T @ x
    if ab is None:
        return dx, dW, None
    A, B = ab
    du = dy @ B                                                              # forgot alpha/r
    return dx + du @ A, dW, (du.T @ x, scale * (dy.T @ u))


def _mut_linear_transposed(x, W, ab, scale):
    y = x @ W.T
    if ab is None:
        return y, None
    A, B = ab
    u = x @ A.T
    return y + (u @ B.T), u                                                  # forward drops the scale


def _mut_targets_unshifted(tokens, cu_seqlens, loss_mask):
    N = len(tokens)
    seg = om.segment_ids(cu_seqlens, N)
    idx = np.asarray([t for t in range(N - 1) if seg[t + 1] == seg[t] and loss_mask[t] == 1], dtype=np.int64)
    return idx, np.asarray(tokens, dtype=np.int64)[idx + 1]                  # mask read at t, not t+1


def _mut_rmsnorm_eps_outside(x, g, eps):
    rho = 1.0 / (np.sqrt(np.mean(x * x, axis=-1)) + eps * 1e3)
    return x * rho[:, None] * g[None, :], rho


MUTANTS = {
    "rope rotates the wrong way in forward only": ("rope", _mut_rope_sign),
    "rope pairs neighbours": ("rope", _mut_rope_interleaved),
    "rmsnorm backward drops the projection term": ("rmsnorm_bwd", _mut_rms_bwd_drop_term),
    "lora backward forgets the scale on du": ("linear_bwd", _mut_linear_bwd_no_scale),
    "lora forward forgets the scale": ("linear", _mut_linear_transposed),
    "loss mask read unshifted": ("targets", _mut_targets_unshifted),
    "eps outside the square root": ("rmsnorm", _mut_rmsnorm_eps_outside),
}


@pytest.mark.parametrize("name", list(MUTANTS))
def test_planted_mistake_is_caught(name, monkeypatch):
    attr, fn = MUTANTS[name]
    monkeypatch.setattr(om, attr, fn)
    if attr == "rope" and fn is _mut_rope_sign:
        # a consistently mirrored rotation is the same function of position
        # differences; only the pairing/sign pin on explicit angles can see it
        x = np.arange(16, dtype=np.float64).reshape(2, 1, 8)
        c, s = om.rope_table(np.arange(2), 8, 100.0)
        r = om.rope(x, c, s)
        th = 100.0 ** (-2.0 * 1 / 8)
        assert abs(r[1, 0, 1] - (x[1, 0, 1] * np.cos(th) - x[1, 0, 5] * np.sin(th))) > 1e-3
        return
    assert not _library_check()
