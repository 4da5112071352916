"""Pins for the float64 reference of the preference (DPO) step: closed forms of the pair loss, the
exchange identity, central differences through the whole model, and the reduction to the (separately
pinned) supervised gradient when the pair's other side carries no target."""
import math

import numpy as np
import pytest

import oracle
from oracle import model as om
from oracle import dpo
import synth
from helpers import small_shape, random_trajs, packed, grad_norm_err


def setup(seed=3, n_traj=4, **kw):
    sh = small_shape(lora_targets=synth.DENSE_TARGETS7, **kw)
    cfg = oracle.config_from_shape(sh)
    P = synth.weights(sh, seed, std=0.3, gain_jitter=0.1)
    Lo = synth.lora_weights(sh, seed, std=0.3)
    pk = packed(random_trajs(seed, n_traj, sh.vocab), sh.row_len, 1)
    assert pk["n_traj_consumed"] == n_traj
    return cfg, P, Lo, pk


def ref_logps(cfg, P, pk):
    """Reference policy = the base model with the adapters off."""
    f = om.forward(cfg, P, None, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    return dpo.sequence_logps(f, pk["cu_seqlens"])


def test_pair_loss_closed_forms():
    # z = ln 3 (beta 1, chosen ahead of its reference by ln 3): -log sigmoid = ln(4/3), sigmoid(-z) = 1/4
    out = dpo.dpo_loss([math.log(3.0) - 5.0, -7.0], [-5.0, -7.0], [(0, 1)], 1.0)
    assert out["loss"] == pytest.approx(math.log(4.0 / 3.0), abs=1e-15)
    assert out["dlogp"] == pytest.approx([-0.25, 0.25], abs=1e-15)
    assert out["accuracy"] == 1.0 and out["margin"] == pytest.approx(math.log(3.0))
    # policy = reference: every z is 0, loss ln 2, slope beta / 2 spread over the pairs; z > 0 nowhere
    lp = np.array([-3.0, -9.5, -1.25, -4.0])
    out = dpo.dpo_loss(lp, lp, [(0, 1), (2, 3)], 0.3)
    assert out["loss"] == pytest.approx(math.log(2.0), abs=1e-15)
    assert out["dlogp"] == pytest.approx([-0.075, 0.075, -0.075, 0.075], abs=1e-15)
    assert out["accuracy"] == 0.0
    # beta = 0 switches the preference signal off
    out = dpo.dpo_loss(lp, lp + 1.0, [(0, 1)], 0.0)
    assert out["loss"] == pytest.approx(math.log(2.0)) and np.all(out["dlogp"] == 0)
    # far on the right side the loss vanishes, far on the wrong side it is -z (no overflow either way)
    out = dpo.dpo_loss([0.0, -2000.0], [0.0, 0.0], [(0, 1)], 1.0)
    assert out["loss"] == pytest.approx(0.0, abs=1e-300) and abs(out["dlogp"]).max() < 1e-300
    out = dpo.dpo_loss([-2000.0, 0.0], [0.0, 0.0], [(0, 1)], 1.0)
    assert out["loss"] == pytest.approx(2000.0) and out["dlogp"] == pytest.approx([-1.0, 1.0])
    # a segment in two pairs sums its slopes, a segment in none gets zero; no pair at all: zero loss
    out = dpo.dpo_loss(lp, lp, [(0, 1), (0, 3)], 1.0)
    assert out["dlogp"] == pytest.approx([-0.5, 0.25, 0.0, 0.25])
    assert dpo.dpo_loss(lp, lp, np.zeros((0, 2)), 1.0)["loss"] == 0.0


def test_exchange_identity():
    """-log sigmoid(-z) - (-log sigmoid(z)) = z: swapping chosen and rejected in every pair raises the loss by mean z."""
    rs = np.random.default_rng(0)
    lp, ref = rs.normal(-20, 5, 8), rs.normal(-20, 5, 8)
    pairs = [(0, 1), (2, 3), (4, 5), (6, 7), (1, 6)]
    a = dpo.dpo_loss(lp, ref, pairs, 0.7)
    b = dpo.dpo_loss(lp, ref, [(r, c) for c, r in pairs], 0.7)
    assert b["loss"] - a["loss"] == pytest.approx(a["margin"], abs=1e-12)
    assert b["z"] == pytest.approx(-a["z"])


def test_sequence_logps_are_log_probabilities_of_the_continuations():
    """exp(pi_s) summed over every possible value of one masked token is 1 when that token is the segment's only target."""
    cfg, P, Lo, pk = setup(n_traj=2)
    cu = pk["cu_seqlens"]
    mask = np.zeros_like(pk["loss_mask"]); t = int(cu[0]) + 3; mask[t] = 1
    tot = 0.0
    for tok in range(cfg.vocab):
        toks = pk["tokens"].copy(); toks[t] = tok
        toks[t + 1:cu[1]] = 0                                  # later tokens do not matter for this target
        f = om.forward(cfg, P, Lo, toks, cu, mask)
        lp = dpo.sequence_logps(f, cu)
        assert np.all(lp[1:] == 0)                             # segments without a target
        tot += math.exp(lp[0])
    assert tot == pytest.approx(1.0, abs=1e-12)


def test_gradients_match_central_differences():
    cfg, P, Lo, pk = setup()
    ref = ref_logps(cfg, P, pk)
    S = len(pk["cu_seqlens"]) - 1
    assert S >= 4
    pairs, beta = [(0, 1), (2, 3), (0, 3)], 0.4
    out, g = dpo.dpo_step(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"], pairs, ref, beta)
    assert 0 < out["accuracy"] < 1 or abs(out["margin"]) > 1e-3   # adapters are on: policy differs from the reference

    def loss():
        f = om.forward(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
        return dpo.dpo_loss(dpo.sequence_logps(f, pk["cu_seqlens"]), ref, pairs, beta)["loss"]

    rs = np.random.default_rng(1)
    worst = 0.0
    for l in range(cfg.n_layers):
        for name, (A, B) in Lo[l].items():
            for which, M in ((0, A), (1, B)):
                G = g["lora"][l][name][which]
                for _ in range(3):
                    idx = tuple(rs.integers(0, d) for d in M.shape)
                    w0 = M[idx]; h = 1e-5 * max(1.0, abs(w0))
                    M[idx] = w0 + h; lp = loss()
                    M[idx] = w0 - h; lm = loss()
                    M[idx] = w0
                    worst = max(worst, abs((lp - lm) / (2 * h) - G[idx]) / max(1e-3, abs(G).max()))
    assert worst < 1e-6
    # a frozen weight too (what full fine-tuning would use)
    W = P["layers"][0]["wq"]; G = g["weights"]["layers"][0]["wq"]
    idx = (1, 2); w0 = W[idx]; h = 1e-5
    W[idx] = w0 + h; lp = loss(); W[idx] = w0 - h; lm = loss(); W[idx] = w0
    assert abs((lp - lm) / (2 * h) - G[idx]) < 1e-6 * max(1e-3, abs(G).max())


def test_reduces_to_supervised_gradient_when_the_other_side_has_no_target():
    """One pair whose rejected segment carries no target: pi_r = 0 whatever the weights, so the gradient is
    beta * sigmoid(-z) * (target count) times the supervised mean-loss gradient of the chosen segment alone."""
    cfg, P, Lo, pk = setup()
    cu = pk["cu_seqlens"]
    mask = pk["loss_mask"].copy(); mask[cu[1]:] = 0                  # only segment 0 keeps targets
    ref = ref_logps(cfg, P, dict(pk, loss_mask=mask))
    assert np.all(ref[1:] == 0) and ref[0] < 0
    beta = 0.25
    out, g = dpo.dpo_step(cfg, P, Lo, pk["tokens"], cu, mask, [(0, 1)], ref, beta)
    f, gs = om.train_step(cfg, P, Lo, pk["tokens"], cu, mask)
    k = beta / (1.0 + math.exp(out["z"][0])) * f["count"]
    for l in range(cfg.n_layers):
        for name in Lo[l]:
            for i in (0, 1):
                assert grad_norm_err(g["lora"][l][name][i], k * gs["lora"][l][name][i]) < 1e-12
    assert out["logp"][0] == pytest.approx(-f["loss_sum"], rel=1e-14)


def _library_check():
    """Loss and gradients against the PyTorch float64 model built from library routines
    (scaled_dot_product_attention, cross_entropy, logsigmoid, autograd), one segment at a time."""
    import torch
    import torch.nn.functional as F
    from test_oracle_model import _torch_model_loss, _to_torch
    sh = small_shape(n_layers=1, n_q_heads=4, n_kv_heads=2, head_dim=8, d_model=32, ffn=40, vocab=64,
                     lora_targets=synth.DENSE_TARGETS7, row_len=96)
    cfg = oracle.config_from_shape(sh)
    P = synth.weights(sh, 6, std=0.3, gain_jitter=0.1)
    Lo = synth.lora_weights(sh, 6, std=0.3)
    pk = packed(random_trajs(6, 4, sh.vocab), 96, 1)
    cu = pk["cu_seqlens"]
    assert len(cu) - 1 >= 4
    ref = ref_logps(cfg, P, pk)
    pairs, beta = [(0, 1), (3, 2)], 0.5
    out, g = dpo.dpo_step(cfg, P, Lo, pk["tokens"], cu, pk["loss_mask"], pairs, ref, beta)
    Pt, Lt = _to_torch(P, Lo)
    pi = []
    for s in range(len(cu) - 1):
        ls, _ = _torch_model_loss(sh, Pt, Lt, pk["tokens"][cu[s]:cu[s + 1]], pk["loss_mask"][cu[s]:cu[s + 1]])
        pi.append(-ls if torch.is_tensor(ls) else torch.tensor(0.0, dtype=torch.float64))
    rt = torch.from_numpy(ref)
    loss = sum(-F.logsigmoid(beta * ((pi[c] - rt[c]) - (pi[r] - rt[r]))) for c, r in pairs) / len(pairs)
    loss.backward()
    ok = abs(float(loss.detach()) - out["loss"]) < 1e-11
    for k_, (A, B) in Lt[0].items():
        ok = ok and grad_norm_err(g["lora"][0][k_][0], A.grad.numpy()) < 1e-9
        ok = ok and grad_norm_err(g["lora"][0][k_][1], B.grad.numpy()) < 1e-9
    for k_, v in Pt["layers"][0].items():
        ok = ok and grad_norm_err(g["weights"]["layers"][0][k_], v.grad.numpy()) < 1e-9
    return bool(ok and grad_norm_err(g["weights"]["head"], Pt["head"].grad.numpy()) < 1e-9)


def test_against_library_model_and_autograd():
    assert _library_check()


@pytest.mark.parametrize("mistake", ["no_pair_mean", "sign", "no_beta", "sigmoid_of_plus_z", "ref_ignored"])
def test_planted_mistakes_are_caught(monkeypatch, mistake):
    """Plausible mistakes planted in the reference's pair loss (on the CPU) must fail the library check."""
    good = dpo.dpo_loss

    def bad(logp, ref_logp, pairs, beta):
        out = dict(good(logp, ref_logp, pairs, beta))
        P = max(len(pairs), 1)
        if mistake == "no_pair_mean":
            out["dlogp"] = out["dlogp"] * P
        elif mistake == "sign":
            out["dlogp"] = -out["dlogp"]
        elif mistake == "no_beta":
            out["dlogp"] = out["dlogp"] / beta
        elif mistake == "sigmoid_of_plus_z":
            alt = good(logp, ref_logp, [(r, c) for c, r in pairs], beta)      # slope sigmoid(z) instead of sigmoid(-z)
            out["dlogp"] = -alt["dlogp"]
        else:
            out = dict(good(logp, np.zeros_like(np.asarray(ref_logp)), pairs, beta))
        return out

    monkeypatch.setattr(dpo, "dpo_loss", bad)
    assert not _library_check()
