"""Whole-step parity of sparse (top-2 of 8 experts) layers against the float64 reference.

Top-2 routing is discontinuous where the second and third largest router logits tie, so each case
first checks, on the reference side only, that every token's decision margin is far above the
rounding error of the tier under test; the comparison is meaningless otherwise."""
import numpy as np
import pytest

import oracle
import synth
from helpers import random_trajs

pytestmark = pytest.mark.gpu

MOE = dict(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=32, d_model=64, ffn=96, vocab=128,
           lora_targets=("q", "k", "v", "o", "router"), lora_rank=4, lora_alpha=8.0, n_experts=8, top_k=2)


def router_margin(sh, params, lora, trajs, rows, row_len):
    """min over layers and tokens of (second largest - third largest router logit), float64."""
    pk = oracle.pack(trajs, row_len, rows)
    f = oracle.forward(oracle.config_from_shape(sh), params, lora, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    m = np.inf
    for c in f["cache"]["layers"]:
        lg = np.sort(c["ffn"]["logit"], axis=1)
        m = min(m, float((lg[:, -2] - lg[:, -3]).min()))
    return m


def structured_router_params(sh, seed, live=None, dtype=np.float64):
    """Weights whose routing is decided by the token id with a wide margin: orthonormal router rows,
    and embeddings that are a 1.0 / 0.8 mix of two router rows (per layer the rows are permuted)
    plus the usual small noise.  The rest of the model is the ordinary random draw."""
    g = synth.rng(seed, 11)
    P = synth.weights(sh, seed, dtype=dtype)
    d, E, V = sh.d_model, sh.n_experts, sh.vocab
    basis, _ = np.linalg.qr(g.standard_normal((d, E)))          # [d, E], orthonormal columns
    live = E if live is None else live                          # experts beyond `live` are never chosen
    e1 = g.integers(0, live, size=V)
    e2 = (e1 + g.integers(1, live, size=V)) % live
    P["embed"] = basis[:, e1].T + 0.8 * basis[:, e2].T + 0.02 * g.standard_normal((V, d))
    for W in P["layers"]:
        perm = np.concatenate([g.permutation(live), np.arange(live, E)])
        W["wrouter"] = 0.16 * basis[:, perm].T
    return P


def _compare(sh, params, lora, trajs, rows, row_len, bf16, recompute):
    import gpu_util as G
    from helpers import grad_norm_err, rel_err
    from paper_2503_22673_amd import binding as B
    params = G.quantise_params(params, bf16)
    lora = G.quantise_lora(lora)
    margin = router_margin(sh, params, lora, trajs, rows, row_len)
    assert margin > (0.1 if bf16 else 1e-4), "routing margin %.3g too small for this tier" % margin
    res, model, pk, ctx = G.run_step(sh, params, lora, trajs, rows, row_len, mode=B.AS_BF16 if bf16 else B.AS_FP32,
                                     recompute=recompute)
    ref_pk = oracle.pack(trajs, row_len, rows)
    f, g = oracle.train_step(oracle.config_from_shape(sh), params, lora, ref_pk["tokens"], ref_pk["cu_seqlens"], ref_pk["loss_mask"])
    loss_tol, grad_tol = (2e-3, 3e-2) if bf16 else (1e-4, 1e-4)
    assert res["count"] == f["count"] and f["count"] > 0
    assert rel_err(res["loss"], f["loss"]) <= loss_tol, (res["loss"], f["loss"])
    errs = {}
    for l in range(sh.n_layers):
        assert set(model.lora_grads[l]) == set(sh.lora_targets)
        for name, (dA, dB) in model.lora_grads[l].items():
            errs["L%d.%s.A" % (l, name)] = grad_norm_err(G.to_np(dA), g["lora"][l][name][0])
            errs["L%d.%s.B" % (l, name)] = grad_norm_err(G.to_np(dB), g["lora"][l][name][1])
            assert np.abs(g["lora"][l][name][0]).max() > 0 and np.abs(g["lora"][l][name][1]).max() > 0
    bad = {k: v for k, v in errs.items() if v > grad_tol}
    assert not bad, (bad, margin)
    return res, {k: (G.to_np(a), G.to_np(b)) for l in range(sh.n_layers) for k, (a, b) in
                 (("L%d.%s" % (l, n), v) for n, v in model.lora_grads[l].items())}, max(errs.values())


def test_moe_fp32_random_router_all_recompute_modes():
    sh = synth.CONFIGS[1].replace(**MOE)
    trajs = random_trajs(16, 6, sh.vocab, turn_lo=8, turn_hi=30, turns=(2, 5))
    params, lora = synth.weights(sh, 16), synth.lora_weights(sh, 16)
    outs = [_compare(sh, params, lora, trajs, 2, 200, False, rc) for rc in (0, 1, 2)]
    print("moe fp32 worst grad err %.2e" % outs[0][2])
    for o in outs[1:]:
        assert o[0] == outs[0][0]
        for k in o[1]:
            assert np.array_equal(o[1][k][0], outs[0][1][k][0]) and np.array_equal(o[1][k][1], outs[0][1][k][1])


@pytest.mark.parametrize("bf16", [False, True])
def test_moe_structured_router(bf16):
    sh = synth.CONFIGS[1].replace(**dict(MOE, d_model=128, ffn=192, head_dim=64, n_q_heads=2, n_kv_heads=1, lora_rank=8, lora_alpha=16.0))
    trajs = random_trajs(3, 8, sh.vocab, turn_lo=10, turn_hi=40, turns=(2, 5))
    params, lora = structured_router_params(sh, 3), synth.lora_weights(sh, 3)
    res, _, worst = _compare(sh, params, lora, trajs, 2, 384, bf16, 2)
    print("moe structured %s worst grad err %.2e" % ("bf16" if bf16 else "fp32", worst))


def test_moe_experts_without_tokens_and_single_token_segment():
    """Routing that only ever picks experts 0..3 leaves four experts without rows."""
    sh = synth.CONFIGS[1].replace(**MOE)
    params, lora = structured_router_params(sh, 5, live=4), synth.lora_weights(sh, 5)
    trajs = [[(1, np.array([5], dtype=np.int32))], [(1, np.array([5], dtype=np.int32)), (2, np.array([9, 3], dtype=np.int32))]]
    trajs += random_trajs(2, 3, sh.vocab, turn_lo=3, turn_hi=9)
    pk = oracle.pack(trajs, 96, 1)
    f = oracle.forward(oracle.config_from_shape(sh), params, lora, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    assert all(int(c["ffn"]["sel"].max()) <= 3 for c in f["cache"]["layers"])
    _compare(sh, params, lora, trajs, 1, 96, False, 0)
    _compare(sh, params, lora, trajs, 1, 96, True, 2)
