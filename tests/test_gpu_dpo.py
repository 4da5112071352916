"""Parity of the preference (DPO) entry points against the float64 reference (oracle/dpo.py).

Tolerances: the per-segment log-probability sums pi_s carry the tier's loss tolerance (fp32 1e-4, bf16 2e-3,
relative to |pi_s|).  The pair loss and the factor of every gradient row are functions of
z_p = beta [(pi_c - ref_c) - (pi_r - ref_r)] with slope at most 1 in z (|d log(1+e^-z)/dz| <= 1,
|d log sigmoid(-z)/dz| <= 1), so an error dz in z moves the loss by at most dz and a gradient by at most a
relative dz: the loss tolerance is the observed max |dz| (itself bounded by the pi tolerance) plus float
rounding, the gradient tolerance the tier's (1e-4 / 3e-2) plus that max |dz|."""
import numpy as np
import pytest
import torch

import oracle
from oracle import model as om
from oracle import dpo
import synth
from helpers import random_trajs, grad_norm_err

pytestmark = pytest.mark.gpu


def _run(sh, seed, trajs, rows, row_len, pairs, beta, bf16, full=False, skip=True, recompute=None):
    import gpu_util as G
    from paper_2503_22673_amd import binding as B
    params = G.quantise_params(synth.weights(sh, seed), bf16)
    lora = None if full else G.quantise_lora(synth.lora_weights(sh, seed))
    ref_params = G.quantise_params(synth.weights(sh, seed + 100), bf16) if full else params      # frozen reference policy
    ctx = B.Context(B.make_config(sh, mode=B.AS_BF16 if bf16 else B.AS_FP32, recompute=recompute,
                                  train_mode=B.AS_FULL if full else B.AS_LORA))
    pk = ctx.pack(*synth.flatten_trajectories(trajs), row_len, rows)
    torch.cuda.synchronize()
    n_rows, hcu = pk["n_rows"], pk["cu_seqlens"].cpu().numpy()
    ref_pk = oracle.pack(trajs, row_len, rows)
    assert np.array_equal(hcu, ref_pk["cu_seqlens"]) and np.array_equal(pk["tokens"].cpu().numpy(), ref_pk["tokens"])
    cfg = oracle.config_from_shape(sh if not full else sh.replace(lora_rank=0, lora_alpha=0.0, lora_targets=()))
    tok, cu, mask = ref_pk["tokens"], ref_pk["cu_seqlens"], ref_pk["loss_mask"]
    ref = dpo.sequence_logps(om.forward(cfg, ref_params, None, tok, cu, mask), cu)
    want, g = dpo.dpo_step(cfg, params, lora, tok, cu, mask, pairs, ref, beta)
    model = B.DeviceModel(ctx, params, lora)
    ws = torch.empty(ctx.workspace_bytes(n_rows, row_len), dtype=torch.uint8, device="cuda")
    sk = pk["seg_skip"] if skip else None
    args = (pk["tokens"], pk["cu_seqlens"], hcu, pk["loss_mask"], n_rows, row_len, ws)
    # reference sums on the device: adapters off (LoRA), the other weights (full)
    ref_model = model if not full else B.DeviceModel(ctx, ref_params, None)
    ref_dev = ctx.sequence_logps(ref_model, *args, seg_skip=sk, adapters=False)
    out = ctx.dpo_step(model, *args, pairs, torch.from_numpy(ref.astype(np.float32)).cuda(), beta, seg_skip=sk)
    torch.cuda.synchronize()
    return dict(ctx=ctx, model=model, pk=pk, args=args, want=want, g=g, ref=ref, ref_dev=ref_dev.cpu().numpy().astype(np.float64),
                logp=out["logp"].cpu().numpy().astype(np.float64), stats=out["stats"].cpu().numpy().astype(np.float64), full=full, sh=sh)


def _check(r, pairs, beta, bf16):
    pi_tol, grad_tol = (2e-3, 3e-2) if bf16 else (1e-4, 1e-4)
    want = r["want"]
    scale = np.maximum(np.abs(want["logp"]), 1.0)
    assert np.all(np.abs(r["logp"] - want["logp"]) <= pi_tol * scale), (r["logp"], want["logp"])
    assert np.all(np.abs(r["ref_dev"] - r["ref"]) <= pi_tol * np.maximum(np.abs(r["ref"]), 1.0)), (r["ref_dev"], r["ref"])
    assert np.all(r["logp"][want["logp"] == 0] == 0)                      # segments without target: exactly 0
    ref32 = r["ref"].astype(np.float32).astype(np.float64)               # what the device was given
    z_dev = np.array([beta * ((r["logp"][c] - ref32[c]) - (r["logp"][q] - ref32[q])) for c, q in pairs])
    dz = float(np.abs(z_dev - want["z"]).max()) if len(pairs) else 0.0
    assert abs(r["stats"][0] - want["loss"]) <= dz + 1e-6 * max(1.0, abs(want["loss"])), (r["stats"], want["loss"], dz)
    assert abs(r["stats"][1] - want["margin"]) <= dz + 1e-6 * max(1.0, abs(want["margin"]))
    if len(pairs) and np.abs(want["z"]).min() > 2 * dz:
        assert r["stats"][2] == pytest.approx(want["accuracy"], abs=1e-6)
    tol = grad_tol + dz
    bad, worst = {}, 0.0
    if not r["full"]:
        for l in range(r["sh"].n_layers):
            for name, (dA, dB) in r["model"].lora_grads[l].items():
                for tag, got, ref in (("A", dA, r["g"]["lora"][l][name][0]), ("B", dB, r["g"]["lora"][l][name][1])):
                    e = grad_norm_err(got.float().cpu().numpy(), ref); worst = max(worst, e)
                    if e > tol: bad["L%d.%s.%s" % (l, name, tag)] = e
    else:
        gw, wg = r["g"]["weights"], r["model"].w_grads
        for k in ("embed", "head", "g_final"):
            e = grad_norm_err(wg[k].float().cpu().numpy(), gw[k]); worst = max(worst, e)
            if e > tol: bad[k] = e
        for l in range(r["sh"].n_layers):
            for k, t in wg["layers"][l].items():
                e = grad_norm_err(t.float().cpu().numpy(), gw["layers"][l][k]); worst = max(worst, e)
                if e > tol: bad["L%d.%s" % (l, k)] = e
    assert not bad, (bad, dz)
    return dz, worst


@pytest.mark.parametrize("bf16", [False, True])
def test_config1_pairs(bf16):
    sh = synth.CONFIGS[1]
    pairs, beta = [(0, 1), (2, 3), (3, 0)], 0.1
    r = _run(sh, 0, synth.workload(1, 0), 1, 512, pairs, beta, bf16)
    dz, worst = _check(r, pairs, beta, bf16)
    print("config1 dpo %s: max dz %.2e worst grad %.2e loss %.6f (ref %.6f)" % ("bf16" if bf16 else "fp32", dz, worst, r["stats"][0], r["want"]["loss"]))
    if not bf16:
        assert dz < 1e-3                                                   # float32 sums of a few hundred terms


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("recompute", [0, 1, 2])
def test_seven_targets_gqa_two_rows_skipped_tails(bf16, recompute):
    """Grouped KV heads, all seven adapters, two rows whose pad tails are left out of the computation (the
    segment indices of the pairs are the caller's, before the tails are squeezed out), a segment in two pairs
    and segments in none, large beta so that the pair factors differ."""
    sh = synth.CONFIGS[1].replace(n_layers=3, n_q_heads=4, n_kv_heads=2, head_dim=64, d_model=128, ffn=200,
                                  lora_targets=synth.DENSE_TARGETS7, lora_rank=8, lora_alpha=16.0, recompute=recompute)
    trajs = random_trajs(3, 9, sh.vocab, turn_lo=10, turn_hi=40, turns=(2, 5))
    pk = oracle.pack(trajs, 320, 2)
    cu = pk["cu_seqlens"]
    skip = np.array([not pk["loss_mask"][cu[s] + 1:cu[s + 1]].any() for s in range(len(cu) - 1)])      # no target inside
    live = [s for s in range(len(cu) - 1) if not skip[s]]
    assert len(live) >= 5 and skip.any() and live != list(range(len(live)))        # a skipped segment sits between live ones
    pairs, beta = [(live[0], live[1]), (live[3], live[2]), (live[4], live[0])], 0.5
    r = _run(sh, 1, trajs, 2, 320, pairs, beta, bf16, recompute=recompute)
    _check(r, pairs, beta, bf16)
    # not squeezing the tails out gives the same numbers (not the same bits: rows sit in other tiles)
    r2 = _run(sh, 1, trajs, 2, 320, pairs, beta, bf16, recompute=recompute, skip=False)
    _check(r2, pairs, beta, bf16)
    assert np.allclose(r["logp"], r2["logp"], rtol=2e-3 if bf16 else 1e-5, atol=0)
    assert np.array_equal(r["logp"] == 0, r2["logp"] == 0)


def test_full_fine_tuning_fp32():
    sh = synth.CONFIGS[1].replace(n_layers=2, lora_rank=0, lora_alpha=0.0, lora_targets=(), full_ft=True)
    pairs, beta = [(0, 1), (2, 3)], 0.05
    r = _run(sh, 2, synth.workload(1, 0), 1, 512, pairs, beta, False, full=True)
    dz, worst = _check(r, pairs, beta, False)
    print("full-FT dpo fp32: max dz %.2e worst grad %.2e" % (dz, worst))


def test_policy_equal_to_reference_gives_ln2_and_half_beta_factors():
    """LoRA with B = 0: the policy is the base model, every z is 0 whatever the data; loss ln 2, accuracy 0."""
    import gpu_util as G
    from paper_2503_22673_amd import binding as B
    sh = synth.CONFIGS[1]
    params, lora = synth.weights(sh, 0), synth.lora_weights(sh, 0, zero_b=True)
    ctx = B.Context(B.make_config(sh, mode=B.AS_FP32))
    pk = ctx.pack(*synth.flatten_trajectories(synth.workload(1, 0)), 512, 1)
    hcu = pk["cu_seqlens"].cpu().numpy()
    model = B.DeviceModel(ctx, params, lora)
    ws = torch.empty(ctx.workspace_bytes(1, 512), dtype=torch.uint8, device="cuda")
    args = (pk["tokens"], pk["cu_seqlens"], hcu, pk["loss_mask"], 1, 512, ws)
    ref = ctx.sequence_logps(model, *args, adapters=False)
    pol = ctx.sequence_logps(model, *args, adapters=True)
    assert torch.equal(ref, pol)                                            # the zero adapter term changes no bit
    out = ctx.dpo_step(model, *args, [(0, 1), (2, 3)], ref, 0.3)
    torch.cuda.synchronize()
    st = out["stats"].cpu().numpy()
    assert st[0] == pytest.approx(np.log(2.0), rel=1e-6) and st[1] == 0.0 and st[2] == 0.0
    assert torch.equal(out["logp"], ref)
    for Lg in model.lora_grads:
        for dA, dB in Lg.values():
            assert not dA.any().item() and dB.any().item()                 # dA = s B^T(...) = 0, dB live


def test_no_pair_and_invalid_arguments():
    import gpu_util as G
    from paper_2503_22673_amd import binding as B
    sh = synth.CONFIGS[1]
    ctx = B.Context(B.make_config(sh, mode=B.AS_FP32))
    pk = ctx.pack(*synth.flatten_trajectories(synth.workload(1, 0)), 512, 1)
    hcu = pk["cu_seqlens"].cpu().numpy()
    S = len(hcu) - 1
    model = B.DeviceModel(ctx, synth.weights(sh, 0), synth.lora_weights(sh, 0))
    ws = torch.empty(ctx.workspace_bytes(1, 512), dtype=torch.uint8, device="cuda")
    args = (pk["tokens"], pk["cu_seqlens"], hcu, pk["loss_mask"], 1, 512, ws)
    ref = torch.zeros(S, dtype=torch.float32, device="cuda")
    out = ctx.dpo_step(model, *args, np.zeros((0, 2), dtype=np.int32), ref, 0.1)
    torch.cuda.synchronize()
    assert not out["stats"].any().item()
    for Lg in model.lora_grads:
        for dA, dB in Lg.values():
            assert not dA.any().item() and not dB.any().item()
    for bad_pairs, beta in (([(0, S)], 0.1), ([(-1, 0)], 0.1), ([(1, 1)], 0.1), ([(0, 1)], -0.5), ([(0, 1)], float("nan"))):
        with pytest.raises(B.ASError) as e:
            ctx.dpo_step(model, *args, bad_pairs, ref, beta)
        assert e.value.code == B.ERR["SHAPE"]


def test_batch_without_any_target():
    """Every turn a user turn: all segments are left out of the computation; log-probabilities are 0, the pair
    loss follows from the reference sums alone, the gradients are exactly zero."""
    import math
    from paper_2503_22673_amd import binding as B
    sh = synth.CONFIGS[1]
    trajs = [[(1, t) for _, t in tr] for tr in synth.workload(1, 0)]
    ctx = B.Context(B.make_config(sh, mode=B.AS_FP32))
    pk = ctx.pack(*synth.flatten_trajectories(trajs), 512, 1)
    hcu = pk["cu_seqlens"].cpu().numpy()
    assert pk["seg_skip"].all()
    model = B.DeviceModel(ctx, synth.weights(sh, 0), synth.lora_weights(sh, 0))
    for Lg in model.lora_grads:
        for dA, dB in Lg.values():
            dA.fill_(1.0); dB.fill_(1.0)
    ws = torch.empty(ctx.workspace_bytes(1, 512), dtype=torch.uint8, device="cuda")
    args = (pk["tokens"], pk["cu_seqlens"], hcu, pk["loss_mask"], 1, 512, ws)
    lp = ctx.sequence_logps(model, *args, seg_skip=pk["seg_skip"])
    assert not lp.any().item()
    ref = torch.tensor([-3.0, -1.0] + [0.0] * (len(hcu) - 3), dtype=torch.float32, device="cuda")
    out = ctx.dpo_step(model, *args, [(0, 1)], ref, 0.5, seg_skip=pk["seg_skip"])
    torch.cuda.synchronize()
    z = 0.5 * ((0.0 - -3.0) - (0.0 - -1.0))                                   # = 1
    want = dpo.dpo_loss(np.zeros(len(hcu) - 1), ref.cpu().numpy(), [(0, 1)], 0.5)
    st = out["stats"].cpu().numpy()
    assert st[0] == pytest.approx(math.log1p(math.exp(-z)), rel=1e-6) and st[0] == pytest.approx(want["loss"], rel=1e-6)
    assert st[1] == pytest.approx(z) and st[2] == 1.0
    assert not out["logp"].any().item()
    for Lg in model.lora_grads:
        for dA, dB in Lg.values():
            assert not dA.any().item() and not dB.any().item()
