"""Helpers for the GPU parity tests (imported only by tests marked gpu)."""
import numpy as np
import torch

import oracle
import synth
from paper_2503_22673_amd import binding as B
from helpers import grad_norm_err, rel_err

DEV = "cuda"


def to_dev(x, dtype):
    return torch.from_numpy(np.ascontiguousarray(x)).to(device=DEV, dtype=dtype).contiguous()


def to_np(t):
    return t.detach().to(torch.float64).cpu().numpy()


def quantise(x, bf16):
    """Round host float64 data to what the device will hold, so that the
    reference sees the same inputs as the kernels."""
    t = torch.from_numpy(np.ascontiguousarray(x))
    t = t.to(torch.bfloat16) if bf16 else t.to(torch.float32)
    return t.to(torch.float64).numpy()


def quantise_params(P, bf16):
    return dict(embed=quantise(P["embed"], bf16), head=quantise(P["head"], bf16), g_final=quantise(P["g_final"], bf16),
                layers=[{k: quantise(v, bf16) for k, v in W.items()} for W in P["layers"]])


def quantise_lora(Lo):
    if Lo is None:
        return None
    return [{k: (quantise(A, False), quantise(B_, False)) for k, (A, B_) in L.items()} for L in Lo]


def run_step(sh, params, lora, trajs, rows, row_len, mode=None, recompute=None, train_mode=None, skip=True):
    """Packs on the GPU, runs one step, returns (out dict on host, model, pack dict, ctx)."""
    ctx = B.Context(B.make_config(sh, mode=mode, recompute=recompute, train_mode=train_mode))
    pk = ctx.pack(*synth.flatten_trajectories(trajs), row_len, rows)
    torch.cuda.synchronize()
    n_rows = pk["n_rows"]
    hcu = pk["cu_seqlens"].cpu().numpy()
    model = B.DeviceModel(ctx, params, lora)
    ws = torch.empty(ctx.workspace_bytes(n_rows, row_len), dtype=torch.uint8, device=DEV)
    out = ctx.train_step(model, pk["tokens"], pk["cu_seqlens"], hcu, pk["loss_mask"], n_rows, row_len, ws,
                         seg_skip=pk["seg_skip"] if skip else None)
    torch.cuda.synchronize()
    res = dict(loss=float(out["loss"].item()), loss_sum=float(out["loss_sum"].item()), count=int(out["count"].item()))
    return res, model, pk, ctx


def compare_step(sh, seed, trajs, rows, row_len, bf16, loss_tol, grad_tol, recompute=None, full=False, skip=True):
    """Whole-step parity against the float64 reference on the same (rounded) inputs."""
    params = quantise_params(synth.weights(sh, seed), bf16)
    lora = None if full else quantise_lora(synth.lora_weights(sh, seed))
    mode = B.AS_BF16 if bf16 else B.AS_FP32
    res, model, pk, ctx = run_step(sh, params, lora, trajs, rows, row_len, mode=mode, recompute=recompute,
                                   train_mode=B.AS_FULL if full else B.AS_LORA, skip=skip)
    ref_pk = oracle.pack(trajs, row_len, rows)
    assert np.array_equal(pk["tokens"].cpu().numpy(), ref_pk["tokens"])
    assert np.array_equal(pk["loss_mask"].cpu().numpy(), ref_pk["loss_mask"])
    assert np.array_equal(pk["cu_seqlens"].cpu().numpy(), ref_pk["cu_seqlens"])
    cfg = oracle.config_from_shape(sh if not full else sh.replace(lora_rank=0, lora_alpha=0.0, lora_targets=()))
    f, g = oracle.train_step(cfg, params, lora, ref_pk["tokens"], ref_pk["cu_seqlens"], ref_pk["loss_mask"])
    assert res["count"] == f["count"]
    report = dict(loss=res["loss"], ref_loss=f["loss"], loss_rel=rel_err(res["loss"], f["loss"]), grads={})
    assert report["loss_rel"] <= loss_tol, report
    assert rel_err(res["loss_sum"], f["loss_sum"]) <= loss_tol
    worst = 0.0
    if not full:
        for l in range(sh.n_layers):
            for name, (dA, dB) in model.lora_grads[l].items():
                for tag, got, ref in (("A", dA, g["lora"][l][name][0]), ("B", dB, g["lora"][l][name][1])):
                    e = grad_norm_err(to_np(got), ref)
                    report["grads"]["L%d.%s.%s" % (l, name, tag)] = e
                    worst = max(worst, e)
    else:
        gw = g["weights"]
        for k in ("embed", "head", "g_final"):
            e = grad_norm_err(to_np(model.w_grads[k]), gw[k]); report["grads"][k] = e; worst = max(worst, e)
        for l in range(sh.n_layers):
            for k, t in model.w_grads["layers"][l].items():
                e = grad_norm_err(to_np(t), gw["layers"][l][k]); report["grads"]["L%d.%s" % (l, k)] = e; worst = max(worst, e)
    report["worst_grad"] = worst
    bad = {k: v for k, v in report["grads"].items() if v > grad_tol}
    assert not bad, (bad, report["loss_rel"])
    return report
