"""NF4 quantised frozen base: quantise / dequantise kernels against the reference (codes bit for bit),
and the whole LoRA step on a quantised base against the float64 reference run on the dequantised weights."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle import nf4
from helpers import grad_norm_err, random_trajs, rel_err

pytestmark = pytest.mark.gpu
PROJ = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_quantise_and_dequantise_kernels(dtype):
    from paper_2503_22673_amd import binding as B
    ctx = B.Context(B.make_config(synth.CONFIGS[1]))
    g = synth.rng(4, 31)
    w = 0.02 * g.standard_normal(64 * 1000 + 64 * 3)
    w[64:128] = 0.0                                            # an all-zero block
    w[128:192] *= 1e-30                                        # a block of tiny values
    w[200] = 3.0                                               # an outlier sets its block's maximum
    wt = torch.from_numpy(w).to(dtype).cuda()
    w_dev = wt.to(torch.float64).cpu().numpy()                 # what the device holds
    codes_ref, absmax_ref = nf4.quantise(w_dev)
    codes, absmax = ctx.nf4_quantize(wt)
    torch.cuda.synchronize()
    assert np.array_equal(absmax.cpu().numpy(), absmax_ref)
    assert np.array_equal(codes.cpu().numpy(), nf4.pack_codes(codes_ref))            # bit for bit, packing included
    out = ctx.nf4_dequantize(codes, absmax, dtype)
    torch.cuda.synchronize()
    ref = nf4.dequantise(codes_ref, absmax_ref)
    got = out.to(torch.float64).cpu().numpy()
    if dtype == torch.float32:
        assert np.array_equal(got, ref.astype(np.float32).astype(np.float64))
    else:                                                      # float product rounded to bf16: within one rounding of the exact product
        assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref))


def _quantised_model(sh, seed, bf16):
    """Host-side preparation with the reference quantiser: device params (codes + maxima) and the dense
    weights the kernels will see after dequantisation (for the float64 reference)."""
    P = synth.weights(sh, seed)
    dev, ref = dict(embed=P["embed"], head=P["head"], g_final=P["g_final"], layers=[]), None
    dt = torch.bfloat16 if bf16 else torch.float32
    rnd = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dt).to(torch.float64).numpy()
    ref = dict(embed=rnd(P["embed"]), head=rnd(P["head"]), g_final=rnd(P["g_final"]), layers=[])
    for W in P["layers"]:
        dW, rW = dict(g1=W["g1"], g2=W["g2"]), dict(g1=rnd(W["g1"]), g2=rnd(W["g2"]))
        for k in PROJ:
            codes, absmax = nf4.quantise(rnd(W[k]))            # the weights are first held in the device type, then quantised
            dW[k] = nf4.pack_codes(codes)
            dW["a" + k[1:]] = absmax
            lv = nf4.LEVELS.astype(np.float32)[codes.reshape(-1, 64)] * absmax[:, None]     # float32 product, as the kernel
            rW[k] = rnd(lv.reshape(W[k].shape))
        dev["layers"].append(dW); ref["layers"].append(rW)
    return dev, ref


@pytest.mark.parametrize("bf16", [False, True])
def test_lora_step_on_nf4_base(bf16):
    from paper_2503_22673_amd import binding as B
    import gpu_util as G
    sh = synth.CONFIGS[1].replace(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=32, d_model=128, ffn=192,
                                  lora_targets=synth.DENSE_TARGETS7, lora_rank=8, lora_alpha=16.0)
    dev, ref = _quantised_model(sh, 6, bf16)
    lora = G.quantise_lora(synth.lora_weights(sh, 6))
    trajs = random_trajs(6, 7, sh.vocab, turn_lo=8, turn_hi=30, turns=(2, 5))
    rows, row_len = 2, 256
    mode = B.AS_BF16 if bf16 else B.AS_FP32
    outs = []
    for rc in (0, 2):
        ctx = B.Context(B.make_config(sh, mode=mode, recompute=rc, weight_format=B.AS_W_NF4))
        pk = ctx.pack(*synth.flatten_trajectories(trajs), row_len, rows)
        model = B.DeviceModel(ctx, dev, lora)
        ws = torch.empty(ctx.workspace_bytes(pk["n_rows"], row_len), dtype=torch.uint8, device="cuda")
        out = ctx.train_step(model, pk["tokens"], pk["cu_seqlens"], pk["cu_seqlens"].cpu().numpy(), pk["loss_mask"],
                             pk["n_rows"], row_len, ws, seg_skip=pk["seg_skip"])
        torch.cuda.synchronize()
        outs.append((float(out["loss"].item()), int(out["count"].item()), model))
    ref_pk = oracle.pack(trajs, row_len, rows)
    f, g = oracle.train_step(oracle.config_from_shape(sh), ref, lora, ref_pk["tokens"], ref_pk["cu_seqlens"], ref_pk["loss_mask"])
    loss_tol, grad_tol = (2e-3, 3e-2) if bf16 else (1e-4, 1e-4)
    loss, count, model = outs[0]
    assert count == f["count"] and rel_err(loss, f["loss"]) <= loss_tol
    worst = 0.0
    for l in range(sh.n_layers):
        for name, (dA, dB) in model.lora_grads[l].items():
            worst = max(worst, grad_norm_err(G.to_np(dA), g["lora"][l][name][0]), grad_norm_err(G.to_np(dB), g["lora"][l][name][1]))
    assert worst <= grad_tol, worst
    # the quantised base is a different model: the reference on the unquantised weights has other gradients,
    # well outside the tolerance, so the comparison above does see the quantisation
    _, g_dense = oracle.train_step(oracle.config_from_shape(sh), G.quantise_params(synth.weights(sh, 6), bf16), lora,
                                   ref_pk["tokens"], ref_pk["cu_seqlens"], ref_pk["loss_mask"])
    assert grad_norm_err(g_dense["lora"][0]["q"][0], g["lora"][0]["q"][0]) > 3 * grad_tol
    # recompute mode changes nothing
    assert outs[1][0] == loss
    for l in range(sh.n_layers):
        for name in model.lora_grads[l]:
            assert torch.equal(model.lora_grads[l][name][0], outs[1][2].lora_grads[l][name][0])


def test_nf4_config_checks():
    from paper_2503_22673_amd import binding as B
    sh = synth.CONFIGS[1]
    for kw in (dict(train_mode=B.AS_FULL), ):
        with pytest.raises(B.ASError):
            B.Context(B.make_config(sh, weight_format=B.AS_W_NF4, **kw))
    with pytest.raises(B.ASError):
        B.Context(B.make_config(sh.replace(ffn=344), weight_format=B.AS_W_NF4))       # 344 is no multiple of 64
    B.Context(B.make_config(sh.replace(ffn=320), weight_format=B.AS_W_NF4)).close()
