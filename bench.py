"""Throughput of one LoRA fine-tuning step (forward + backward) on one MI355X.

A step is one pass of the whole hot path over one packed batch: embedding,
all layers forward, fused head + masked cross-entropy, all layers backward,
adapter gradients.  Inputs (weights, adapters, packed tokens, masks) are in
HBM before the timed region; packing and AdamW are timed separately and
reported beside the headline value.

Prints ONE JSON line (the README lists the fields).
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
# HBM-side bytes per launch of the dominant kernel at config 3: FETCH_SIZE and WRITE_SIZE of two counter runs over one
# bench step, each scaled by what the counter reads for a 1 GiB copy (profiles/bench_config3_counters.md).  The figure
# belongs to the kernel sources those runs saw: the digest below names them, and the line reports null when they differ.
TRAFFIC_BYTES_PER_LAUNCH = {(3, "gemm_mfma_rs_kernel<0, 0>"): 13.15e9}
TRAFFIC_SOURCES = ("gemm.hip", "gemm_rs_loop.inc", "common.h")
TRAFFIC_SOURCE_DIGEST = "c18174f2a2f31f2f"
DOMINANT_KERNEL = "gemm_mfma_rs_kernel<0, 0>"                  # dense models; expert GEMMs: the same kernel with live-row limits, <1>
GROUPED_KERNEL = "gemm_mfma_rs_kernel<1, 0>"


def kernel_sources_digest():
    """Digest of the sources of the dominant kernel, to tie the stored counter figure to the code it was taken on."""
    import hashlib
    h = hashlib.sha256()
    for f in TRAFFIC_SOURCES:
        with open(os.path.join(ROOT, "paper_2503_22673_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def device_weights(sh, seed, dtype):
    """Random-init weights of the architecture, drawn on the device."""
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    D, Dkv, d, F = sh.n_q_heads * sh.head_dim, sh.n_kv_heads * sh.head_dim, sh.d_model, sh.ffn

    def mat(*shape):
        return torch.empty(shape, dtype=dtype, device="cuda").normal_(0.0, 0.02, generator=g)

    def ones():
        return torch.ones(d, dtype=dtype, device="cuda")

    P = dict(embed=mat(sh.vocab, d), head=mat(sh.vocab, d), g_final=ones(), layers=[])
    E = sh.n_experts
    for _ in range(sh.n_layers):
        W = dict(g1=ones(), wq=mat(D, d), wk=mat(Dkv, d), wv=mat(Dkv, d), wo=mat(d, D), g2=ones())
        if E:
            W.update(wgate=mat(E, F, d), wup=mat(E, F, d), wdown=mat(E, d, F), wrouter=mat(E, d))
        else:
            W.update(wgate=mat(F, d), wup=mat(F, d), wdown=mat(d, F))
        P["layers"].append(W)
    return P


def device_lora(sh, seed):
    import torch
    import synth
    g = torch.Generator(device="cuda")
    g.manual_seed(seed + 1)
    dims = synth.lora_dims(sh)
    out = []
    for _ in range(sh.n_layers):
        L = {}
        for t in sh.lora_targets:
            din, dout = dims[t]
            L[t] = (torch.empty(sh.lora_rank, din, dtype=torch.float32, device="cuda").normal_(0.0, 0.02, generator=g),
                    torch.empty(dout, sh.lora_rank, dtype=torch.float32, device="cuda").normal_(0.0, 0.02, generator=g))
        out.append(L)
    return out


def algorithmic_flops(sh, seg_lens_nonpad, n_nonpad, n_targets, dpo=False):
    """Flops the method must do for this batch: causal half of attention inside
    each trajectory only, no weight gradients for frozen matrices, head on
    target rows only, no recompute, nothing for pad tokens."""
    D, Dkv, d, F, L, V, r = (sh.n_q_heads * sh.head_dim, sh.n_kv_heads * sh.head_dim, sh.d_model, sh.ffn, sh.n_layers,
                             sh.vocab, sh.lora_rank)
    # a sparse layer runs top_k expert FFNs and the router per token
    p_layer = d * (D + 2 * Dkv) + D * d + (sh.top_k * 3 * d * F + d * sh.n_experts if sh.n_experts else 3 * d * F)
    dense = (6.0 if sh.full_ft else 4.0) * L * p_layer * n_nonpad
    attn = 7.0 * D * L * float(sum(x * x for x in seg_lens_nonpad))
    import synth
    dims = synth.lora_dims(sh)
    lora = 6.0 * r * sum(sum(dims[t]) for t in sh.lora_targets) * L * n_nonpad
    head = (6.0 if sh.full_ft else 4.0) * d * V * n_targets
    if dpo:     # forward of the frozen reference policy (no adapters), and the first of the two passes over the head
        dense += 2.0 * L * p_layer * n_nonpad
        attn += 2.0 * D * L * float(sum(x * x for x in seg_lens_nonpad))
        head += 2.0 * 2.0 * d * V * n_targets
    recompute = 0.0
    if sh.recompute == 1:
        recompute = (2.0 * p_layer * n_nonpad + 2.0 * D * float(sum(x * x for x in seg_lens_nonpad)) +
                     2.0 * r * sum(sum(dims[t]) for t in sh.lora_targets) * n_nonpad) * (L - 1)
    return dict(dense=dense, attention=attn, lora=lora, head=head, total=dense + attn + lora + head, recompute=recompute)


def cpu_baseline(sh, seed, budget_tokens=2048):
    """The float64 reference, as it stands, timed on the host on a bounded
    sample: true layer widths and vocabulary, one packed row of `budget_tokens`
    tokens, models of 1 and 2 layers; per-layer and head cost are separated by
    the difference and extrapolated linearly to the full depth."""
    import numpy as np
    import oracle
    import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    rs = np.random.default_rng(seed)
    pool = 0.02 * rs.standard_normal(1 << 20)

    def mat(*shape):
        n = int(np.prod(shape))
        return np.resize(pool, n).reshape(shape)

    d, F, D, Dkv = sh.d_model, sh.ffn, sh.n_q_heads * sh.head_dim, sh.n_kv_heads * sh.head_dim

    def params(n_layers):
        return dict(embed=mat(sh.vocab, d), head=mat(sh.vocab, d), g_final=np.ones(d),
                    layers=[dict(g1=np.ones(d), wq=mat(D, d), wk=mat(Dkv, d), wv=mat(Dkv, d), wo=mat(d, D), g2=np.ones(d),
                                 wgate=mat(F, d), wup=mat(F, d), wdown=mat(d, F)) for _ in range(n_layers)])

    trajs = synth.trajectories_lognormal(seed, 1, budget_tokens, sh.vocab, budget_tokens // 3, 0.4, 16, budget_tokens,
                                         turns=(2, 6), assistant_share=0.2)
    pk = oracle.pack(trajs, budget_tokens, 1)
    times = {}
    for nl in (1, 2):
        s2 = sh.replace(n_layers=nl)
        cfg = oracle.config_from_shape(s2)
        P = params(nl)
        Lo = synth.lora_weights(s2, seed)
        t0 = time.perf_counter()
        oracle.train_step(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
        times[nl] = time.perf_counter() - t0
    per_layer = max(times[2] - times[1], 1e-9)
    rest = max(times[1] - per_layer, 0.0)
    full = rest + sh.n_layers * per_layer
    nonpad = int(sum(sum(len(t) for _, t in tr) for tr in trajs))
    return dict(value=nonpad / full, unit="trained tokens/s (extrapolated)", cores=int(cores), kind="oracle",
                sample="float64 numpy reference, true widths and vocab, one %d-token packed row (%d non-pad), "
                       "1- and 2-layer models timed (%.1f s, %.1f s); per-layer and head cost separated by "
                       "difference and extrapolated linearly to %d layers" % (budget_tokens, nonpad, times[1], times[2], sh.n_layers))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3, help="benchmark configuration (2..5); 3 is the headline")
    ap.add_argument("--layers", type=int, default=0, help="override the depth (bring-up only; the result is then not the headline)")
    ap.add_argument("--recompute", type=int, default=-1, help="override the recompute mode (0, 1, 2)")
    ap.add_argument("--copy-probe", action="store_true", help="only copy 1 GiB device to device (calibrates the FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--rows", type=int, default=0, help="override the number of packed rows")
    ap.add_argument("--row-len", type=int, default=0, help="override the row length")
    ap.add_argument("--nf4", action="store_true", help="frozen base held as NF4 blocks (quantised base + LoRA)")
    ap.add_argument("--single-trajectory", action="store_true",
                    help="long-context stress: every row is ONE trajectory of row_len tokens")
    ap.add_argument("--bfd", action="store_true",
                    help="pack the rows by best fit decreasing from a pool three times the batch (as_pack_policy)")
    ap.add_argument("--dpo", action="store_true",
                    help="preference step instead of the supervised one: reference pass with the adapters off + "
                         "DPO step, consecutive trajectories paired as (chosen, rejected)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU; --gpus %d is not supported (it has no collectives)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    if args.copy_probe:
        import torch
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": 1 << 30}))
        return

    import numpy as np
    import torch
    import synth
    from paper_2503_22673_amd import binding as B

    sh = synth.CONFIGS[args.config]
    if args.layers:
        sh = sh.replace(n_layers=args.layers)
    if args.recompute >= 0:
        sh = sh.replace(recompute=args.recompute)
    if args.rows:
        sh = sh.replace(rows=args.rows)
    if args.row_len:
        sh = sh.replace(row_len=args.row_len)
    torch.cuda.set_device(0)
    ctx = B.Context(B.make_config(sh, weight_format=B.AS_W_NF4 if args.nf4 else B.AS_W_DENSE))
    if args.single_trajectory:
        trajs = synth.trajectories_lognormal(args.seed, sh.rows, sh.row_len, sh.vocab, sh.row_len, 0.0, sh.row_len, sh.row_len,
                                             turns=(8, 12), assistant_share=0.2)
    else:
        trajs = synth.workload(args.config, seed=args.seed, rows=(3 if args.bfd else 1) * sh.rows, row_len=sh.row_len)
    flat = synth.flatten_trajectories(trajs)
    # the first call also loads the library's code objects; the second is what a training loop pays per batch
    pack_first_ms = pack_ms = 0.0
    for i in range(2):
        t0 = time.perf_counter()
        pk = ctx.pack(*flat, sh.row_len, sh.rows, policy=B.AS_PACK_BEST_FIT_DECREASING if args.bfd else None)
        torch.cuda.synchronize()
        pack_ms = (time.perf_counter() - t0) * 1e3
        if i == 0:
            pack_first_ms = pack_ms
    assert pk["n_rows"] == sh.rows, pk["n_rows"]
    hcu = pk["cu_seqlens"].cpu().numpy()
    tok_h = pk["tokens"].cpu().numpy()
    consumed = trajs[:pk["n_traj_consumed"]] if not args.bfd else [tr for tr, r in zip(trajs, pk["traj_row"]) if r >= 0]
    seg_nonpad = [min(sum(len(t) for _, t in tr), sh.row_len) for tr in consumed if sum(len(t) for _, t in tr) > 0]
    n_nonpad = int(sum(seg_nonpad))
    N = sh.rows * sh.row_len

    dt = torch.bfloat16 if sh.bf16 else torch.float32
    params = device_weights(sh, args.seed, dt)
    weight_bytes = sum(v.numel() * v.element_size() for W in params["layers"] for v in W.values())
    if args.nf4:                                    # quantise the seven projections of every layer on the device
        for W in params["layers"]:
            for k in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown"):
                W[k], W["a" + k[1:]] = ctx.nf4_quantize(W[k])
        torch.cuda.synchronize()
        weight_bytes = sum(v.numel() * v.element_size() for W in params["layers"] for v in W.values())
    lora = None if sh.full_ft else device_lora(sh, args.seed)
    model = B.DeviceModel(ctx, params, lora)
    del params, lora
    ws = torch.empty(ctx.workspace_bytes(sh.rows, sh.row_len), dtype=torch.uint8, device="cuda")
    out = None

    live = [s for s in range(len(hcu) - 1) if not pk["seg_skip"][s]]
    pairs = np.asarray(live[:len(live) // 2 * 2], dtype=np.int32).reshape(-1, 2)
    dpo_out = None

    def step():
        nonlocal out, dpo_out
        if args.dpo:
            a = (model, pk["tokens"], pk["cu_seqlens"], hcu, pk["loss_mask"], sh.rows, sh.row_len, ws)
            ref = ctx.sequence_logps(*a, seg_skip=pk["seg_skip"], adapters=False)
            dpo_out = ctx.dpo_step(*a, pairs, ref, 0.1, seg_skip=pk["seg_skip"])
            return
        out = ctx.train_step(model, pk["tokens"], pk["cu_seqlens"], hcu, pk["loss_mask"], sh.rows, sh.row_len, ws, out,
                             seg_skip=pk["seg_skip"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: HIP events around the launches of the dominant kernel only (events around every launch cost 0.5 % of the step)
    dom = "gemm_grouped" if sh.n_experts else "gemm_mfma_rs"
    ctx.profile(True, only=dom)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = e0.elapsed_time(e1) / args.steps
    prof = ctx.profile_read()
    # one more step, outside the timed region, with events around every launch: the per-class breakdown
    ctx.profile(True)
    e2, e3 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e2.record()
    step()
    e3.record()
    torch.cuda.synchronize()
    prof_all, ms_extra = ctx.profile_read(), e2.elapsed_time(e3)
    ctx.profile(False)
    if args.dpo:
        loss = float(dpo_out["stats"][0].item())
        mask_h = pk["loss_mask"].cpu().numpy().astype(bool)
        first = np.zeros(len(mask_h), dtype=bool); first[hcu[:-1]] = True
        count = int((mask_h & ~first).sum())
    else:
        loss, count = float(out["loss"].item()), int(out["count"].item())
    assert math.isfinite(loss), loss

    fl = algorithmic_flops(sh, seg_nonpad, n_nonpad, count, dpo=args.dpo)
    tokens_per_s = n_nonpad / (ms_per_step * 1e-3)
    mfu = fl["total"] / (ms_per_step * 1e-3) / (PEAK_BF16_TFLOPS * 1e12)
    hfu = (fl["total"] + fl["recompute"]) / (ms_per_step * 1e-3) / (PEAK_BF16_TFLOPS * 1e12)
    n_l, ms_l, fl_l = prof[dom]
    ach = fl_l / (ms_l * 1e-3) / 1e12 if ms_l > 0 else 0.0
    breakdown = {k: round(v[1], 2) for k, v in prof_all.items() if v[0]}
    breakdown["untracked"] = round(ms_extra - sum(breakdown.values()), 2)

    # AdamW on the adapters (reported beside the step; not part of `value`)
    adam_ms = None
    if not sh.full_ft:
        ws_t, gs_t = [], []
        for Lw, Lg in zip(model.lora, model.lora_grads):
            for k in Lw:
                ws_t += [Lw[k][0], Lw[k][1]]
                gs_t += [Lg[k][0], Lg[k][1]]
        ms_t = [torch.zeros_like(w) for w in ws_t]
        vs_t = [torch.zeros_like(w) for w in ws_t]
        ctx.adamw_update(ws_t, None, gs_t, ms_t, vs_t, [0] * len(ws_t), 1, 1e-4, 0.9, 0.95, 1e-8, 0.0)
        torch.cuda.synchronize()
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record()
        ctx.adamw_update(ws_t, None, gs_t, ms_t, vs_t, [0] * len(ws_t), 2, 1e-4, 0.9, 0.95, 1e-8, 0.0)
        a1.record()
        torch.cuda.synchronize()
        adam_ms = a0.elapsed_time(a1)

    rec = {
        "metric": "trained tokens/s per MI355X (LoRA step, 8B shapes, 16k packed); % bf16 MFMA peak"
                  if args.config == 3 and not (args.rows or args.row_len or args.single_trajectory or args.layers or args.nf4 or args.dpo or args.bfd) else
                  "trained tokens/s per MI355X (one fine-tuning step, config %d%s)" % (
                      args.config, ", rows/row_len overridden" if (args.rows or args.row_len or args.single_trajectory) else "") +
                  (", NF4 base" if args.nf4 else "") + (", DPO step incl. reference pass" if args.dpo else "") + (", rows packed by best fit decreasing" if args.bfd else ""),
        "value": round(tokens_per_s, 1), "unit": "trained tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 2), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if sh.bf16 else "f32", "data": "synthetic",
        "config": {"workload": "config %d: %s, %d layers, %d rows x %d tokens packed, LoRA r=%d on %s, recompute=%s" % (
            args.config, sh.name, sh.n_layers, sh.rows, sh.row_len, sh.lora_rank, "/".join(sh.lora_targets) or "none (full FT)",
            {0: "none", 1: "full layer", 2: "selective (norm outputs, SwiGLU product)"}[sh.recompute]), "non_pad_tokens": n_nonpad, "packed_tokens": N, "segments": int(len(hcu) - 1),
            "loss_tokens": count, "mean_sq_len_over_len": round(sum(x * x for x in seg_nonpad) / max(n_nonpad, 1), 1)},
        "mfu_pct_of_bf16_peak": round(100 * mfu, 2), "hfu_pct_of_bf16_peak": round(100 * hfu, 2),
        "algorithmic_gflop_per_token": round(fl["total"] / n_nonpad / 1e9, 2),
        "layer_weight_gb": round(weight_bytes / 1e9, 2),
        "loss": round(loss, 5), "pack_ms": round(pack_ms, 2), "pack_first_call_ms": round(pack_first_ms, 2), "adamw_ms": None if adam_ms is None else round(adam_ms, 3),
        "wall_s_timed_region": round(wall, 3),
        "kernel_ms_per_step": breakdown,
        "roofline": {"kernel": (GROUPED_KERNEL + " (expert GEMMs over grouped rows, forward + dX)" if sh.n_experts else DOMINANT_KERNEL +
                                                  " (projection GEMMs forward + dX, LoRA term as second K segment)"),
                     "bound": "mfma", "achieved": round(ach, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(ach / PEAK_BF16_TFLOPS, 4),
                     "traffic": None if (sh.n_experts or args.rows or args.row_len or args.single_trajectory or args.nf4 or args.dpo or args.bfd) else
                                (TRAFFIC_BYTES_PER_LAUNCH.get((args.config, DOMINANT_KERNEL)) if kernel_sources_digest() == TRAFFIC_SOURCE_DIGEST else None),
                     "traffic_unit": "HBM-side bytes per launch (counters)",
                     "launches_per_step": n_l // max(args.steps, 1), "avg_launch_ms": round(ms_l / max(n_l, 1), 4)},
    }
    if not args.no_cpu_baseline and not sh.n_experts and not args.dpo:     # the sparse model's float64 weights do not fit the sample budget
        rec["cpu_baseline"] = cpu_baseline(sh, args.seed)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
