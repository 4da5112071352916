"""Pins for the float64 reference of the training step.

Nothing here compares the reference with itself through the same formula:
the checks are finite differences, exact invariants, closed forms, and an
independently written PyTorch-float64 model built from library routines
(scaled_dot_product_attention, cross_entropy, autograd).
"""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import model as om
import synth
from helpers import small_shape, random_trajs, packed, grad_norm_err


def setup(sh, seed=0, n_traj=3, row_len=None, gain_jitter=0.1, **kw):
    cfg = oracle.config_from_shape(sh)
    P = synth.weights(sh, seed, std=0.3, gain_jitter=gain_jitter)
    Lo = synth.lora_weights(sh, seed, std=0.3)
    trajs = random_trajs(seed, n_traj, sh.vocab, **kw)
    pk = packed(trajs, row_len or sh.row_len, 1)
    assert pk["n_traj_consumed"] == len(trajs)
    return cfg, P, Lo, trajs, pk


def loss_of(cfg, P, Lo, pk):
    return om.forward(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])["loss"]


# ------------------------------------------------------- finite differences

@pytest.mark.parametrize("variant", ["mha", "gqa7", "moe"])
def test_backward_matches_central_differences(variant):
    if variant == "mha":
        sh = small_shape()
    elif variant == "gqa7":
        sh = small_shape(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=4, d_model=12, ffn=20,
                         lora_targets=synth.DENSE_TARGETS7)
    else:
        sh = small_shape(n_experts=4, top_k=2, ffn=10, lora_targets=("q", "k", "v", "o", "router"))
    cfg, P, Lo, _, pk = setup(sh, seed=1)
    f, g = om.train_step(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    assert f["count"] > 3
    worst = 0.0
    # every LoRA entry
    for l in range(cfg.n_layers):
        for name, (A, B) in Lo[l].items():
            for which, M in (("A", A), ("B", B)):
                G = g["lora"][l][name][0 if which == "A" else 1]
                num = np.zeros_like(M)
                for idx in np.ndindex(M.shape):
                    w0 = M[idx]
                    h = 1e-5 * max(1.0, abs(w0))
                    M[idx] = w0 + h; lp = loss_of(cfg, P, Lo, pk)
                    M[idx] = w0 - h; lm = loss_of(cfg, P, Lo, pk)
                    M[idx] = w0
                    num[idx] = (lp - lm) / (2 * h)
                err = np.max(np.abs(num - G)) / max(np.max(np.abs(G)), 1e-30)
                worst = max(worst, err)
                assert err < 1e-6, (l, name, which, err)
    # a sample of every frozen-weight tensor (what full fine-tuning trains)
    rs = np.random.default_rng(0)
    tensors = [("embed", P["embed"], g["weights"]["embed"]), ("head", P["head"], g["weights"]["head"]),
               ("g_final", P["g_final"], g["weights"]["g_final"])]
    for l in range(cfg.n_layers):
        for k_, M in P["layers"][l].items():
            tensors.append((f"L{l}.{k_}", M, g["weights"]["layers"][l][k_]))
    for name, M, G in tensors:
        assert G.shape == M.shape, name
        n = min(M.size, 40)
        flat = rs.choice(M.size, size=n, replace=False)
        scale = max(np.max(np.abs(G)), 1e-30)
        for fi in flat:
            idx = np.unravel_index(fi, M.shape)
            w0 = M[idx]
            h = 1e-5 * max(1.0, abs(w0))
            M[idx] = w0 + h; lp = loss_of(cfg, P, Lo, pk)
            M[idx] = w0 - h; lm = loss_of(cfg, P, Lo, pk)
            M[idx] = w0
            assert abs((lp - lm) / (2 * h) - G[idx]) / scale < 1e-6, (name, idx)


# ------------------------------------- independent library-built model

def _torch_model_loss(sh, P, Lo, tokens, loss_mask_seg):
    """One trajectory alone, through torch library routines.  RoPE is written
    as a complex multiplication (x_i + i x_{i+d/2}) * exp(i p theta_i)."""
    F = torch.nn.functional
    n = len(tokens)
    d, Hq, Hkv, dh = sh.d_model, sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    s = sh.lora_alpha / sh.lora_rank if sh.lora_rank else 0.0
    half = dh // 2
    theta = torch.tensor([sh.rope_base ** (-2.0 * i / dh) for i in range(half)], dtype=torch.float64)
    ang = torch.arange(n, dtype=torch.float64)[:, None] * theta[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)                      # e^{i p theta}

    def rope(x):                                                      # [n,H,dh]
        z = torch.complex(x[..., :half], x[..., half:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    def lin(x, W, ab):
        y = F.linear(x, W)
        if ab is not None:
            y = y + s * F.linear(F.linear(x, ab[0]), ab[1])
        return y

    def norm(x, g):
        return x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + sh.rms_eps) * g

    h = P["embed"][torch.as_tensor(tokens, dtype=torch.long)]
    for l in range(sh.n_layers):
        W = P["layers"][l]
        Lr = Lo[l] if Lo is not None else {}
        a = norm(h, W["g1"])
        q = rope(lin(a, W["wq"], Lr.get("q")).view(n, Hq, dh))
        k = rope(lin(a, W["wk"], Lr.get("k")).view(n, Hkv, dh))
        v = lin(a, W["wv"], Lr.get("v")).view(n, Hkv, dh)
        k = k.repeat_interleave(Hq // Hkv, dim=1)
        v = v.repeat_interleave(Hq // Hkv, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True)[0]
        o = o.transpose(0, 1).reshape(n, Hq * dh)
        h = h + lin(o, W["wo"], Lr.get("o"))
        b = norm(h, W["g2"])
        m = F.silu(lin(b, W["wgate"], Lr.get("gate"))) * lin(b, W["wup"], Lr.get("up"))
        h = h + lin(m, W["wdown"], Lr.get("down"))
    z = F.linear(norm(h, P["g_final"]), P["head"])
    labels = torch.as_tensor(tokens[1:], dtype=torch.long)
    keep = torch.as_tensor(np.asarray(loss_mask_seg[1:]) == 1)
    if keep.sum() == 0:
        return z.sum() * 0.0, 0
    return F.cross_entropy(z[:-1][keep], labels[keep], reduction="sum"), int(keep.sum())


def _to_torch(P, Lo):
    def t(x):
        return torch.tensor(np.asarray(x), dtype=torch.float64, requires_grad=True)
    Pt = dict(embed=t(P["embed"]), head=t(P["head"]), g_final=t(P["g_final"]),
              layers=[{k: t(v) for k, v in W.items()} for W in P["layers"]])
    Lt = None if Lo is None else [{k: (t(A), t(B)) for k, (A, B) in L.items()} for L in Lo]
    return Pt, Lt


@pytest.mark.parametrize("gqa", [False, True])
def test_against_torch_library_model_with_autograd(gqa):
    sh = small_shape(n_layers=2, n_q_heads=4, n_kv_heads=2 if gqa else 4, head_dim=8, d_model=32, ffn=40,
                     vocab=64, lora_targets=synth.DENSE_TARGETS7, row_len=64)
    cfg, P, Lo, trajs, pk = setup(sh, seed=5, n_traj=4, turn_lo=2, turn_hi=5)
    f, g = om.train_step(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    Pt, Lt = _to_torch(P, Lo)
    cu = pk["cu_seqlens"]
    total, count = 0.0, 0
    for s in range(len(cu) - 1):
        b, e = cu[s], cu[s + 1]
        ls, c = _torch_model_loss(sh, Pt, Lt, pk["tokens"][b:e], pk["loss_mask"][b:e])
        total = total + ls
        count += c
    assert count == f["count"]
    loss = total / count
    loss.backward()
    assert abs(float(loss.detach()) - f["loss"]) < 1e-12 * max(1.0, abs(f["loss"]))
    assert abs(float(total.detach()) - f["loss_sum"]) < 1e-11 * abs(f["loss_sum"])
    assert grad_norm_err(g["weights"]["embed"], Pt["embed"].grad.numpy()) < 1e-10
    assert grad_norm_err(g["weights"]["head"], Pt["head"].grad.numpy()) < 1e-10
    assert grad_norm_err(g["weights"]["g_final"], Pt["g_final"].grad.numpy()) < 1e-10
    for l in range(sh.n_layers):
        for k_, v in Pt["layers"][l].items():
            assert grad_norm_err(g["weights"]["layers"][l][k_], v.grad.numpy()) < 1e-10, (l, k_)
        for k_, (A, B) in Lt[l].items():
            assert grad_norm_err(g["lora"][l][k_][0], A.grad.numpy()) < 1e-10, (l, k_, "A")
            assert grad_norm_err(g["lora"][l][k_][1], B.grad.numpy()) < 1e-10, (l, k_, "B")


# ------------------------------------------------------------------ masking

def test_all_zero_mask_gives_exact_zeros():
    sh = small_shape()
    cfg, P, Lo, _, pk = setup(sh)
    z = np.zeros_like(pk["loss_mask"])
    f, g = om.train_step(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], z)
    assert f["loss"] == 0.0 and f["loss_sum"] == 0.0 and f["count"] == 0
    for l in range(cfg.n_layers):
        for name, (dA, dB) in g["lora"][l].items():
            assert not dA.any() and not dB.any()
        for k_, v in g["weights"]["layers"][l].items():
            assert not v.any()
    assert not g["weights"]["embed"].any() and not g["weights"]["head"].any()
    assert np.all(np.isfinite(f["per_token_loss"]))


def test_mask_bits_of_one_trajectory_touch_only_its_terms():
    sh = small_shape(row_len=80)
    cfg, P, Lo, _, pk = setup(sh, n_traj=3)
    cu = pk["cu_seqlens"]
    f0 = om.forward(cfg, P, Lo, pk["tokens"], cu, pk["loss_mask"])
    m2 = pk["loss_mask"].copy()
    m2[cu[1]:cu[2]] = 0
    f1 = om.forward(cfg, P, Lo, pk["tokens"], cu, m2)
    pt0, pt1 = f0["per_token_loss"], f1["per_token_loss"]
    assert np.array_equal(pt0[:cu[1]], pt1[:cu[1]]) and np.array_equal(pt0[cu[2]:], pt1[cu[2]:])
    assert not pt1[cu[1]:cu[2]].any()
    assert abs((f0["loss_sum"] - f1["loss_sum"]) - pt0[cu[1]:cu[2]].sum()) < 1e-12


def test_first_token_of_a_segment_is_never_a_target():
    sh = small_shape()
    cfg, P, Lo, _, pk = setup(sh)
    ones = np.ones_like(pk["loss_mask"])
    f = om.forward(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], ones)
    N, S = len(pk["tokens"]), len(pk["cu_seqlens"]) - 1
    assert f["count"] == N - S
    last = pk["cu_seqlens"][1:] - 1
    assert not f["per_token_loss"][last].any()


# --------------------------------------------------------------------- LoRA

def test_lora_b_zero_reproduces_base_exactly():
    sh = small_shape(lora_targets=synth.DENSE_TARGETS7)
    cfg, P, Lo, _, pk = setup(sh)
    Lz = [{k: (A, np.zeros_like(B)) for k, (A, B) in L.items()} for L in Lo]
    fb = om.forward(cfg, P, None, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    fz, gz = om.train_step(cfg, P, Lz, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    assert fz["loss"] == fb["loss"]
    assert np.array_equal(fz["cache"]["z"], fb["cache"]["z"])
    for name, (dA, dB) in gz["lora"][0].items():
        assert not dA.any()
        assert dB.any()


def test_lora_merge_identity_and_chain_rule_to_full_finetuning():
    sh = small_shape(n_layers=2, lora_targets=synth.DENSE_TARGETS7)
    cfg, P, Lo, _, pk = setup(sh)
    f, g = om.train_step(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    Pm = om.merge_lora(cfg, P, Lo)
    fm, gm = om.train_step(cfg, Pm, None, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    assert abs(fm["loss"] - f["loss"]) < 1e-12
    s = cfg.lora_scale
    for l in range(cfg.n_layers):
        for name, (A, B) in Lo[l].items():
            dW = gm["weights"]["layers"][l][om._WNAME[name]]
            assert grad_norm_err(g["lora"][l][name][0], s * B.T @ dW) < 1e-10
            assert grad_norm_err(g["lora"][l][name][1], s * dW @ A.T) < 1e-10


# ---------------------------------------------- packing / segments / causality

def test_packed_row_equals_sum_of_single_trajectory_runs():
    sh = small_shape(n_layers=2, row_len=80)
    cfg, P, Lo, trajs, pk = setup(sh, n_traj=3)
    f, g = om.train_step(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    tot, cnt = 0.0, 0
    acc = {k: [np.zeros_like(x) for x in g["lora"][0][k]] for k in g["lora"][0]}
    for tr in trajs:
        p1 = packed([tr], sum(len(t) for _, t in tr), 1)
        f1, g1 = om.train_step(cfg, P, Lo, p1["tokens"], p1["cu_seqlens"], p1["loss_mask"])
        tot += f1["loss_sum"]; cnt += f1["count"]
        for k in acc:
            for i in range(2):
                acc[k][i] += f1["count"] * g1["lora"][0][k][i]
    assert cnt == f["count"] and abs(tot - f["loss_sum"]) < 1e-11
    for k in acc:
        for i in range(2):
            assert grad_norm_err(f["count"] * g["lora"][0][k][i], acc[k][i]) < 1e-11
    # order of trajectories inside the pack does not matter
    p2 = packed(trajs[::-1], 80, 1)
    f2 = om.forward(cfg, P, Lo, p2["tokens"], p2["cu_seqlens"], p2["loss_mask"])
    assert abs(f2["loss_sum"] - f["loss_sum"]) < 1e-11


def test_segments_are_independent_and_attention_is_causal():
    sh = small_shape(row_len=80)
    cfg, P, Lo, trajs, pk = setup(sh, n_traj=3)
    cu = pk["cu_seqlens"]
    ones = np.ones_like(pk["loss_mask"])
    f0 = om.forward(cfg, P, Lo, pk["tokens"], cu, ones)
    u = int(cu[1]) + 3                         # a token inside segment 1
    tok = pk["tokens"].copy()
    tok[u] = (tok[u] + 1) % sh.vocab
    f1 = om.forward(cfg, P, Lo, tok, cu, ones)
    d = f0["per_token_loss"] != f1["per_token_loss"]
    assert not d[:u - 1].any()                 # nothing before position u-1 (whose label changed)
    assert not d[cu[2]:].any()                 # nothing in later segments
    assert d[u - 1] and d[u:cu[2] - 1].any()


# ------------------------------------------------------------ closed forms

def test_zero_head_gives_log_vocab():
    for V in (40, 1024):
        sh = small_shape(vocab=V)
        cfg, P, Lo, _, pk = setup(sh)
        P["head"][:] = 0.0
        f = om.forward(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
        assert abs(f["loss"] - math.log(V)) < 1e-12
    assert abs(math.log(1024) - 6.931471805599453) < 1e-15


def test_dz_rows_sum_to_zero_and_initial_loss_near_log_vocab():
    sh = synth.CONFIGS[1].replace(n_layers=1)
    cfg = oracle.config_from_shape(sh)
    P = synth.weights(sh, 0); Lo = synth.lora_weights(sh, 0)
    pk = packed(synth.workload(1, 0), 512, 1)
    f = om.forward(cfg, P, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    assert abs(f["loss"] - math.log(1024)) < 5e-2
    z, lse, tgt = f["cache"]["z"], f["cache"]["lse"], f["cache"]["tgt"]
    sm = np.exp(z[tgt] - lse[tgt][:, None])
    assert np.max(np.abs(sm.sum(axis=1) - 1.0)) < 1e-12


def test_attention_closed_forms():
    g = synth.rng(0, 9)
    n, Hq, Hkv, dh = 7, 4, 2, 6
    q = g.standard_normal((n + 1, Hq, dh)); k = g.standard_normal((n + 1, Hkv, dh)); v = g.standard_normal((n + 1, Hkv, dh))
    cu = np.array([0, n, n + 1])
    # q = 0: uniform scores -> running mean of v; the length-1 segment returns v
    o, _ = om.attention(np.zeros_like(q), k, v, cu, Hq // Hkv)
    for j in range(Hq):
        pref = np.cumsum(v[:n, j // 2], axis=0) / np.arange(1, n + 1)[:, None]
        assert np.max(np.abs(o[:n, j] - pref)) < 1e-14
        assert np.array_equal(o[n, j], v[n, j // 2])
    # GQA equals MHA on duplicated KV heads
    o1, _ = om.attention(q, k, v, cu, 2)
    o2, _ = om.attention(q, np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1), cu, 1)
    assert np.array_equal(o1, o2)
    # against the brute-force scalar definition on one row
    t, j = 4, 3
    sc = np.array([q[t, j] @ k[u_, 1] / math.sqrt(dh) for u_ in range(t + 1)])
    p = np.exp(sc - sc.max()); p /= p.sum()
    assert np.max(np.abs(o1[t, j] - sum(p[u_] * v[u_, 1] for u_ in range(t + 1)))) < 1e-14


def test_rope_closed_forms():
    g = synth.rng(0, 10)
    n, H, dh = 9, 2, 8
    x = g.standard_normal((n, H, dh)); y = g.standard_normal((n, H, dh))
    pos = np.arange(n)
    c0, s0 = om.rope_table(pos, dh, 100.0)
    c1, s1 = om.rope_table(pos + 17, dh, 100.0)
    # scores depend on position differences only
    a = np.einsum("thd,uhd->htu", om.rope(x, c0, s0), om.rope(y, c0, s0))
    b = np.einsum("thd,uhd->htu", om.rope(x, c1, s1), om.rope(y, c1, s1))
    assert np.max(np.abs(a - b)) < 1e-12
    # infinite base: theta_i = 0 for i > 0; position 0: identity
    assert np.array_equal(om.rope(x, c0, s0)[0], x[0])
    ci, si = om.rope_table(pos, dh, 1e300)
    assert np.max(np.abs(om.rope(x, ci, si)[..., 1:4] - x[..., 1:4])) < 1e-12
    # inverse undoes; explicit 2x2 rotation of pair (i, i+dh/2) at one spot
    assert np.max(np.abs(om.rope(om.rope(x, c0, s0), c0, s0, inverse=True) - x)) < 1e-14
    t, i = 5, 2
    th = t * 100.0 ** (-2.0 * i / dh)
    r = om.rope(x, c0, s0)
    assert abs(r[t, 1, i] - (x[t, 1, i] * math.cos(th) - x[t, 1, i + 4] * math.sin(th))) < 1e-14
    assert abs(r[t, 1, i + 4] - (x[t, 1, i] * math.sin(th) + x[t, 1, i + 4] * math.cos(th))) < 1e-14


def test_rmsnorm_and_silu_closed_forms():
    g = np.array([0.5, 2.0, -1.0, 3.0])
    y, rho = om.rmsnorm(np.full((1, 4), 3.0), g, 1e-5)
    assert np.max(np.abs(y[0] - g * 3.0 / math.sqrt(9.0 + 1e-5))) < 1e-15
    assert om.silu(np.array([0.0]))[0] == 0.0
    h = 1e-6
    assert abs((om.silu(np.array([h]))[0] - om.silu(np.array([-h]))[0]) / (2 * h) - 0.5) < 1e-9


def test_moe_identical_experts_reduce_to_dense_and_router_grads_cancel():
    shd = small_shape(ffn=10, lora_targets=("q", "k", "v", "o"))
    shm = shd.replace(n_experts=4, top_k=2, lora_targets=("q", "k", "v", "o"))
    cfgd, Pd, Lo, _, pk = setup(shd)
    cfgm = oracle.config_from_shape(shm)
    Pm = synth.weights(shm, 3, std=0.3)
    Pm["embed"], Pm["head"], Pm["g_final"] = Pd["embed"], Pd["head"], Pd["g_final"]
    for l in range(shd.n_layers):
        Wd, Wm = Pd["layers"][l], Pm["layers"][l]
        for k_ in ("g1", "wq", "wk", "wv", "wo", "g2"):
            Wm[k_] = Wd[k_]
        for k_ in ("wgate", "wup", "wdown"):
            Wm[k_] = np.repeat(Wd[k_][None], 4, axis=0)
    fd = om.forward(cfgd, Pd, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    fm, gm = om.train_step(cfgm, Pm, Lo, pk["tokens"], pk["cu_seqlens"], pk["loss_mask"])
    assert abs(fd["loss"] - fm["loss"]) < 1e-12
    # with identical experts the loss does not depend on the router at all
    assert np.max(np.abs(gm["weights"]["layers"][0]["wrouter"])) < 1e-12
    # top-k ties go to the lower index
    W = Pm["layers"][0]
    W["wrouter"][:] = 0.0
    _, c = om._ffn_moe(cfgm, np.ones((3, shm.d_model)), W, None, 0.0)
    assert np.array_equal(c["sel"], np.tile([0, 1], (3, 1))) and np.allclose(c["w"], 0.5)
