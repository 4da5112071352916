"""Float64 reference of one loss-masked causal-LM fine-tuning step.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this
module; only the tests, the smoke check and the CPU-baseline leg of the
benchmark do.

The paper (Sections 3.2.1, 3.2.2 and 4.1/4.5) names the computation without
printing formulas: supervised fine-tuning of decoder-only Llama / Mistral /
Mixtral models on multi-turn agent trajectories, with a per-element loss
mask, under LoRA (Section 4.5: q/k/v/o adapters, rank and alpha given) or
full fine-tuning.  This file writes that computation out from the standard
definitions of its parts, everything materialised (full score matrices per
segment and head, full logits), float64 throughout, with a backward pass
derived by hand (no automatic differentiation):

  h0_t   = E[token_t]
  layer: a = RMSNorm(h; g1);  q,k,v = lin(a);  RoPE on q,k with positions
         that restart at every segment;  causal softmax attention inside a
         segment only, query head j reading KV head j // (Hq/Hkv);
         h += lin_o(attn);  b = RMSNorm(h; g2);
         h += lin_down(silu(lin_gate(b)) * lin_up(b))          (dense)
         h += sum_{e in top2} w_e FFN_e(b)                     (MoE)
  lin_X(x) = W_X x + (alpha/r) B_X (A_X x)   when X carries an adapter
  loss   = mean over targets t (positions whose NEXT token lies in the same
           segment and has loss_mask 1) of  logsumexp(z_t) - z_t[token_{t+1}]

numpy's matmul, exp, sqrt are the only library primitives; there is no
blocking, fusion or reordering.
"""
from dataclasses import dataclass, field
import numpy as np

LORA_TARGETS = ("q", "k", "v", "o", "gate", "up", "down", "router")
_WNAME = {"q": "wq", "k": "wk", "v": "wv", "o": "wo", "gate": "wgate",
          "up": "wup", "down": "wdown", "router": "wrouter"}


@dataclass
class Config:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    lora_rank: int = 0
    lora_alpha: float = 0.0
    lora_targets: tuple = ()
    n_experts: int = 0
    top_k: int = 0

    @property
    def lora_scale(self):
        return self.lora_alpha / self.lora_rank if self.lora_rank else 0.0


# ----------------------------------------------------------------- pieces

def segment_ids(cu_seqlens, n):
    seg = np.zeros(n, dtype=np.int64)
    for s in range(len(cu_seqlens) - 1):
        seg[cu_seqlens[s]:cu_seqlens[s + 1]] = s
    return seg


def rmsnorm(x, g, eps):
    rho = 1.0 / np.sqrt(np.mean(x * x, axis=-1) + eps)
    return x * rho[:, None] * g[None, :], rho


def rmsnorm_bwd(dy, x, g, rho):
    d = x.shape[-1]
    gdy = dy * g[None, :]
    dot = np.sum(gdy * x, axis=-1)
    dx = rho[:, None] * gdy - x * (rho ** 3 / d * dot)[:, None]
    dg = np.sum(dy * x * rho[:, None], axis=0)
    return dx, dg


def rope_table(pos, head_dim, base):
    half = head_dim // 2
    theta = base ** (-2.0 * np.arange(half, dtype=np.float64) / head_dim)
    ang = pos.astype(np.float64)[:, None] * theta[None, :]
    return np.cos(ang), np.sin(ang)


def rope(x, cos, sin, inverse=False):
    """x [n, H, d_h]; component i is paired with i + d_h/2."""
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    if inverse:
        s = -s
    return np.concatenate([x1 * c - x2 * s, x1 * s + x2 * c], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def linear(x, W, ab, scale):
    """y = W x (+ scale * B (A x)); returns (y, u = A x or None)."""
    y = x @ W.T
    if ab is None:
        return y, None
    A, B = ab
    u = x @ A.T
    return y + scale * (u @ B.T), u


def linear_bwd(dy, x, W, ab, scale, u):
    """Returns dx, dW, (dA, dB) or None."""
    dx = dy @ W
    dW = dy.T @ x
    if ab is None:
        return dx, dW, None
    A, B = ab
    du = scale * (dy @ B)
    dB = scale * (dy.T @ u)
    dA = du.T @ x
    dx = dx + du @ A
    return dx, dW, (dA, dB)


def attention(q, k, v, cu_seqlens, group):
    """q [N,Hq,dh], k,v [N,Hkv,dh] (already rotated).  Returns o and the
    probability matrices per (segment, query head)."""
    N, Hq, dh = q.shape
    o = np.zeros_like(q)
    probs = {}
    inv = 1.0 / np.sqrt(dh)
    for s in range(len(cu_seqlens) - 1):
        b, e = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        n = e - b
        future = np.triu(np.ones((n, n), dtype=bool), k=1)
        for j in range(Hq):
            g = j // group
            S = (q[b:e, j] @ k[b:e, g].T) * inv
            S[future] = -np.inf
            S = S - S.max(axis=1, keepdims=True)
            P = np.exp(S)
            P = P / P.sum(axis=1, keepdims=True)
            probs[(s, j)] = P
            o[b:e, j] = P @ v[b:e, g]
    return o, probs


def attention_bwd(do, q, k, v, o, probs, cu_seqlens, group):
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    N, Hq, dh = q.shape
    inv = 1.0 / np.sqrt(dh)
    for s in range(len(cu_seqlens) - 1):
        b, e = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        for j in range(Hq):
            g = j // group
            P = probs[(s, j)]
            dv[b:e, g] += P.T @ do[b:e, j]
            dP = do[b:e, j] @ v[b:e, g].T
            delta = np.sum(do[b:e, j] * o[b:e, j], axis=1, keepdims=True)
            dS = P * (dP - delta)
            dq[b:e, j] = (dS @ k[b:e, g]) * inv
            dk[b:e, g] += (dS.T @ q[b:e, j]) * inv
    return dq, dk, dv


def targets(tokens, cu_seqlens, loss_mask):
    """Positions t whose next token is a loss-bearing token of the same
    segment, and the labels token[t+1]."""
    N = len(tokens)
    seg = segment_ids(cu_seqlens, N)
    idx = [t for t in range(N - 1)
           if seg[t + 1] == seg[t] and loss_mask[t + 1] == 1]
    idx = np.asarray(idx, dtype=np.int64)
    return idx, np.asarray(tokens, dtype=np.int64)[idx + 1]


# ------------------------------------------------------------------ model

def _ab(lora_layer, name):
    if lora_layer is None:
        return None
    return lora_layer.get(name)


def _ffn_dense(cfg, b, W, Lr, sc):
    gate, u_g = linear(b, W["wgate"], _ab(Lr, "gate"), sc)
    up, u_u = linear(b, W["wup"], _ab(Lr, "up"), sc)
    m = silu(gate) * up
    y, u_d = linear(m, W["wdown"], _ab(Lr, "down"), sc)
    return y, dict(gate=gate, up=up, m=m, u_gate=u_g, u_up=u_u, u_down=u_d)


def _ffn_dense_bwd(cfg, dy, b, W, Lr, sc, c):
    dm, dWd, lo_d = linear_bwd(dy, c["m"], W["wdown"], _ab(Lr, "down"), sc, c["u_down"])
    g, u = c["gate"], c["up"]
    sig = 1.0 / (1.0 + np.exp(-g))
    dgate = dm * u * sig * (1.0 + g * (1.0 - sig))
    dup = dm * g * sig
    db1, dWg, lo_g = linear_bwd(dgate, b, W["wgate"], _ab(Lr, "gate"), sc, c["u_gate"])
    db2, dWu, lo_u = linear_bwd(dup, b, W["wup"], _ab(Lr, "up"), sc, c["u_up"])
    return db1 + db2, dict(wdown=dWd, wgate=dWg, wup=dWu), dict(down=lo_d, gate=lo_g, up=lo_u)


def _ffn_moe(cfg, b, W, Lr, sc):
    """Mixtral-style router: the k largest router logits (ties to the lower
    index), softmax over the selected ones, weighted sum of expert FFNs."""
    N = b.shape[0]
    logit, u_r = linear(b, W["wrouter"], _ab(Lr, "router"), sc)
    sel = np.argsort(-logit, axis=1, kind="stable")[:, :cfg.top_k]      # [N,k]
    lsel = np.take_along_axis(logit, sel, axis=1)
    ex = np.exp(lsel - lsel.max(axis=1, keepdims=True))
    w = ex / ex.sum(axis=1, keepdims=True)                              # [N,k]
    y = np.zeros_like(b)
    per = []
    for e in range(cfg.n_experts):
        rows, slot = np.nonzero(sel == e)
        xe = b[rows]
        gate = xe @ W["wgate"][e].T
        up = xe @ W["wup"][e].T
        m = silu(gate) * up
        ye = m @ W["wdown"][e].T
        y[rows] += w[rows, slot][:, None] * ye
        per.append(dict(rows=rows, slot=slot, gate=gate, up=up, m=m, y=ye))
    return y, dict(logit=logit, u_router=u_r, sel=sel, w=w, per=per)


def _ffn_moe_bwd(cfg, dy, b, W, Lr, sc, c):
    N = b.shape[0]
    sel, w = c["sel"], c["w"]
    db = np.zeros_like(b)
    dw = np.zeros_like(w)
    dWg = np.zeros_like(W["wgate"]); dWu = np.zeros_like(W["wup"]); dWd = np.zeros_like(W["wdown"])
    for e in range(cfg.n_experts):
        p = c["per"][e]
        rows, slot = p["rows"], p["slot"]
        dye = dy[rows]
        dw[rows, slot] = np.sum(dye * p["y"], axis=1)
        dout = dye * w[rows, slot][:, None]
        dm = dout @ W["wdown"][e]
        dWd[e] = dout.T @ p["m"]
        g, u = p["gate"], p["up"]
        sig = 1.0 / (1.0 + np.exp(-g))
        dgate = dm * u * sig * (1.0 + g * (1.0 - sig))
        dup = dm * g * sig
        dWg[e] = dgate.T @ b[rows]
        dWu[e] = dup.T @ b[rows]
        db[rows] += dgate @ W["wgate"][e] + dup @ W["wup"][e]
    # softmax over the selected logits only; nothing flows through the choice
    dl_sel = w * (dw - np.sum(w * dw, axis=1, keepdims=True))
    dlogit = np.zeros_like(c["logit"])
    np.put_along_axis(dlogit, sel, dl_sel, axis=1)
    dbr, dWr, lo_r = linear_bwd(dlogit, b, W["wrouter"], _ab(Lr, "router"), sc, c["u_router"])
    return db + dbr, dict(wdown=dWd, wgate=dWg, wup=dWu, wrouter=dWr), dict(router=lo_r)


def forward(cfg, params, lora, tokens, cu_seqlens, loss_mask):
    """Returns dict(loss, loss_sum, count, per_token_loss [N], cache)."""
    tokens = np.asarray(tokens, dtype=np.int64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    N = len(tokens)
    assert cu[0] == 0 and cu[-1] == N and np.all(np.diff(cu) > 0)
    seg = segment_ids(cu, N)
    pos = np.arange(N) - cu[seg]
    cos, sin = rope_table(pos, cfg.head_dim, cfg.rope_base)
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    group = Hq // Hkv
    sc = cfg.lora_scale
    h = np.asarray(params["embed"], dtype=np.float64)[tokens]
    layers = []
    for l in range(cfg.n_layers):
        W = params["layers"][l]
        Lr = lora[l] if lora is not None else None
        c = dict(h_in=h)
        a, c["rho1"] = rmsnorm(h, W["g1"], cfg.rms_eps)
        q, c["u_q"] = linear(a, W["wq"], _ab(Lr, "q"), sc)
        k, c["u_k"] = linear(a, W["wk"], _ab(Lr, "k"), sc)
        v, c["u_v"] = linear(a, W["wv"], _ab(Lr, "v"), sc)
        qr = rope(q.reshape(N, Hq, dh), cos, sin)
        kr = rope(k.reshape(N, Hkv, dh), cos, sin)
        vh = v.reshape(N, Hkv, dh)
        o, probs = attention(qr, kr, vh, cu, group)
        y, c["u_o"] = linear(o.reshape(N, Hq * dh), W["wo"], _ab(Lr, "o"), sc)
        h_mid = h + y
        b, c["rho2"] = rmsnorm(h_mid, W["g2"], cfg.rms_eps)
        if cfg.n_experts:
            y2, c["ffn"] = _ffn_moe(cfg, b, W, Lr, sc)
        else:
            y2, c["ffn"] = _ffn_dense(cfg, b, W, Lr, sc)
        h = h_mid + y2
        c.update(a=a, q=qr, k=kr, v=vh, o=o, probs=probs, h_mid=h_mid, b=b, h_out=h)
        layers.append(c)
    hf, rho_f = rmsnorm(h, params["g_final"], cfg.rms_eps)
    z = hf @ np.asarray(params["head"], dtype=np.float64).T              # [N,V]
    tgt, labels = targets(tokens, cu, loss_mask)
    zmax = z.max(axis=1)
    lse = zmax + np.log(np.sum(np.exp(z - zmax[:, None]), axis=1))
    per_token = np.zeros(N)
    per_token[tgt] = lse[tgt] - z[tgt, labels]
    count = len(tgt)
    loss_sum = float(np.sum(per_token[tgt]))
    loss = loss_sum / count if count else 0.0
    cache = dict(layers=layers, h_final=h, hf=hf, rho_f=rho_f, z=z, lse=lse,
                 tgt=tgt, labels=labels, cos=cos, sin=sin, cu=cu, tokens=tokens)
    return dict(loss=loss, loss_sum=loss_sum, count=count,
                per_token_loss=per_token, cache=cache)


def backward(cfg, params, lora, fwd, target_weights=None):
    """Gradients of the masked-mean loss.  Returns dict(weights=..., lora=...)
    where ``weights`` mirrors ``params`` (always filled: the frozen-weight
    gradients are what full fine-tuning uses) and ``lora`` mirrors ``lora``
    with (dA, dB) pairs.

    ``target_weights`` (one value per target, in target order) replaces the
    1/count of the mean: the result is then the gradient of
    sum_i target_weights[i] * per_token_loss[target i], which is what a loss
    built on per-sequence log-probabilities needs (oracle/dpo.py)."""
    ca = fwd["cache"]
    N = len(ca["tokens"])
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    group = Hq // Hkv
    sc = cfg.lora_scale
    C = fwd["count"]
    head = np.asarray(params["head"], dtype=np.float64)
    dz = np.zeros_like(ca["z"])
    if C:
        tgt, labels = ca["tgt"], ca["labels"]
        sm = np.exp(ca["z"][tgt] - ca["lse"][tgt][:, None])
        sm[np.arange(len(tgt)), labels] -= 1.0
        dz[tgt] = sm / C if target_weights is None else sm * np.asarray(target_weights, dtype=np.float64)[:, None]
    g_head = dz.T @ ca["hf"]
    dhf = dz @ head
    dres, g_gfinal = rmsnorm_bwd(dhf, ca["h_final"], params["g_final"], ca["rho_f"])
    gW_layers, gL_layers = [None] * cfg.n_layers, [None] * cfg.n_layers
    for l in reversed(range(cfg.n_layers)):
        W = params["layers"][l]
        Lr = lora[l] if lora is not None else None
        c = ca["layers"][l]
        gW, gL = {}, {}
        if cfg.n_experts:
            db, gw, gl = _ffn_moe_bwd(cfg, dres, c["b"], W, Lr, sc, c["ffn"])
        else:
            db, gw, gl = _ffn_dense_bwd(cfg, dres, c["b"], W, Lr, sc, c["ffn"])
        gW.update(gw); gL.update(gl)
        dx, gW["g2"] = rmsnorm_bwd(db, c["h_mid"], W["g2"], c["rho2"])
        dh_mid = dres + dx
        do, gW["wo"], gL["o"] = linear_bwd(dh_mid, c["o"].reshape(N, Hq * dh), W["wo"],
                                           _ab(Lr, "o"), sc, c["u_o"])
        dq, dk, dv = attention_bwd(do.reshape(N, Hq, dh), c["q"], c["k"], c["v"], c["o"],
                                   c["probs"], ca["cu"], group)
        dq = rope(dq, ca["cos"], ca["sin"], inverse=True).reshape(N, Hq * dh)
        dk = rope(dk, ca["cos"], ca["sin"], inverse=True).reshape(N, Hkv * dh)
        dv = dv.reshape(N, Hkv * dh)
        da1, gW["wq"], gL["q"] = linear_bwd(dq, c["a"], W["wq"], _ab(Lr, "q"), sc, c["u_q"])
        da2, gW["wk"], gL["k"] = linear_bwd(dk, c["a"], W["wk"], _ab(Lr, "k"), sc, c["u_k"])
        da3, gW["wv"], gL["v"] = linear_bwd(dv, c["a"], W["wv"], _ab(Lr, "v"), sc, c["u_v"])
        dx, gW["g1"] = rmsnorm_bwd(da1 + da2 + da3, c["h_in"], W["g1"], c["rho1"])
        dres = dh_mid + dx
        gW_layers[l] = gW
        gL_layers[l] = {k_: v_ for k_, v_ in gL.items() if v_ is not None}
    g_embed = np.zeros_like(np.asarray(params["embed"], dtype=np.float64))
    np.add.at(g_embed, ca["tokens"], dres)
    return dict(weights=dict(embed=g_embed, head=g_head, g_final=g_gfinal, layers=gW_layers),
                lora=gL_layers if lora is not None else None,
                dh0=dres)


def train_step(cfg, params, lora, tokens, cu_seqlens, loss_mask):
    f = forward(cfg, params, lora, tokens, cu_seqlens, loss_mask)
    g = backward(cfg, params, lora, f)
    return f, g


def merge_lora(cfg, params, lora):
    """W' = W + (alpha/r) B A for every adapted projection."""
    out = dict(embed=params["embed"], head=params["head"], g_final=params["g_final"], layers=[])
    for l, W in enumerate(params["layers"]):
        W2 = dict(W)
        for name, (A, B) in lora[l].items():
            W2[_WNAME[name]] = W[_WNAME[name]] + cfg.lora_scale * (B @ A)
        out["layers"].append(W2)
    return out


def config_from_shape(sh):
    """Build a Config from any object carrying the same attribute names."""
    return Config(**{f: getattr(sh, f) for f in Config.__dataclass_fields__})
