"""Seeded synthetic inputs shared by the reference and the GPU path.

Holds no arithmetic of the training step: only shapes, random draws
(numpy's counter-based Philox generator) and the recipes that stand in for
the paper's actionstudio-98k trajectories (Section 3.1: multi-turn, about
nine steps on average, roles system / user / assistant / tool) and for the
model families of Section 4.1.
"""
from dataclasses import dataclass, field
import numpy as np

ROLE_SYSTEM, ROLE_USER, ROLE_ASSISTANT, ROLE_TOOL = 0, 1, 2, 3
DENSE_TARGETS7 = ("q", "k", "v", "o", "gate", "up", "down")


@dataclass
class Shape:
    """Model shape + workload of one benchmark configuration."""
    name: str
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
    rows: int = 1
    row_len: int = 512
    full_ft: bool = False
    recompute: int = 0
    bf16: bool = True

    def replace(self, **kw):
        d = dict(self.__dict__)
        d.update(kw)
        return Shape(**d)


CONFIGS = {
    1: Shape("tiny-fp32", 2, 128, 4, 4, 32, 344, 1024, 1e-5, 1e4, 8, 16.0, ("q", "k", "v", "o"),
             rows=1, row_len=512, bf16=False),
    2: Shape("llama-1b-lora", 16, 2048, 32, 8, 64, 8192, 32000, 1e-5, 1e4, 16, 32.0, DENSE_TARGETS7,
             rows=8, row_len=4096),
    3: Shape("llama3-8b-lora", 32, 4096, 32, 8, 128, 14336, 128256, 1e-5, 5e5, 64, 128.0, DENSE_TARGETS7,
             rows=4, row_len=16384, recompute=2),
    4: Shape("llama-1b-fullft", 16, 2048, 32, 8, 64, 8192, 32000, 1e-5, 1e4, 0, 0.0, (),
             rows=16, row_len=4096, full_ft=True),
    5: Shape("mixtral-8x7b-lora", 32, 4096, 32, 8, 128, 14336, 32000, 1e-5, 1e6, 16, 32.0,
             ("q", "k", "v", "o", "router"), n_experts=8, top_k=2, rows=2, row_len=8192),
}


def rng(seed, stream=0):
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


# ------------------------------------------------------------ trajectories

def role_pattern(n_turns):
    """system, then (user, assistant, tool, assistant) repeating; a two-turn
    trajectory is (user, assistant); a single turn is an assistant turn."""
    if n_turns == 1:
        return [ROLE_ASSISTANT]
    if n_turns == 2:
        return [ROLE_USER, ROLE_ASSISTANT]
    cyc = [ROLE_USER, ROLE_ASSISTANT, ROLE_TOOL, ROLE_ASSISTANT]
    return [ROLE_SYSTEM] + [cyc[i % 4] for i in range(n_turns - 1)]


def zipf_cdf(vocab, exponent=1.1):
    p = np.arange(1, vocab + 1, dtype=np.float64) ** (-exponent)
    c = np.cumsum(p)
    return c / c[-1]


def draw_tokens(g, n, vocab, dist, cdf=None):
    if dist == "uniform":
        return g.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)
    u = g.random(n)
    return np.minimum(np.searchsorted(cdf, u, side="left"), vocab - 1).astype(np.int32)


def split_length(g, total, roles, assistant_share):
    """Split ``total`` tokens over the turns so that assistant turns hold
    about ``assistant_share`` of them; every turn gets at least one token."""
    n = len(roles)
    k_a = sum(1 for r in roles if r == ROLE_ASSISTANT)
    w = np.ones(n)
    if 0 < k_a < n:
        wa = assistant_share * (n - k_a) / (k_a * (1.0 - assistant_share))
        w = np.array([wa if r == ROLE_ASSISTANT else 1.0 for r in roles])
    w = w * g.uniform(0.5, 1.5, size=n)
    total = max(total, n)
    raw = w / w.sum() * (total - n)
    lens = np.floor(raw).astype(np.int64) + 1
    rem = total - int(lens.sum())
    order = np.argsort(-(raw - np.floor(raw)), kind="stable")
    for i in range(rem):
        lens[order[i % n]] += 1
    return lens


def trajectories_lognormal(seed, rows, row_len, vocab, median, sigma, lo, hi,
                           turns=(2, 12), assistant_share=0.25, token_dist="zipf"):
    """Draw trajectories until ``rows`` rows of a next-fit packer would be
    closed (configs 2-4 style).  Returns a list of trajectories, each a list
    of (role, int32 token array)."""
    g = rng(seed, 1)
    cdf = zipf_cdf(vocab) if token_dist == "zipf" else None
    out, fill, closed = [], 0, 0
    while closed < rows:
        L = int(np.clip(np.round(np.exp(np.log(median) + sigma * g.standard_normal())), lo, hi))
        L = min(L, row_len)
        n_turns = int(g.integers(turns[0], turns[1] + 1))
        n_turns = min(n_turns, L)
        roles = role_pattern(n_turns)
        lens = split_length(g, L, roles, assistant_share)
        if fill + L > row_len:
            closed += 1
            fill = 0
            if closed >= rows:
                break
        traj = [(r, draw_tokens(g, int(n), vocab, token_dist, cdf)) for r, n in zip(roles, lens)]
        out.append(traj)
        fill += L
        if fill == row_len:
            closed += 1
            fill = 0
    return out


def trajectories_uniform(seed, rows, row_len, vocab, lo, hi, turns=(2, 6),
                         assistant_share=0.25, token_dist="zipf"):
    """Many short trajectories with lengths uniform in [lo, hi] (config 5)."""
    g = rng(seed, 1)
    cdf = zipf_cdf(vocab) if token_dist == "zipf" else None
    out, fill, closed = [], 0, 0
    while closed < rows:
        L = int(g.integers(lo, hi + 1))
        L = min(L, row_len)
        roles = role_pattern(int(g.integers(turns[0], turns[1] + 1)))
        lens = split_length(g, L, roles, assistant_share)
        if fill + L > row_len:
            closed += 1
            fill = 0
            if closed >= rows:
                break
        out.append([(r, draw_tokens(g, int(n), vocab, token_dist, cdf)) for r, n in zip(roles, lens)])
        fill += L
        if fill == row_len:
            closed += 1
            fill = 0
    return out


def trajectories_tiny(seed, n_traj=4, row_len=512, vocab=1024, turn_lo=16, turn_hi=64):
    """Config 1: ``n_traj`` trajectories of 3-5 turns, turn lengths uniform in
    [turn_lo, turn_hi], redrawn until all of them fit one row with a pad tail."""
    g = rng(seed, 1)
    while True:
        spec = []
        for _ in range(n_traj):
            n_turns = int(g.integers(3, 6))
            spec.append([int(g.integers(turn_lo, turn_hi + 1)) for _ in range(n_turns)])
        if sum(sum(s) for s in spec) <= row_len - 8:
            break
    out = []
    for lens in spec:
        roles = role_pattern(len(lens))
        out.append([(r, draw_tokens(g, n, vocab, "uniform")) for r, n in zip(roles, lens)])
    return out


def workload(cfg_id, seed=0, rows=None, row_len=None):
    """Trajectories for one of the five benchmark configurations."""
    sh = CONFIGS[cfg_id]
    rows = sh.rows if rows is None else rows
    row_len = sh.row_len if row_len is None else row_len
    if cfg_id == 1:
        return trajectories_tiny(seed, 4, row_len, sh.vocab)
    if cfg_id in (2, 4):
        return trajectories_lognormal(seed, rows, row_len, sh.vocab, 1200, 0.6, 128, 4096,
                                      assistant_share=0.25)
    if cfg_id == 3:
        return trajectories_lognormal(seed, rows, row_len, sh.vocab, 2000, 0.6, 256, 16384,
                                      assistant_share=0.20)
    if cfg_id == 5:
        return trajectories_uniform(seed, rows, row_len, sh.vocab, 64, 1024, assistant_share=0.25)
    raise KeyError(cfg_id)


def flatten_trajectories(trajs):
    """CSR form used by the C interface: turn_tokens, turn_offsets,
    turn_roles, traj_offsets (offsets count turns)."""
    toks, toff, roles, joff = [], [0], [], [0]
    for tr in trajs:
        for r, t in tr:
            toks.append(np.asarray(t, dtype=np.int32))
            toff.append(toff[-1] + len(t))
            roles.append(r)
        joff.append(len(roles))
    flat = np.concatenate(toks) if toks else np.zeros(0, dtype=np.int32)
    return (flat.astype(np.int32), np.asarray(toff, dtype=np.int32),
            np.asarray(roles, dtype=np.uint8), np.asarray(joff, dtype=np.int32))


# ------------------------------------------------------------------ weights

def normal_f32_blocks(seed, stream, shape, std, block=1 << 24):
    """N(0, std) float32 array whose blocks of ``block`` elements come from Philox streams of their own
    (key = seed, stream, block index), filled by a thread pool: billions of weights in seconds."""
    from concurrent.futures import ThreadPoolExecutor
    import os
    out = np.empty(int(np.prod(shape)), dtype=np.float32)

    def fill(i):
        g = np.random.Generator(np.random.Philox(key=[int(seed), (int(stream) << 20) + i]))
        v = out[i * block:(i + 1) * block]
        g.standard_normal(out=v, dtype=np.float32)
        v *= np.float32(std)

    n_blocks = (out.size + block - 1) // block
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        list(ex.map(fill, range(n_blocks)))
    return out.reshape(shape)


def lora_dims(sh):
    D = sh.n_q_heads * sh.head_dim
    Dkv = sh.n_kv_heads * sh.head_dim
    return {"q": (sh.d_model, D), "k": (sh.d_model, Dkv), "v": (sh.d_model, Dkv),
            "o": (D, sh.d_model), "gate": (sh.d_model, sh.ffn), "up": (sh.d_model, sh.ffn),
            "down": (sh.ffn, sh.d_model), "router": (sh.d_model, max(sh.n_experts, 1))}


def weights(sh, seed=0, std=0.02, dtype=np.float64, gain_jitter=0.0):
    """N(0, std) matrices [out, in]; gains 1 (+ optional jitter so that tests
    can tell a dropped gain from a kept one)."""
    g = rng(seed, 2)
    D = sh.n_q_heads * sh.head_dim
    Dkv = sh.n_kv_heads * sh.head_dim
    d, F = sh.d_model, sh.ffn

    n_big = [0]

    def mat(*shape):
        if dtype == np.float32:            # true-width models: single precision, drawn in parallel blocks
            n_big[0] += 1
            return normal_f32_blocks(seed, 1000 + n_big[0], shape, std)
        return (std * g.standard_normal(shape)).astype(dtype)

    def gain():
        return (1.0 + gain_jitter * g.standard_normal(d)).astype(dtype)

    P = dict(embed=mat(sh.vocab, d), head=mat(sh.vocab, d), g_final=gain(), layers=[])
    for _ in range(sh.n_layers):
        W = dict(g1=gain(), wq=mat(D, d), wk=mat(Dkv, d), wv=mat(Dkv, d), wo=mat(d, D), g2=gain())
        if sh.n_experts:
            W.update(wgate=mat(sh.n_experts, F, d), wup=mat(sh.n_experts, F, d),
                     wdown=mat(sh.n_experts, d, F), wrouter=mat(sh.n_experts, d))
        else:
            W.update(wgate=mat(F, d), wup=mat(F, d), wdown=mat(d, F))
        P["layers"].append(W)
    return P


def lora_weights(sh, seed=0, std=0.02, dtype=np.float64, zero_b=False):
    """Per layer: name -> (A [r, d_in], B [d_out, r]); both N(0, std) so that
    every gradient is non-zero (B = 0 on request)."""
    if not sh.lora_rank:
        return None
    g = rng(seed, 3)
    dims = lora_dims(sh)
    out = []
    for _ in range(sh.n_layers):
        L = {}
        for name in sh.lora_targets:
            din, dout = dims[name]
            A = (std * g.standard_normal((sh.lora_rank, din))).astype(dtype)
            B = (std * g.standard_normal((dout, sh.lora_rank))).astype(dtype)
            if zero_b:
                B = np.zeros_like(B)
            L[name] = (A, B)
        out.append(L)
    return out
