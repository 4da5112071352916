"""Shared test helpers: small shapes, packed inputs, error metrics."""
import numpy as np

import oracle
import synth


def small_shape(**kw):
    base = dict(name="t", n_layers=1, d_model=16, n_q_heads=2, n_kv_heads=2, head_dim=8, ffn=24,
                vocab=40, rms_eps=1e-5, rope_base=100.0, lora_rank=2, lora_alpha=4.0,
                lora_targets=("q", "k", "v", "o"), rows=1, row_len=80, bf16=False)
    base.update(kw)
    return synth.Shape(**base)


def random_trajs(seed, n_traj, vocab, turn_lo=2, turn_hi=5, turns=(2, 5)):
    g = synth.rng(seed, 7)
    out = []
    for _ in range(n_traj):
        roles = synth.role_pattern(int(g.integers(turns[0], turns[1] + 1)))
        out.append([(r, g.integers(0, vocab, size=int(g.integers(turn_lo, turn_hi + 1))).astype(np.int32))
                    for r in roles])
    return out


def packed(trajs, row_len, max_rows, pad_id=0):
    return oracle.pack(trajs, row_len, max_rows, pad_id=pad_id)


def grad_norm_err(got, ref):
    """max |got - ref| / max |ref| (the normalised max error of one tensor)."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def rel_err(got, ref):
    return abs(float(got) - float(ref)) / max(abs(float(ref)), 1e-30)
