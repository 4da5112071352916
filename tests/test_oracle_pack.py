"""Pins for the reference packer: hand-worked example, invariants, edge cases."""
import os

import numpy as np
import pytest

import oracle
import synth
from helpers import random_trajs

A, U, S, T_ = oracle.ROLE_ASSISTANT, oracle.ROLE_USER, oracle.ROLE_SYSTEM, oracle.ROLE_TOOL
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _parse_golden(path):
    """tiny text format: key: space-separated ints"""
    out = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        k, v = line.split(":")
        out[k.strip()] = [int(x) for x in v.split()]
    return out


def test_hand_worked_example():
    """tests/golden/pack_example.txt was written by hand from the packing
    policy (next-fit, tail pad, assistant-only mask); it is not produced by
    any code."""
    gold = _parse_golden(os.path.join(GOLD, "pack_example.txt"))
    trajs = [
        [(S, [11, 12]), (U, [13]), (A, [14, 15])],          # length 5
        [(U, [21]), (A, [22, 23])],                          # length 3  -> row 0 full (8)
        [(U, [31, 32]), (A, [33]), (T_, [34]), (A, [35])],   # length 5  -> row 1
        [(U, [41, 42, 43]), (A, [44, 45])],                  # length 5: does not fit (5+5>8) -> row 2
    ]
    r = oracle.pack(trajs, row_len=8, max_rows=3, pad_id=99)
    assert r["tokens"].tolist() == gold["tokens"]
    assert r["loss_mask"].tolist() == gold["loss_mask"]
    assert r["cu_seqlens"].tolist() == gold["cu_seqlens"]
    assert [r["n_rows"], r["n_segments"], r["n_traj_consumed"]] == gold["rows_segments_consumed"]


@pytest.mark.parametrize("seed", range(6))
def test_invariants_random(seed):
    T, PAD = 50, 49
    trajs = random_trajs(seed, 25, vocab=49, turn_lo=0, turn_hi=9)   # longest possible: 5 turns x 9 < T
    r = oracle.pack(trajs, T, max_rows=100, pad_id=PAD)
    cu, tok, m = r["cu_seqlens"], r["tokens"], r["loss_mask"]
    N = r["n_rows"] * T
    assert tok.shape == (N,) and m.shape == (N,)
    assert cu[0] == 0 and cu[-1] == N and np.all(np.diff(cu) > 0)
    for k in range(r["n_rows"] + 1):
        assert k * T in cu
    assert r["n_traj_consumed"] == len(trajs)
    assert int(m.sum()) == sum(len(t) for tr in trajs for ro, t in tr if ro == A)
    # non-pad tokens, in order, are exactly the input stream
    flat = [int(x) for tr in trajs for _, t in tr for x in t]
    assert tok[tok != PAD].tolist() == flat
    flat_mask = [1 if ro == A else 0 for tr in trajs for ro, t in tr for _ in t]
    assert m[tok != PAD].tolist() == flat_mask
    assert np.all(m[tok == PAD] == 0)
    # next-fit: a row was closed only because the next trajectory did not fit
    lens = [sum(len(t) for _, t in tr) for tr in trajs]
    lens = [x for x in lens if x > 0]
    fill, rows = 0, 0
    for L in lens:
        if fill + L > T:
            rows, fill = rows + 1, 0
        fill += L
        if fill == T:
            rows, fill = rows + 1, 0
    assert r["n_rows"] == rows + (1 if fill else 0)


def test_no_segment_straddles_a_row():
    trajs = random_trajs(3, 40, vocab=30, turn_lo=1, turn_hi=6)
    T = 29
    r = oracle.pack(trajs, T, max_rows=1000)
    cu = r["cu_seqlens"]
    for s in range(len(cu) - 1):
        assert cu[s] // T == (cu[s + 1] - 1) // T


def test_max_rows_stops_and_reports():
    trajs = [[(U, [1] * 3), (A, [2] * 3)] for _ in range(10)]     # length 6 each, T=8 -> one per row
    r = oracle.pack(trajs, 8, max_rows=4)
    assert r["n_rows"] == 4 and r["n_traj_consumed"] == 4
    assert r["tokens"].shape == (32,)
    assert r["cu_seqlens"].tolist() == [0, 6, 8, 14, 16, 22, 24, 30, 32]


def test_truncate_and_too_long():
    trajs = [[(U, list(range(1, 8))), (A, list(range(8, 15)))]]   # length 14
    r = oracle.pack(trajs, 10, 2, truncate=True)
    assert r["tokens"].tolist() == list(range(1, 11))
    assert r["loss_mask"].tolist() == [0] * 7 + [1] * 3
    assert r["cu_seqlens"].tolist() == [0, 10]
    with pytest.raises(oracle.PackError):
        oracle.pack(trajs, 10, 2, truncate=False)


def test_empty_inputs():
    r = oracle.pack([], 16, 4)
    assert r["n_rows"] == 0 and r["cu_seqlens"].tolist() == [0] and r["tokens"].size == 0
    r = oracle.pack([[(U, [])], [(A, [5])]], 4, 4, pad_id=9)
    assert r["n_traj_consumed"] == 2 and r["tokens"].tolist() == [5, 9, 9, 9]
    assert r["cu_seqlens"].tolist() == [0, 1, 4] and r["loss_mask"].tolist() == [1, 0, 0, 0]


def test_bad_role_and_token():
    with pytest.raises(oracle.PackError):
        oracle.pack([[(7, [1])]], 4, 1)
    with pytest.raises(oracle.PackError):
        oracle.pack([[(U, [100])]], 4, 1, vocab=100)
    with pytest.raises(oracle.PackError):
        oracle.pack([[(U, [-1])]], 4, 1)


def test_synthetic_recipes_have_the_stated_structure():
    tr = synth.workload(1, seed=0)
    r = oracle.pack(tr, 512, 1)
    assert r["n_rows"] == 1 and r["n_traj_consumed"] == 4 and r["n_segments"] == 5
    frac = r["loss_mask"].mean()
    assert 0.15 < frac < 0.5
    tr = synth.workload(2, seed=0, rows=2)
    r = oracle.pack(tr, 4096, 2)
    assert r["n_rows"] == 2 and r["n_traj_consumed"] == len(tr)
    nonpad = sum(sum(len(t) for _, t in x) for x in tr)
    assert 0.15 < r["loss_mask"].sum() / nonpad < 0.35
    assert r["tokens"].max() < 32000
