"""as_pack on the GPU against the reference packer, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import synth
from helpers import random_trajs

pytestmark = pytest.mark.gpu


def _ctx(vocab=1024):
    from paper_2503_22673_amd import binding as B
    return B, B.Context(B.make_config(synth.CONFIGS[1].replace(vocab=vocab)))


def _same(B, ctx, trajs, T, rows, pad_id=0, truncate=True):
    ref = oracle.pack(trajs, T, rows, pad_id=pad_id, truncate=truncate)
    got = ctx.pack(*synth.flatten_trajectories(trajs), T, rows, pad_id=pad_id, truncate=truncate)
    torch.cuda.synchronize()
    assert (got["n_rows"], got["n_segments"], got["n_traj_consumed"]) == (ref["n_rows"], ref["n_segments"], ref["n_traj_consumed"])
    assert np.array_equal(got["tokens"].cpu().numpy(), ref["tokens"])
    assert np.array_equal(got["loss_mask"].cpu().numpy(), ref["loss_mask"])
    assert np.array_equal(got["cu_seqlens"].cpu().numpy(), ref["cu_seqlens"])
    return ref


@pytest.mark.parametrize("seed", range(4))
def test_random_batches(seed):
    B, ctx = _ctx(50)
    _same(B, ctx, random_trajs(seed, 60, 50, turn_lo=0, turn_hi=9), 37, 100, pad_id=49)


def test_edge_cases():
    B, ctx = _ctx(100)
    U, A = 1, 2
    _same(B, ctx, [], 16, 4)                                                   # nothing in
    _same(B, ctx, [[(U, [])], [(A, [5])]], 4, 4, pad_id=9)                     # empty trajectory, ragged tail
    _same(B, ctx, [[(U, list(range(1, 8))), (A, list(range(8, 15)))]], 10, 2)  # truncation cuts a turn
    _same(B, ctx, [[(U, [1] * 3), (A, [2] * 3)] for _ in range(10)], 8, 4)     # max_rows stops early
    _same(B, ctx, [[(U, [1] * 4), (A, [2] * 4)] for _ in range(3)], 8, 8)      # rows exactly full: no pad segment


@pytest.mark.parametrize("cfg_id,rows", [(1, 1), (2, 8), (3, 4), (5, 2)])
def test_benchmark_workloads_full_size(cfg_id, rows):
    sh = synth.CONFIGS[cfg_id]
    B, ctx = _ctx(sh.vocab)
    trajs = synth.workload(cfg_id, seed=0)
    ref = _same(B, ctx, trajs, sh.row_len, rows)
    assert ref["n_rows"] == rows
