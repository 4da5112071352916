"""Pins of the NF4 reference (oracle/nf4.py) against what the public description fixes."""
import numpy as np
from scipy.stats import norm

import synth
from oracle import nf4


def test_levels_are_the_published_quantile_construction():
    """Eight positive and seven negative equally spaced normal quantiles plus an exact zero, normalised
    to [-1, 1] (QLoRA, Section 3): built here from scipy's inverse normal CDF, independent of the table."""
    off = 0.9677083                                       # outermost probability mass of the construction
    pos = norm.ppf(np.linspace(off, 0.5, 9)[:-1])
    neg = -norm.ppf(np.linspace(off, 0.5, 8)[:-1])
    v = np.sort(np.concatenate([pos, [0.0], neg]))
    v = v / v.max()
    assert nf4.LEVELS.shape == (16,) and np.all(np.diff(nf4.LEVELS) > 0)
    assert nf4.LEVELS[0] == -1.0 and nf4.LEVELS[7] == 0.0 and nf4.LEVELS[15] == 1.0
    assert np.abs(v - nf4.LEVELS).max() < 2e-7
    # asymmetric on purpose: 8 positive levels, 7 negative ones
    assert (nf4.LEVELS > 0).sum() == 8 and (nf4.LEVELS < 0).sum() == 7


def test_quantise_is_nearest_level_and_bounded():
    g = synth.rng(0, 30)
    w = (0.02 * g.standard_normal((48, 128))).astype(np.float32)
    codes, absmax = nf4.quantise(w)
    assert codes.dtype == np.uint8 and codes.max() <= 15 and absmax.shape == (48 * 128 // 64,)
    blocks = w.reshape(-1, 64)
    assert np.array_equal(absmax, np.abs(blocks).max(axis=1))
    deq = nf4.dequantise(codes, absmax, w.shape)
    # brute force: no level is closer than the chosen one (in the normalised domain, float64)
    x = blocks.astype(np.float64) / absmax[:, None].astype(np.float64)
    dist = np.abs(x[:, :, None] - nf4.LEVELS[None, None, :])
    chosen = np.take_along_axis(dist, codes.reshape(-1, 64, 1).astype(np.int64), axis=2)[:, :, 0]
    assert np.all(chosen <= dist.min(axis=2) + 1e-6)
    # the element that sets absmax is reproduced exactly; the error is at most half the widest gap
    i = np.abs(blocks).argmax(axis=1)
    assert np.array_equal(deq.reshape(-1, 64)[np.arange(len(i)), i], blocks[np.arange(len(i)), i].astype(np.float64))
    gap = np.diff(nf4.LEVELS).max()
    assert np.abs(deq - w).max() <= 0.5 * gap * absmax.max() * (1 + 1e-6)


def test_requantising_a_dequantised_tensor_changes_nothing_and_edge_blocks():
    g = synth.rng(1, 30)
    w = g.standard_normal(64 * 20).astype(np.float32)
    codes, absmax = nf4.quantise(w)
    deq = nf4.dequantise(codes, absmax)
    codes2, absmax2 = nf4.quantise(deq.astype(np.float32))
    assert np.array_equal(codes, codes2) and np.allclose(absmax, absmax2, rtol=1e-7)
    # all-zero block: absmax 0, zero level, dequantises to zero
    z = np.zeros(64, dtype=np.float32)
    c, a = nf4.quantise(z)
    assert a[0] == 0 and np.all(c == 7) and np.all(nf4.dequantise(c, a) == 0)
    # a value exactly on a midpoint goes to the higher level
    mid = np.float32((np.float32(nf4.LEVELS[7]) + np.float32(nf4.LEVELS[8])) * np.float32(0.5))
    blk = np.zeros(64, dtype=np.float32); blk[0] = 1.0; blk[1] = mid
    c, _ = nf4.quantise(blk)
    assert c[0] == 15 and c[1] == 8 and c[2] == 7


def test_pack_layout_and_roundtrip():
    codes = np.arange(64, dtype=np.uint8) % 16
    p = nf4.pack_codes(codes)
    assert p.shape == (32,) and p[0] == (0 | (1 << 4)) and p[1] == (2 | (3 << 4))
    assert np.array_equal(nf4.unpack_codes(p), codes)
