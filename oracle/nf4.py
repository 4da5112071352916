"""Reference of the 4-bit NormalFloat (NF4) block quantisation of frozen weights ("Q+LoRA").

TEST INFRASTRUCTURE ONLY (see oracle/model.py).

The paper under study only names the regime (quantised base + LoRA, Section 4.5 and Table 3); the
format is the one of the public QLoRA description (Dettmers et al. 2023, Section 3 and the table of
NF4 values in its appendix): a weight tensor is flattened row-major and cut into blocks of 64
elements; a block stores its absolute maximum (float32 here, no second-level quantisation) and, per
element, the index of the nearest of 16 fixed levels to w / absmax.  The levels are quantiles of
N(0, 1), normalised to [-1, 1], with an exact zero.

Readings fixed here (the sources leave them open): the nearest-level decision is taken in float32
on w / absmax against the 15 midpoints between neighbouring levels, a value exactly on a midpoint
goes to the higher level; an all-zero block has absmax 0 and codes of the zero level; two codes per
byte, element 2j in the low nibble and 2j + 1 in the high nibble; dequantised value =
level * absmax.
"""
import numpy as np

BLOCK = 64

# the 16 levels as printed in the QLoRA appendix (float32 values)
LEVELS = np.array([
    -1.0, -0.6961928009986877, -0.5250730514526367, -0.39491748809814453,
    -0.28444138169288635, -0.18477343022823334, -0.09105003625154495, 0.0,
    0.07958029955625534, 0.16093020141124725, 0.24611230194568634, 0.33791524171829224,
    0.44070982933044434, 0.5626170039176941, 0.7229568362236023, 1.0], dtype=np.float64)


def quantise(w):
    """w: array with a multiple of 64 elements.  Returns (codes uint8 [numel], absmax float32 [numel/64])."""
    flat = np.asarray(w, dtype=np.float32).reshape(-1)
    assert flat.size % BLOCK == 0, "tensor size must be a multiple of the block size"
    blocks = flat.reshape(-1, BLOCK)
    absmax = np.abs(blocks).max(axis=1).astype(np.float32)
    safe = np.where(absmax > 0, absmax, np.float32(1.0)).astype(np.float32)
    x = (blocks / safe[:, None]).astype(np.float32)                    # float32 division, as the device does
    lv = LEVELS.astype(np.float32)
    mid = ((lv[:-1] + lv[1:]) * np.float32(0.5)).astype(np.float32)    # 15 midpoints, float32
    codes = (x[:, :, None] >= mid[None, None, :]).sum(axis=2).astype(np.uint8)
    return codes.reshape(-1), absmax


def dequantise(codes, absmax, shape=None):
    """float64 values level[code] * absmax[block]."""
    codes = np.asarray(codes).reshape(-1, BLOCK)
    out = LEVELS.astype(np.float32).astype(np.float64)[codes] * np.asarray(absmax, dtype=np.float64)[:, None]
    out = out.reshape(-1)
    return out.reshape(shape) if shape is not None else out


def pack_codes(codes):
    """Two 4-bit codes per byte: element 2j in the low nibble, 2j + 1 in the high nibble."""
    c = np.asarray(codes, dtype=np.uint8).reshape(-1, 2)
    return (c[:, 0] | (c[:, 1] << 4)).astype(np.uint8)


def unpack_codes(packed):
    p = np.asarray(packed, dtype=np.uint8).reshape(-1)
    return np.stack([p & 15, p >> 4], axis=1).reshape(-1).astype(np.uint8)
