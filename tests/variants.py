"""Input transformations that give the parity tests the power to see single terms of the projection.

Input manufacture only (no forward arithmetic): each function returns a copy of a synth.Layer whose canonical
arrays were edited; the same arrays then feed the oracle and the GPU.

  pure_lowrank   codes := zero-point of their group (an integer in [0, qmax] from the RTN quantiser), so the
                 dequantised matrix is exactly 0 and the output is the rank-r chain alone.  Used on amplified
                 factors: the bf16 kernels evaluate the quantised term as s * sum x (128 + q) - s (128 + z) * sum x,
                 whose two halves cancel here only up to the rounding of the second (about 2^-17 of s (128 + z) sum x
                 per group, a few 1e-5 in absolute terms), and the un-amplified rank-r output of a small layer
                 (a few 1e-3) would be compared against that noise instead of against the kernels' low-rank steps
  amplified      A and B times 8 (exact on fp16 bit patterns): the rank-r term grows 64x, to the size of the
                 quantised term and beyond
  odd_quant      fractional zero-points, zero-points below 0 and above qmax, subnormal and large fp16 scales
"""
import dataclasses

import numpy as np


def pure_lowrank(layer):
    c = layer.cfg
    codes = np.empty_like(layer.codes)
    for e in range(c.E + c.S):
        for p in range(3):
            z = layer.zero_matrix(e, p).astype(np.float32)
            assert np.all(z == np.rint(z)) and z.min() >= 0 and z.max() <= c.qmax
            codes[e, p] = np.repeat(z.astype(np.uint8), c.g, axis=1).reshape(-1)
    return dataclasses.replace(layer, codes=codes)


def _times_pow2(bits: np.ndarray, mult: float) -> np.ndarray:
    v = bits.view(np.float16).astype(np.float32) * np.float32(mult)
    out = v.astype(np.float16)
    assert np.all(np.isfinite(out)) and np.array_equal(out.astype(np.float32), v)      # exact
    return out.view(np.uint16)


def amplified(layer, mult: float = 8.0):
    assert layer.cfg.r > 0
    return dataclasses.replace(layer, A=_times_pow2(layer.A, mult), B=_times_pow2(layer.B, mult))


def odd_quant(layer, seed: int):
    c = layer.cfg
    rng = np.random.default_rng(seed)
    z = layer.zero.view(np.float16).astype(np.float32)
    z = z + rng.uniform(-0.5, 0.5, z.shape).astype(np.float32)
    pick = rng.random(z.shape)
    z[pick < 0.03] = -3.25
    z[pick > 0.97] = c.qmax + 5.5
    s = layer.scale.view(np.float16).astype(np.float32)
    pick = rng.random(s.shape)
    s = np.where(pick < 0.03, s * np.float32(2.0 ** -10), s)      # fp16 subnormals (below 6.1e-5)
    s = np.where(pick > 0.97, s * np.float32(16.0), s)
    s16 = s.astype(np.float16)
    assert np.any((s16 != 0) & (np.abs(s16.astype(np.float32)) < 6.1e-5))
    return dataclasses.replace(layer, zero=z.astype(np.float16).view(np.uint16), scale=s16.view(np.uint16))


def zero_factor(layer, p: int):
    """A copy whose A factor of projection p (0 gate, 1 up, 2 down) is zero: a planted mistake for the oracle side."""
    c = layer.cfg
    A = layer.A.copy()
    K = c.H if p < 2 else c.F
    o = layer.a_offset(p)
    A[:, o:o + K * c.r] = 0
    return dataclasses.replace(layer, A=A)


def segment_edge_tokens(idx: np.ndarray, E: int, extra_rows=(63, 64)):
    """Tokens that own the first and the last row of every expert's segment of the stable expert-sorted order (and
    the rows at the given offsets from each segment start, e.g. the last row of the first 64-row tile and the first
    row of the second), computed with a plain stable argsort.  Experts without rows contribute nothing; the row after
    an empty expert is the first row of the next expert that has rows, which is included."""
    T, k = idx.shape
    flat = idx.reshape(-1)
    order = np.argsort(flat, kind="stable")
    counts = np.bincount(flat, minlength=E)
    starts = np.concatenate([[0], np.cumsum(counts)])
    rows = []
    for e in range(E):
        if counts[e] == 0:
            continue
        rows += [starts[e], starts[e + 1] - 1]
        rows += [starts[e] + o for o in extra_rows if o < counts[e]]
    return np.unique(order[np.array(rows, dtype=np.int64)] // k).astype(np.int32)
