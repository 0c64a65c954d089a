"""Pins of the oracle's layer on shared 2D-tiled factors (Eq. 4 / the fused form of Section 3.2).

Its low-rank term is written as projection on every row tile, scatter into the [M][r N] accumulator and one
contraction with the stacked right factors.  Pinned against (a) explicit dense matrices W_e = dequant + (U Sigma)_m V_n
formed with numpy (no accumulator, no per-tile projection), (b) the per-expert oracle on factors copied out per
expert, (c) the degenerate tiling in which every expert owns its tile, and (d) planted mistakes: swapped tile
coordinates or a wrong tile must move the result."""
import numpy as np
import pytest

import oracle
from synth import make_layer, make_shared_layer, make_x, make_logits
from helpers import tiny_cfg, f16, rel_err


def _route(cfg, seed=0):
    x = make_x(cfg)
    logits, _ = make_logits(cfg)
    idx, w = oracle.route(logits, None, cfg.k)
    return x, idx, w


def _dense_shared(sl, x, idx, w):
    c = sl.cfg
    x64 = x.astype(np.float64)
    y = np.zeros((x.shape[0], c.H))

    def weight(e, p):
        N, K = (c.F, c.H) if p < 2 else (c.H, c.F)
        q = sl.codes[e, p].reshape(N, K).astype(np.float64)
        s = np.repeat(f16(sl.scale[e, p]).reshape(N, K // c.g), c.g, axis=1)
        z = np.repeat(f16(sl.zero[e, p]).reshape(N, K // c.g), c.g, axis=1)
        m, n = sl.phi[e]
        return ((q - z) * s).T + f16(sl.us[p][m]) @ f16(sl.v[p][n])

    def expert(e):
        G = x64 @ weight(e, 0)
        U = x64 @ weight(e, 1)
        return (G / (1.0 + np.exp(-G)) * U) @ weight(e, 2)

    for e in range(c.E):
        Y = expert(e)
        for j in range(c.k):
            sel = idx[:, j] == e
            y[sel] += w[sel, j][:, None].astype(np.float64) * Y[sel]
    for s in range(c.S):
        y += expert(c.E + s)
    return y


@pytest.mark.parametrize("kw,M,N", [(dict(E=6, S=0, k=2), 2, 3), (dict(E=5, S=1, k=3, r=3), 3, 2),
                                    (dict(E=8, S=2, k=2, H=16, F=8, g=8), 2, 2), (dict(E=4, k=1), 1, 1)])
def test_shared_oracle_vs_dense_matrices(kw, M, N):
    cfg = tiny_cfg(cfg_id=140 + M * 3 + N, **kw)
    sl = make_shared_layer(cfg, M, N)
    x, idx, w = _route(cfg)
    got = oracle.moe_forward_shared(sl, x, idx, w)
    want = _dense_shared(sl, x, idx, w)
    assert rel_err(got, want) < 1e-12


def test_shared_oracle_equals_per_expert_oracle_on_copied_factors():
    cfg = tiny_cfg(cfg_id=151, E=7, S=1, k=3, H=16, F=24, g=8, r=4, T=9)
    sl = make_shared_layer(cfg)      # default near-square grid: 8 experts -> 3 x 3
    assert (sl.M, sl.N) == (3, 3)
    x, idx, w = _route(cfg)
    got = oracle.moe_forward_shared(sl, x, idx, w)
    want = oracle.moe_forward_layer(sl.expanded(), x, idx, w)
    assert rel_err(got, want) < 1e-12


def test_degenerate_tiling_is_the_per_expert_layer():
    cfg = tiny_cfg(cfg_id=152, E=5, S=1, k=2, r=2)
    layer = make_layer(cfg)
    sl = make_shared_layer(cfg, layer=layer, degenerate=True)
    assert sl.M == sl.N == cfg.n_exp and np.array_equal(sl.phi[:, 0], np.arange(cfg.n_exp))
    x, idx, w = _route(cfg)
    assert rel_err(oracle.moe_forward_shared(sl, x, idx, w), oracle.moe_forward_layer(layer, x, idx, w)) < 1e-12


def test_planted_tile_mistakes_are_seen():
    cfg = tiny_cfg(cfg_id=153, E=6, S=0, k=2, r=2)
    sl = make_shared_layer(cfg, 2, 3)
    x, idx, w = _route(cfg)
    want = _dense_shared(sl, x, idx, w)
    import copy
    bad = copy.copy(sl)
    bad.phi = sl.phi.copy()
    e = int(idx[0, 0])
    bad.phi[e, 1] = (bad.phi[e, 1] + 1) % 3          # wrong column tile for one routed expert
    assert rel_err(oracle.moe_forward_shared(bad, x, idx, w), want) > 1e-4
    bad.phi = sl.phi.copy()
    bad.phi[e, 0] = (bad.phi[e, 0] + 1) % 2          # wrong row tile
    assert rel_err(oracle.moe_forward_shared(bad, x, idx, w), want) > 1e-4


def test_tile_index_out_of_range_is_an_error():
    cfg = tiny_cfg(cfg_id=154, E=4, k=2)
    sl = make_shared_layer(cfg, 2, 2)
    sl.phi = sl.phi.copy()
    sl.phi[:, 0] = 2
    x, idx, w = _route(cfg)
    with pytest.raises(ValueError):
        oracle.moe_forward_shared(sl, x, idx, w)
