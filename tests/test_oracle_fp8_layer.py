"""Pins of the oracle's layer with fp8 E4M3 factors and an fp16 Sigma (mixed-precision factor storage, end of
Section 3.1; Appendix A.3 with d_low = 8): explicit dense matrices with the CPU library's fp8 decode, the per-expert
fp16 oracle where fp8 * sigma is exact in fp16, the shared tiled variant against factors copied out per expert, and
planted mistakes."""
import numpy as np
import pytest
import torch

import oracle
from synth import make_layer, make_layer_fp8, make_x, make_logits, Layer, fp8_e4m3_encode
from helpers import tiny_cfg, f16, rel_err, dense_moe


def fp8_lib(a):       # an independent decode: the CPU library's
    return torch.from_numpy(np.ascontiguousarray(a)).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def _route(cfg):
    logits, _ = make_logits(cfg)
    idx, w = oracle.route(logits, None, cfg.k)
    return make_x(cfg), idx, w


def _dense(fl, x, idx, w):
    c = fl.cfg
    x64 = x.astype(np.float64)
    a8, b8 = fl.a8_list(), fl.b8_list()
    y = np.zeros((x.shape[0], c.H))

    def weight(e, p):
        N, K = (c.F, c.H) if p < 2 else (c.H, c.F)
        q = fl.codes[e, p].reshape(N, K).astype(np.float64)
        s = np.repeat(f16(fl.scale[e, p]).reshape(N, K // c.g), c.g, axis=1)
        z = np.repeat(f16(fl.zero[e, p]).reshape(N, K // c.g), c.g, axis=1)
        return ((q - z) * s).T + (fp8_lib(a8[p][e]) * f16(fl.sigma[e, p])) @ fp8_lib(b8[p][e])

    def expert(e):
        G = x64 @ weight(e, 0)
        U = x64 @ weight(e, 1)
        return (G / (1.0 + np.exp(-G)) * U) @ weight(e, 2)

    for e in range(c.E):
        Y = expert(e)
        for j in range(c.k):
            sel = idx[:, j] == e
            y[sel] += w[sel, j][:, None].astype(np.float64) * Y[sel]
    for s_ in range(c.S):
        y += expert(c.E + s_)
    return y


@pytest.mark.parametrize("kw", [dict(E=4, k=2), dict(E=5, S=1, k=3, r=3), dict(E=3, k=1, H=16, F=8, g=8, r=5)])
def test_fp8_layer_vs_dense_matrices(kw):
    cfg = tiny_cfg(cfg_id=160 + kw["E"], **kw)
    fl = make_layer_fp8(cfg)
    x, idx, w = _route(cfg)
    got = oracle.moe_forward_fp8(cfg, fl.codes, fl.scale, fl.zero, fl.a8_list(), fl.b8_list(), fl.sigma, x, idx, w)
    assert rel_err(got, _dense(fl, x, idx, w)) < 1e-12


def test_fp8_layer_equals_the_fp16_layer_where_the_products_are_exact():
    cfg = tiny_cfg(cfg_id=171, E=4, S=1, k=2, r=4)
    fl = make_layer_fp8(cfg, sigma_pow2=True)
    a8, b8 = fl.a8_list(), fl.b8_list()
    # fp8 (3 mantissa bits) times a power of two is an fp16 value exactly; so is fp8 itself
    A16 = np.concatenate([(fp8_lib(a8[p]) * f16(fl.sigma[:, p])[:, None, :]).reshape(cfg.n_exp, -1) for p in range(3)], axis=1)
    B16 = np.concatenate([fp8_lib(b8[p]).reshape(cfg.n_exp, -1) for p in range(3)], axis=1)
    assert np.array_equal(A16.astype(np.float16).astype(np.float64), A16)
    layer = Layer(cfg, fl.codes, fl.scale, fl.zero, A16.astype(np.float16).view(np.uint16), B16.astype(np.float16).view(np.uint16))
    x, idx, w = _route(cfg)
    got = oracle.moe_forward_fp8(cfg, fl.codes, fl.scale, fl.zero, a8, b8, fl.sigma, x, idx, w)
    assert rel_err(got, oracle.moe_forward_layer(layer, x, idx, w)) < 1e-12
    assert rel_err(got, dense_moe(layer, x, idx, w)) < 1e-12


def test_shared_fp8_equals_per_expert_fp8_on_copied_factors():
    cfg = tiny_cfg(cfg_id=172, E=5, S=1, k=2, r=3)
    base = make_layer(cfg)
    rng = np.random.default_rng(172)
    M, N = 2, 3
    dims = ((cfg.H, cfg.F), (cfg.H, cfg.F), (cfg.F, cfg.H))
    us8 = [fp8_e4m3_encode(rng.standard_normal((M, K, cfg.r)).astype(np.float32)) for K, _ in dims]
    v8 = [fp8_e4m3_encode(rng.standard_normal((N, cfg.r, No)).astype(np.float32)) for _, No in dims]
    sigma = (rng.random((3, cfg.r)) * 1e-3 + 1e-4).astype(np.float16).view(np.uint16)
    phi = np.stack([rng.integers(0, M, cfg.n_exp), rng.integers(0, N, cfg.n_exp)], axis=1).astype(np.int32)
    x, idx, w = _route(cfg)
    got = oracle.moe_forward_fp8(cfg, base.codes, base.scale, base.zero, us8, v8, sigma, x, idx, w, phi=phi)
    a8 = [us8[p][phi[:, 0]] for p in range(3)]
    b8 = [v8[p][phi[:, 1]] for p in range(3)]
    sg = np.broadcast_to(sigma[None], (cfg.n_exp, 3, cfg.r)).copy()
    want = oracle.moe_forward_fp8(cfg, base.codes, base.scale, base.zero, a8, b8, sg, x, idx, w)
    assert rel_err(got, want) < 1e-12


def test_planted_sigma_mistakes_are_seen():
    cfg = tiny_cfg(cfg_id=173, E=4, k=2, r=4, f_std=0.3)
    fl = make_layer_fp8(cfg)
    x, idx, w = _route(cfg)
    want = _dense(fl, x, idx, w)
    run = lambda sg: oracle.moe_forward_fp8(cfg, fl.codes, fl.scale, fl.zero, fl.a8_list(), fl.b8_list(), sg, x, idx, w)
    assert rel_err(run(fl.sigma), want) < 1e-12
    assert rel_err(run(np.ascontiguousarray(fl.sigma[:, :, ::-1])), want) > 1e-4            # rank components swapped
    assert rel_err(run(np.ascontiguousarray(fl.sigma[:, ::-1, :])), want) > 1e-4            # gate's Sigma on the down projection
    one = np.full_like(fl.sigma, np.float16(1.0).view(np.uint16))
    assert rel_err(run(one), want) > 1e-2                                                   # Sigma dropped
