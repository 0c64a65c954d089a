"""Pins for the CPU oracle: every function is checked against something other than itself —
library routines (numpy float16, stable argsort, matmul), brute force on tiny inputs, closed forms
and invariants.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
from synth import make_layer, make_x, make_logits, rtn_quantize, bf16_round
from helpers import (tiny_cfg, dense_weight, dense_expert_all_tokens, exhaustive_topk, dense_moe, rel_err)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ fp16 decode
def test_half_to_double_exhaustive_against_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite], ref[finite])
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isinf(got), np.isinf(ref))
    assert np.array_equal(np.signbit(got[finite]), np.signbit(ref[finite]))


# ------------------------------------------------------------------ routing
@pytest.mark.parametrize("T,E,k", [(7, 4, 2), (16, 8, 2), (9, 6, 6), (5, 5, 1), (33, 60, 4), (12, 128, 8)])
def test_route_matches_exhaustive_sort(T, E, k):
    rng = np.random.default_rng(100 + T + E + k)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    bias = (rng.standard_normal(E) * 0.5).astype(np.float32) if E % 2 == 0 else None
    idx, w = oracle.route(logits, bias, k)
    ridx, rw = exhaustive_topk(logits, bias, k)
    assert np.array_equal(idx, ridx)
    # softmax over the selected == softmax over all renormalised over the selected
    assert np.max(np.abs(w.astype(np.float64) - rw)) < 1e-7
    assert np.max(np.abs(w.astype(np.float64).sum(axis=1) - 1.0)) < 1e-6
    assert np.all(w > 0)


def test_route_special_cases():
    rng = np.random.default_rng(5)
    logits = rng.standard_normal((11, 7)).astype(np.float32)
    # k = 1: argmax, weight exactly 1
    idx, w = oracle.route(logits, None, 1)
    assert np.array_equal(idx[:, 0], np.argmax(logits, axis=1))
    assert np.all(w == np.float32(1.0))
    # k = E: a permutation of all experts in descending score, weights = full softmax
    idx, w = oracle.route(logits, None, 7)
    assert np.array_equal(np.sort(idx, axis=1), np.tile(np.arange(7), (11, 1)))
    srt = np.take_along_axis(logits, idx, axis=1)
    assert np.all(np.diff(srt, axis=1) <= 0)
    p = np.exp(logits.astype(np.float64) - logits.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    assert np.max(np.abs(np.take_along_axis(p, idx, axis=1) - w)) < 1e-7
    # all logits equal: lowest indices win, weights 1/k
    eq = np.full((3, 9), 0.25, dtype=np.float32)
    idx, w = oracle.route(eq, None, 4)
    assert np.array_equal(idx, np.tile(np.arange(4), (3, 1)))
    assert np.allclose(w, 0.25, atol=0, rtol=1e-7)
    # ties inside the top-k and at its edge resolve to the lower index
    tie = np.array([[1.0, 3.0, 3.0, 0.0, 3.0, 1.0]], dtype=np.float32)
    idx, _ = oracle.route(tie, None, 4)
    assert idx.tolist() == [[1, 2, 4, 0]]
    # the bias decides the selection (and is added in fp32)
    b = np.array([0, 0, 0, 10, 0, 0], dtype=np.float32)
    idx, _ = oracle.route(tie, b, 1)
    assert idx.tolist() == [[3]]


def test_route_selection_uses_fp32_sum_of_logit_and_bias():
    # 1 + 2^-24 is not representable in fp32: after the fp32 add both scores are equal -> index tie-break.
    logits = np.array([[1.0, 1.0]], dtype=np.float32)
    bias = np.array([0.0, 2.0 ** -25], dtype=np.float32)
    idx, w = oracle.route(logits, bias, 1)
    assert idx.tolist() == [[0]]


# ------------------------------------------------------------------ permutation
@pytest.mark.parametrize("T,E,k,seed", [(1, 4, 2, 0), (16, 8, 2, 1), (257, 60, 4, 2), (1000, 128, 8, 3)])
def test_permute_is_stable_counting_sort(T, E, k, seed):
    rng = np.random.default_rng(seed)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    offsets, slot_of, src_of = oracle.permute(idx, E)
    flat = idx.reshape(-1)
    counts = np.bincount(flat, minlength=E)
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    order = np.argsort(flat, kind="stable")          # slot -> assignment
    assert np.array_equal(src_of, order)
    inv = np.empty_like(order)
    inv[order] = np.arange(order.size)
    assert np.array_equal(slot_of, inv)
    for e in range(E):
        seg = src_of[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)


def test_permute_empty_experts():
    idx = np.array([[2, 5], [5, 2], [2, 5]], dtype=np.int32)
    offsets, slot_of, src_of = oracle.permute(idx, 8)
    assert offsets.tolist() == [0, 0, 0, 3, 3, 3, 6, 6, 6]
    assert src_of.tolist() == [0, 3, 4, 1, 2, 5]


# ------------------------------------------------------------------ dequantisation
def test_dequant_exhaustive_codes():
    # every code x a spread of (scale, zero), including fractional zeros; reference is python float math
    scales = np.array([0.001, 0.0123, 1.0, 0.5, 3.25], dtype=np.float16)
    zeros = np.array([0.0, 7.0, 8.0, 15.0, 3.5], dtype=np.float16)
    g = 16
    rows = []
    for s in scales:
        for z in zeros:
            rows.append((s, z))
    N = len(rows)
    codes = np.tile(np.arange(16, dtype=np.uint8), (N, 1))
    s_bits = np.array([r[0] for r in rows], dtype=np.float16).view(np.uint16).reshape(N, 1)
    z_bits = np.array([r[1] for r in rows], dtype=np.float16).view(np.uint16).reshape(N, 1)
    W = oracle.dequant(codes, s_bits, z_bits, g)
    for n, (s, z) in enumerate(rows):
        for q in range(16):
            assert W[n, q] == (float(q) - float(z)) * float(s)
    # integer zero: the product is exactly representable in fp32
    Wi = W[[i for i, r in enumerate(rows) if float(r[1]).is_integer()]]
    assert np.array_equal(Wi.astype(np.float32).astype(np.float64), Wi)


def test_dequant_group_indexing():
    # distinct scale and zero per (row, group): a transposed or mis-strided lookup cannot pass
    N, K, g = 3, 12, 4
    codes = (np.arange(N * K).reshape(N, K) % 16).astype(np.uint8)
    s = (np.arange(1, N * 3 + 1).reshape(N, 3)).astype(np.float16)
    z = (np.arange(N * 3).reshape(N, 3) % 5).astype(np.float16)
    W = oracle.dequant(codes, s.view(np.uint16), z.view(np.uint16), g)
    for n in range(N):
        for kk in range(K):
            assert W[n, kk] == (float(codes[n, kk]) - float(z[n, kk // g])) * float(s[n, kk // g])


def test_rtn_grid_roundtrip_through_oracle_dequant():
    # weights placed exactly on a quantisation grid survive quantise -> dequantise
    rng = np.random.default_rng(3)
    N, K, g, qmax = 6, 32, 8, 15
    s = rng.choice([0.25, 0.5, 0.125], size=(N, K // g)).astype(np.float32)
    z = rng.integers(3, 12, size=(N, K // g)).astype(np.float32)
    q = rng.integers(0, 16, size=(N, K))
    # make every group span the full code range so RTN recovers scale and zero
    q.reshape(N, K // g, g)[:, :, 0] = 0
    q.reshape(N, K // g, g)[:, :, 1] = 15
    w = ((q - np.repeat(z, g, 1)) * np.repeat(s, g, 1)).astype(np.float32)
    codes, sc, ze = rtn_quantize(w, g, qmax)
    assert np.array_equal(codes, q)
    W = oracle.dequant(codes, sc.view(np.uint16), ze.view(np.uint16), g)
    assert np.array_equal(W, w.astype(np.float64))


# ------------------------------------------------------------------ projection
@pytest.mark.parametrize("r", [0, 1, 3])
def test_project_equals_dense_effective_weight(r):
    cfg = tiny_cfg(cfg_id=110 + r, H=24, F=40, g=8, r=r, E=2)
    layer = make_layer(cfg, workers=1)
    rng = np.random.default_rng(9)
    for p in range(3):
        N, K = layer.shapes(p)
        v = rng.standard_normal(K)
        A = layer.a_matrix(0, p).view(np.uint16) if r else None
        B = layer.b_matrix(0, p).view(np.uint16) if r else None
        got = oracle.project(v, layer.codes_matrix(0, p), layer.scale[0, p], layer.zero[0, p], A, B, cfg.g)
        ref = v @ dense_weight(layer, 0, p)
        assert got.shape == (N,)
        assert rel_err(got, ref) < 1e-12


def test_project_pure_lowrank_chain_and_pure_quantised():
    rng = np.random.default_rng(11)
    N, K, g, r = 10, 16, 4, 3
    z = rng.integers(0, 16, size=(N, K // g)).astype(np.float16)
    codes = np.repeat(z.astype(np.uint8), g, axis=1)             # q == zero everywhere -> W_deq = 0
    s = rng.uniform(0.01, 0.1, size=(N, K // g)).astype(np.float16)
    A = rng.standard_normal((K, r)).astype(np.float16)
    B = rng.standard_normal((r, N)).astype(np.float16)
    v = rng.standard_normal(K)
    got = oracle.project(v, codes, s.view(np.uint16), z.view(np.uint16), A.view(np.uint16), B.view(np.uint16), g)
    ref = (v @ A.astype(np.float64)) @ B.astype(np.float64)
    assert rel_err(got, ref) < 1e-12
    # r = 0: only the quantised term
    codes2 = rng.integers(0, 16, size=(N, K)).astype(np.uint8)
    got = oracle.project(v, codes2, s.view(np.uint16), z.view(np.uint16), None, None, g)
    Wd = oracle.dequant(codes2, s.view(np.uint16), z.view(np.uint16), g)
    assert rel_err(got, Wd @ v) < 1e-12


def test_silu_values():
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(1.0) - 0.7310585786300049) < 1e-15
    assert abs(oracle.silu(-1.0) + 0.2689414213699951) < 1e-15
    assert abs(oracle.silu(30.0) - 30.0) < 1e-11
    with open(os.path.join(GOLDEN, "silu.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            a, b = line.split()
            assert abs(oracle.silu(float(a)) - float(b)) < 1e-12


# ------------------------------------------------------------------ whole layer
@pytest.mark.parametrize("kw", [dict(), dict(S=1, cfg_id=102), dict(E=6, k=3, T=9, r=0, cfg_id=103),
                                dict(E=5, k=1, H=12, F=20, g=4, r=3, T=4, bits=3, cfg_id=104),
                                dict(E=3, S=2, k=2, H=16, F=8, g=8, r=1, T=6, cfg_id=105)])
def test_layer_matches_dense_brute_force(kw):
    cfg = tiny_cfg(**kw)
    layer = make_layer(cfg, workers=1)
    x = make_x(cfg)
    logits, _ = make_logits(cfg)
    bias = (np.arange(cfg.E, dtype=np.float32) * 0.1) if cfg.cfg_id % 2 else None
    idx, w = oracle.route(logits, bias, cfg.k)
    ridx, rw = exhaustive_topk(logits, bias, cfg.k)
    assert np.array_equal(idx, ridx)
    y = oracle.moe_forward_layer(layer, x, idx, w)
    ref = dense_moe(layer, x, idx, w)
    assert rel_err(y, ref) < 1e-12
    assert layer.codes.max() <= cfg.qmax


def test_layer_grid_weights_reproduce_unquantised_moe():
    """rank 0 and weights exactly on the quantisation grid: the layer equals a plain fp64 SwiGLU MoE
    evaluated on the unquantised weight matrices with library matmuls."""
    cfg = tiny_cfg(cfg_id=120, E=4, k=2, H=16, F=24, T=7, g=8, r=0)
    rng = np.random.default_rng(21)
    ne = cfg.E
    Wg = np.zeros((ne, cfg.F, cfg.H), np.float32)
    Wu = np.zeros_like(Wg)
    Wd = np.zeros((ne, cfg.H, cfg.F), np.float32)
    codes = np.zeros((ne, 3, cfg.H * cfg.F), np.uint8)
    scale = np.zeros((ne, 3, cfg.H * cfg.F // cfg.g), np.uint16)
    zero = np.zeros_like(scale)
    for e in range(ne):
        for p, Wm in enumerate((Wg, Wu, Wd)):
            N, K = Wm.shape[1:]
            s = rng.choice([2.0 ** -6, 2.0 ** -5, 2.0 ** -7], size=(N, K // cfg.g)).astype(np.float32)
            z = rng.integers(5, 11, size=(N, K // cfg.g)).astype(np.float32)
            q = rng.integers(0, 16, size=(N, K))
            q.reshape(N, K // cfg.g, cfg.g)[:, :, 0] = 0
            q.reshape(N, K // cfg.g, cfg.g)[:, :, 1] = 15
            Wm[e] = (q - np.repeat(z, cfg.g, 1)) * np.repeat(s, cfg.g, 1)
            c, sc, ze = rtn_quantize(Wm[e], cfg.g, 15)
            codes[e, p] = c.reshape(-1)
            scale[e, p] = sc.view(np.uint16).reshape(-1)
            zero[e, p] = ze.view(np.uint16).reshape(-1)
    x = make_x(cfg)
    logits, _ = make_logits(cfg)
    idx, w = oracle.route(logits, None, cfg.k)
    y = oracle.moe_forward(cfg.E, 0, cfg.k, cfg.H, cfg.F, cfg.g, 4, 0, codes, scale, zero, None, None, x, idx, w)
    x64 = x.astype(np.float64)
    ref = np.zeros((cfg.T, cfg.H))
    for t in range(cfg.T):
        for j in range(cfg.k):
            e = idx[t, j]
            G = Wg[e].astype(np.float64) @ x64[t]
            U = Wu[e].astype(np.float64) @ x64[t]
            h = G / (1 + np.exp(-G)) * U
            ref[t] += float(w[t, j]) * (Wd[e].astype(np.float64) @ h)
    assert rel_err(y, ref) < 1e-12


def test_layer_invariants():
    cfg = tiny_cfg(cfg_id=130, E=6, k=3, H=16, F=24, T=8, g=8, r=2, S=1)
    layer = make_layer(cfg, workers=1)
    x = make_x(cfg)
    logits, _ = make_logits(cfg)
    idx, w = oracle.route(logits, None, cfg.k)
    y = oracle.moe_forward_layer(layer, x, idx, w)

    # (iii) token permutation equivariance, bitwise
    perm = np.random.default_rng(1).permutation(cfg.T)
    yp = oracle.moe_forward_layer(layer, x[perm], idx[perm], w[perm])
    assert np.array_equal(yp, y[perm])
    # token subset selection returns the same rows
    tok = np.array([5, 0, 3], dtype=np.int32)
    assert np.array_equal(oracle.moe_forward_layer(layer, x, idx, w, tokens=tok), y[tok])

    # (iv) expert relabelling: permute routed experts and logit columns together
    ep = np.random.default_rng(2).permutation(cfg.E)          # new expert n holds old expert ep[n]
    full = np.concatenate([ep, np.arange(cfg.E, cfg.n_exp)])
    import copy
    l2 = copy.copy(layer)
    l2.codes, l2.scale, l2.zero, l2.A, l2.B = (layer.codes[full], layer.scale[full], layer.zero[full],
                                               layer.A[full], layer.B[full])
    idx2, w2 = oracle.route(logits[:, ep], None, cfg.k)
    # same scores; ties are measure-zero for random logits, so the selected sets map onto each other
    assert np.array_equal(ep[idx2], idx)
    y2 = oracle.moe_forward_layer(l2, x, idx2, w2)
    assert rel_err(y2, y) < 1e-13

    # (vi) one-hot routing weight -> a single expert MLP
    w1 = np.zeros_like(w)
    w1[:, 1] = 1.0
    y1 = oracle.moe_forward_layer(layer, x, idx, w1)
    x64 = x.astype(np.float64)
    for t in range(cfg.T):
        ref = dense_expert_all_tokens(layer, idx[t, 1], x64[t:t + 1])[0] \
            + dense_expert_all_tokens(layer, cfg.E, x64[t:t + 1])[0]
        assert rel_err(y1[t], ref) < 1e-12

    # linearity in the routing weights: doubling w doubles the routed part
    cfg0 = cfg.replace(S=0)
    l0 = copy.copy(layer)
    l0.cfg = cfg0
    l0.codes, l0.scale, l0.zero, l0.A, l0.B = (layer.codes[:cfg.E], layer.scale[:cfg.E], layer.zero[:cfg.E],
                                               layer.A[:cfg.E], layer.B[:cfg.E])
    ya = oracle.moe_forward_layer(l0, x, idx, w)
    yb = oracle.moe_forward_layer(l0, x, idx, (2 * w).astype(np.float32))
    assert rel_err(yb, 2 * ya) < 1e-14
    # shared expert contributes with weight exactly 1 regardless of routing
    ysh = dense_expert_all_tokens(layer, cfg.E, x64)
    assert rel_err(y - ya, ysh) < 1e-11


def test_layer_k_equals_E_is_dense_softmax_mixture():
    cfg = tiny_cfg(cfg_id=140, E=4, k=4, H=8, F=16, T=6, g=4, r=2)
    layer = make_layer(cfg, workers=1)
    x = make_x(cfg)
    logits, _ = make_logits(cfg)
    idx, w = oracle.route(logits, None, cfg.k)
    y = oracle.moe_forward_layer(layer, x, idx, w)
    p = np.exp(logits.astype(np.float64) - logits.max(axis=1, keepdims=True).astype(np.float64))
    p /= p.sum(axis=1, keepdims=True)
    ref = np.zeros_like(y)
    for e in range(cfg.E):
        ref += p[:, e:e + 1] * dense_expert_all_tokens(layer, e, x.astype(np.float64))
    assert rel_err(y, ref) < 1e-7      # routing weights were rounded to fp32


def test_layer_rejects_bad_expert_index():
    cfg = tiny_cfg(cfg_id=150)
    layer = make_layer(cfg, workers=1)
    x = make_x(cfg)
    idx = np.full((cfg.T, cfg.k), cfg.E, dtype=np.int32)
    w = np.full((cfg.T, cfg.k), 0.5, dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.moe_forward_layer(layer, x, idx, w)


def test_benchmark_config_1_against_dense():
    """The tiny benchmark layer (8 experts, top-2, 256/512, 64 tokens) end to end on a token sample."""
    from synth import CONFIGS
    cfg = CONFIGS[1]
    layer = make_layer(cfg, workers=4)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    idx, w = oracle.route(logits, bias, cfg.k)
    tok = np.array([0, 17, 63], dtype=np.int32)
    y = oracle.moe_forward_layer(layer, x, idx, w, tokens=tok)
    ref = dense_moe(layer, x[tok], idx[tok], w[tok])
    assert rel_err(y, ref) < 1e-12


# ------------------------------------------------------------------ LoTileMoE (Section 3.2)
def _lotile_case(seed, T=7, E=6, k=3, n_in=20, n_out=12, r=5, M=2, N=3, distinct=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, n_in)).astype(np.float32)
    us = (rng.standard_normal((M, n_in, r)) * 0.3).astype(np.float16)
    v = (rng.standard_normal((N, r, n_out)) * 0.3).astype(np.float16)
    tiles = rng.permutation(M * N)[:E]
    phi = np.stack([tiles // N, tiles % N], axis=1).astype(np.int32)
    if distinct:
        idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    else:
        idx = rng.integers(0, E, size=(T, k)).astype(np.int32)
    w = rng.random((T, k)).astype(np.float32)
    return x, us, v, phi, idx, w


@pytest.mark.parametrize("seed,M,N,E", [(0, 2, 3, 6), (1, 3, 3, 7), (2, 1, 5, 5), (3, 4, 1, 4), (4, 3, 4, 12)])
def test_lotile_equals_per_expert_definition(seed, M, N, E):
    """Eq. 4 + Eq. 3: y_b = sum_t g_bt * x_b (U_m Sigma) V_n with (m, n) = phi(e_bt), one expert at a time."""
    x, us, v, phi, idx, w = _lotile_case(seed, E=E, M=M, N=N, k=min(3, E))
    got = oracle.lotile_forward(x, us.view(np.uint16), v.view(np.uint16), phi, idx, w)
    usd, vd, xd = us.astype(np.float64), v.astype(np.float64), x.astype(np.float64)
    ref = np.zeros_like(got)
    for b in range(x.shape[0]):
        for t in range(idx.shape[1]):
            m, n = phi[idx[b, t]]
            ref[b] += float(w[b, t]) * (xd[b] @ usd[m]) @ vd[n]
    assert np.max(np.abs(got - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_lotile_repeated_selection_adds():
    """A token that lists the same expert twice: Eq. 3 sums over the selections, so the accumulator adds (the
    assignment arrow in the construction of Eq. 15 is read as accumulation)."""
    x, us, v, phi, idx, w = _lotile_case(21, T=6, E=3, k=4, M=2, N=2, distinct=False)
    got = oracle.lotile_forward(x, us.view(np.uint16), v.view(np.uint16), phi, idx, w)
    ref = np.zeros_like(got)
    for b in range(x.shape[0]):
        for t in range(idx.shape[1]):
            m, n = phi[idx[b, t]]
            ref[b] += float(w[b, t]) * (x[b].astype(np.float64) @ us[m].astype(np.float64)) @ v[n].astype(np.float64)
    assert np.max(np.abs(got - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_lotile_equals_compact_buffer_form():
    """Eq. 16: S[b]^(n) = sum_{t: n_bt = n} g_bt X_proj[b]^(m_bt); Y = S V_flat - two dense products and a scatter."""
    x, us, v, phi, idx, w = _lotile_case(11, T=9, E=9, k=4, M=3, N=3, r=4)
    got = oracle.lotile_forward(x, us.view(np.uint16), v.view(np.uint16), phi, idx, w)
    M, n_in, r = us.shape
    N, _, n_out = v.shape
    us_reshape = us.astype(np.float64).transpose(1, 0, 2).reshape(n_in, M * r)      # [in, M r]
    v_flat = v.astype(np.float64).reshape(N * r, n_out)                               # [N r, out]
    xproj = x.astype(np.float64) @ us_reshape
    S = np.zeros((x.shape[0], N * r))
    for b in range(x.shape[0]):
        for t in range(idx.shape[1]):
            m, n = phi[idx[b, t]]
            S[b, n * r:(n + 1) * r] += float(w[b, t]) * xproj[b, m * r:(m + 1) * r]
    ref = S @ v_flat
    assert np.max(np.abs(got - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_lotile_one_tile_per_expert_is_the_per_expert_lowrank_projection():
    """M = N = E with phi(e) = (e, e) has no sharing: each term is the pinned per-expert low-rank chain
    (oracle.project with a zero quantised part)."""
    E, n_in, n_out, r, g = 4, 32, 8, 3, 16
    x, us, v, _, idx, w = _lotile_case(5, T=5, E=E, k=2, n_in=n_in, n_out=n_out, r=r, M=E, N=E)
    phi = np.stack([np.arange(E), np.arange(E)], axis=1).astype(np.int32)
    got = oracle.lotile_forward(x, us.view(np.uint16), v.view(np.uint16), phi, idx, w)
    codes = np.zeros((n_out, n_in), dtype=np.uint8)
    zero_scale = np.zeros((n_out, n_in // g), dtype=np.float16).view(np.uint16)
    ref = np.zeros_like(got)
    for b in range(x.shape[0]):
        for t in range(idx.shape[1]):
            e = idx[b, t]
            ref[b] += float(w[b, t]) * oracle.project(x[b].astype(np.float64), codes, zero_scale, zero_scale,
                                                      us[e].view(np.uint16), v[e].view(np.uint16), g)
    assert np.max(np.abs(got - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_lotile_closed_forms():
    x, us, v, phi, idx, w = _lotile_case(8, T=4, E=6, k=2, M=2, N=3)
    # one-hot input, one selected expert: a row of U_m Sigma times V_n, scaled by g
    xo = np.zeros_like(x)
    xo[:, 3] = 1.0
    i1 = idx[:, :1].copy()
    w1 = w[:, :1].copy()
    got = oracle.lotile_forward(xo, us.view(np.uint16), v.view(np.uint16), phi, i1, w1)
    for b in range(4):
        m, n = phi[i1[b, 0]]
        ref = float(w1[b, 0]) * us[m, 3].astype(np.float64) @ v[n].astype(np.float64)
        assert np.allclose(got[b], ref, rtol=0, atol=1e-14)
    # linear in the routing weights and in x; independent of the order of the selected experts
    y = oracle.lotile_forward(x, us.view(np.uint16), v.view(np.uint16), phi, idx, w)
    y2 = oracle.lotile_forward(x, us.view(np.uint16), v.view(np.uint16), phi, idx, 2 * w)
    assert np.allclose(y2, 2 * y, rtol=1e-13, atol=0)
    yr = oracle.lotile_forward(x, us.view(np.uint16), v.view(np.uint16), phi, idx[:, ::-1].copy(), w[:, ::-1].copy())
    assert np.allclose(yr, y, rtol=1e-13, atol=1e-15)
    # two experts that share a column tile accumulate in the same block of the buffer; sharing a row tile reuses
    # the same projection: with M = 1 every expert projects with U_0, with N = 1 every expert ends in V_0
    x1, us1, v1, phi1, idx1, w1 = _lotile_case(9, T=3, E=4, k=4, M=1, N=4)
    y1 = oracle.lotile_forward(x1, us1.view(np.uint16), v1.view(np.uint16), phi1, idx1, w1)
    t = x1.astype(np.float64) @ us1[0].astype(np.float64)
    ref = np.zeros_like(y1)
    for b in range(3):
        for j in range(4):
            ref[b] += float(w1[b, j]) * t[b] @ v1[phi1[idx1[b, j], 1]].astype(np.float64)
    assert np.allclose(y1, ref, rtol=1e-13, atol=1e-15)


# ------------------------------------------------------------------ mixed-precision shared factors (fp8 U, V; fp16 Sigma)
def test_fp8_e4m3_decode_matches_published_values_and_library():
    """The format's landmark values (smallest subnormal 2^-9, smallest normal 2^-6, 1, largest finite 448) and every
    one of the 256 codes against the CPU library conversion."""
    import torch
    with open(os.path.join(os.path.dirname(__file__), "golden", "fp8_e4m3_values.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            b, val = line.split()
            assert oracle.fp8_e4m3_to_double(int(b, 16)) == float(val)
    lib = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(torch.float8_e4m3fn).double().numpy()
    for b in range(256):
        got = oracle.fp8_e4m3_to_double(b)
        if np.isnan(lib[b]):
            assert np.isnan(got) and (b & 0x7F) == 0x7F
        else:
            assert got == lib[b] and np.signbit(got) == np.signbit(lib[b])


def _lotile_fp8_case(seed, T=7, E=6, k=3, n_in=20, n_out=12, r=5, M=2, N=3):
    import torch
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, n_in)).astype(np.float32)
    enc = lambda a: torch.from_numpy(a.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    dec = lambda b: torch.from_numpy(b).view(torch.float8_e4m3fn).double().numpy()
    u8 = enc(rng.standard_normal((M, n_in, r)))
    v8 = enc(rng.standard_normal((N, r, n_out)))
    sigma = (0.5 / (1 + np.arange(r))).astype(np.float16)
    tiles = rng.permutation(M * N)[:E]
    phi = np.stack([tiles // N, tiles % N], axis=1).astype(np.int32)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    w = rng.random((T, k)).astype(np.float32)
    return x, u8, sigma, v8, phi, idx, w, dec


@pytest.mark.parametrize("seed,M,N,E", [(0, 2, 3, 6), (1, 3, 3, 7), (2, 1, 4, 4)])
def test_lotile_fp8_equals_per_expert_definition(seed, M, N, E):
    """y_b = sum_t g_bt * x_b (U_m diag(sigma)) V_n with the factors decoded by the library conversion."""
    x, u8, sigma, v8, phi, idx, w, dec = _lotile_fp8_case(seed, E=E, M=M, N=N, k=min(3, E))
    got = oracle.lotile_forward_fp8(x, u8, sigma.view(np.uint16), v8, phi, idx, w)
    ud, vd, sd = dec(u8), dec(v8), sigma.astype(np.float64)
    ref = np.zeros_like(got)
    for b in range(x.shape[0]):
        for t in range(idx.shape[1]):
            m, n = phi[idx[b, t]]
            ref[b] += float(w[b, t]) * ((x[b].astype(np.float64) @ ud[m]) * sd) @ vd[n]
    assert np.max(np.abs(got - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_lotile_fp8_with_unit_sigma_is_the_fp16_operator_on_the_same_values():
    """Every fp8 value is an fp16 value: with sigma = 1 the mixed-precision operator is the pinned fp16 one."""
    x, u8, sigma, v8, phi, idx, w, dec = _lotile_fp8_case(4)
    ones = np.ones_like(sigma)
    got = oracle.lotile_forward_fp8(x, u8, ones.view(np.uint16), v8, phi, idx, w)
    ref = oracle.lotile_forward(x, dec(u8).astype(np.float16).view(np.uint16), dec(v8).astype(np.float16).view(np.uint16),
                                phi, idx, w)
    assert np.max(np.abs(got - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_lotile_fp8_sigma_scales_its_rank_component():
    """Doubling sigma doubles y; zeroing all but one sigma leaves the rank-1 term of that component."""
    x, u8, sigma, v8, phi, idx, w, dec = _lotile_fp8_case(6)
    y1 = oracle.lotile_forward_fp8(x, u8, sigma.view(np.uint16), v8, phi, idx, w)
    y2 = oracle.lotile_forward_fp8(x, u8, (sigma * 2).astype(np.float16).view(np.uint16), v8, phi, idx, w)
    assert np.max(np.abs(y2 - 2 * y1)) <= 1e-12 * np.max(np.abs(y1))
    parts = np.zeros_like(y1)
    for rho in range(sigma.size):
        one = np.zeros_like(sigma)
        one[rho] = sigma[rho]
        parts += oracle.lotile_forward_fp8(x, u8, one.view(np.uint16), v8, phi, idx, w)
    assert np.max(np.abs(parts - y1)) <= 1e-12 * np.max(np.abs(y1))
