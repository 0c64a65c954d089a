"""CPU check that the inputs of the GPU parity tests can SEE a lost term: on the transformed layers of
tests/variants.py the oracle's output moves by far more than the asserted bound when the low-rank factor of any
single projection is dropped (a planted mistake, on the oracle side), while on the plain benchmark-like layers it
moves by less than 2e-2 for some projections — which is why the transformed layers exist."""
import numpy as np
import pytest

import oracle
from synth import LayerConfig, make_layer, make_x, make_logits
import variants

BOUND = 2e-2


def _cfg(**kw):
    base = dict(name="pw", E=4, S=0, k=2, H=128, F=192, T=37, g=64, r=8, bits=4)
    base.update(kw)
    return LayerConfig(601, **base)


def _move(layer_ok, layer_bad, x, idx, w):
    a = oracle.moe_forward_layer(layer_ok, x, idx, w)
    b = oracle.moe_forward_layer(layer_bad, x, idx, w)
    return float(np.max(np.abs(a - b)) / np.max(np.abs(a)))


@pytest.mark.parametrize("kind", ["pure_lowrank", "amplified"])
@pytest.mark.parametrize("p", [0, 1, 2])
def test_dropping_one_low_rank_term_moves_the_output_far_beyond_the_bound(kind, p):
    cfg = _cfg()
    layer = make_layer(cfg, workers=1)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    idx, w = oracle.route(logits, bias, cfg.k)
    t = variants.pure_lowrank(variants.amplified(layer)) if kind == "pure_lowrank" else variants.amplified(layer)
    moved = _move(t, variants.zero_factor(t, p), x, idx, w)
    assert moved > 10 * BOUND, moved


def test_plain_layers_cannot_see_it():
    cfg = _cfg()
    layer = make_layer(cfg, workers=1)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    idx, w = oracle.route(logits, bias, cfg.k)
    assert _move(layer, variants.zero_factor(layer, 2), x, idx, w) < BOUND


def test_odd_quant_changes_the_result_and_stays_finite():
    cfg = _cfg()
    layer = make_layer(cfg, workers=1)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    idx, w = oracle.route(logits, bias, cfg.k)
    o = variants.odd_quant(layer, 5)
    z = o.zero.view(np.float16).astype(np.float32)
    assert np.any(z < 0) and np.any(z > cfg.qmax) and np.any(z != np.rint(z))
    y = oracle.moe_forward_layer(o, x, idx, w)
    assert np.all(np.isfinite(y))
    assert _move(layer, o, x, idx, w) > BOUND


def test_segment_edge_tokens_brute_force():
    rng = np.random.default_rng(3)
    idx = np.stack([rng.permutation(7)[:3] for _ in range(40)]).astype(np.int32)
    idx[idx == 2] = 3      # expert 2 gets nothing... but a token must not select expert 3 twice
    for t in range(idx.shape[0]):
        if len(set(idx[t])) < 3:
            idx[t] = [0, 1, 4]
    tok = variants.segment_edge_tokens(idx, 7, extra_rows=(5,))
    offsets, slot_of, src_of = oracle.permute(idx, 7)
    want = set()
    for e in range(7):
        n = offsets[e + 1] - offsets[e]
        if n == 0:
            continue
        for s in {offsets[e], offsets[e + 1] - 1} | ({offsets[e] + 5} if n > 5 else set()):
            want.add(int(src_of[s]) // 3)
    assert set(tok.tolist()) == want
