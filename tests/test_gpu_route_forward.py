"""tq_route_moe_forward (routing of Eq. 3 and the expert forward in one call): its three outputs against tq_route followed
by tq_moe_forward bit for bit, on batches whose routing runs inside the permutation's launch and on batches that fall
back to the routing kernel; the routing itself against the oracle; the Mixtral-shaped decode layer end to end."""
import numpy as np
import pytest
import torch

import oracle
from synth import CONFIGS, LayerConfig, make_layer, make_layer_fp8, make_x, make_logits
import paper_2605_09281_amd.binding as tq
from gpu_util import DEV, dev16, desc_of, pack_layer_gpu, x_device, rel_err

pytestmark = pytest.mark.gpu

REG_BF16 = 4 * 2.0 ** -9
TOL_FP32 = 1e-5


def rcfg(cfg_id, **kw):
    base = dict(name="rf", E=8, S=0, k=2, H=128, F=192, T=16, g=64, r=8, bits=4)
    base.update(kw)
    return LayerConfig(cfg_id, **base)


# fused: at most 64 tokens, 16 experts, 256 assignments; the others take the routing kernel
CASES = {
    "decode_16x8": (rcfg(971), True),
    "one_token": (rcfg(972, T=1, E=4, k=1), True),
    "64_tokens_16_experts_k4": (rcfg(973, T=64, E=16, k=4, r=16), True),
    "biased_router_shared_expert": (rcfg(974, T=20, E=12, k=6, S=1, zipf_s=1.1), True),
    "all_experts_selected": (rcfg(975, T=9, E=5, k=5), True),
    "no_lowrank": (rcfg(976, T=12, r=0), True),
    "65_tokens": (rcfg(977, T=65), False),
    "17_experts": (rcfg(978, T=8, E=17, k=2), False),
    "64_experts": (rcfg(985, T=16, E=64, k=4), False),
    "257_assignments": (rcfg(979, T=43, E=16, k=6), False),
    "prefill_sized": (rcfg(980, T=700, E=16, k=4), False),
}


def both_ways(cfg, act, flags=0, logits=None, bias=None):
    layer = make_layer(cfg)
    x = make_x(cfg)
    if logits is None:
        logits, bias = make_logits(cfg)
    packed = pack_layer_gpu(layer)
    desc = desc_of(cfg, act, flags)
    lg = torch.from_numpy(logits).to(DEV)
    bs = None if bias is None else torch.from_numpy(bias).to(DEV)
    xd = x_device(x, act)
    ws = torch.empty(tq.tq_moe_workspace_size(desc, cfg.T), dtype=torch.uint8, device=DEV)
    idx, w = tq.tq_route(lg, bs, cfg.k)
    y = tq.tq_moe_forward(desc, packed, xd, idx, w, workspace=ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    ws.fill_(0x5A)                                 # the second call starts from a dirty workspace
    idx2 = torch.full_like(idx, -7)
    w2 = torch.full_like(w, float("nan"))
    y2, _, _ = tq.tq_route_moe_forward(desc, packed, xd, lg, bs, idx2, w2, workspace=ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    return layer, x, logits, bias, (idx, w, y), (idx2, w2, y2)


@pytest.mark.parametrize("act", [tq.TQ_ACT_BF16, tq.TQ_ACT_FP32], ids=["bf16", "fp32"])
@pytest.mark.parametrize("name", list(CASES))
def test_fused_equals_route_then_forward(name, act):
    cfg, fused = CASES[name]
    print(f"route+forward {name} act {act} fused {fused}", flush=True)
    n_assign = cfg.T * cfg.k
    assert fused == (cfg.T <= 64 and cfg.E <= 16 and n_assign <= 256)      # the case exercises the branch it is listed for
    layer, x, logits, bias, (idx, w, y), (idx2, w2, y2) = both_ways(cfg, act)
    assert torch.equal(idx, idx2)
    assert torch.equal(w.view(torch.int32), w2.view(torch.int32))
    if act == tq.TQ_ACT_BF16:
        assert torch.equal(y.view(torch.int16), y2.view(torch.int16))
    else:
        assert torch.equal(y.view(torch.int32), y2.view(torch.int32))
    ridx, rw = oracle.route(logits, bias, cfg.k)
    assert np.array_equal(idx2.cpu().numpy(), ridx)
    assert np.max(np.abs(w2.cpu().numpy() - rw)) <= 1e-6
    ref = oracle.moe_forward_layer(layer, x, ridx, w2.cpu().numpy())
    assert rel_err(y2.float().cpu().numpy(), ref) <= (REG_BF16 if act == tq.TQ_ACT_BF16 else TOL_FP32)


def test_fused_routing_ties_and_infinite_scores():
    """Equal scores go to the lower index and -inf scores come last, inside the permutation's launch as in tq_route."""
    cfg = rcfg(981, T=4, E=8, k=3)
    logits = np.array([[1, 3, 3, 0, 3, 1, -2, 3],
                       [0.5] * 8,
                       [-np.inf, 0, -np.inf, 0, 1, 1, 1, -np.inf],
                       [7, 6, 5, 4, 3, 2, 1, 0]], dtype=np.float32)
    _, _, _, _, (idx, w, y), (idx2, w2, y2) = both_ways(cfg, tq.TQ_ACT_BF16, logits=logits, bias=None)
    ridx, rw = oracle.route(logits, None, cfg.k)
    assert np.array_equal(idx2.cpu().numpy(), ridx)
    assert torch.equal(idx, idx2) and torch.equal(w.view(torch.int32), w2.view(torch.int32))
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))


@pytest.mark.parametrize("flags", [tq.TQ_FLAG_FORCE_SMALL_TILE, tq.TQ_FLAG_FORCE_LARGE_TILE], ids=["tile32", "tile_large"])
def test_fused_routing_in_front_of_the_tiled_kernels(flags):
    """A decode-sized batch forced onto a tile path: the permutation then has no pre-pass workgroups beside it."""
    cfg = rcfg(982, T=24, E=8, k=2, r=16)
    _, _, _, _, (idx, w, y), (idx2, w2, y2) = both_ways(cfg, tq.TQ_ACT_BF16, flags)
    assert torch.equal(idx, idx2) and torch.equal(w.view(torch.int32), w2.view(torch.int32))
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))


def test_fused_with_fp8_factors():
    cfg = rcfg(983, T=16, E=8, k=2, r=16)
    fl = make_layer_fp8(cfg)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    desc = tq.make_desc(cfg.E, cfg.S, cfg.k, cfg.H, cfg.F, cfg.g, cfg.bits, cfg.r, tq.TQ_ACT_BF16, tq.TQ_FLAG_FP8_FACTORS)
    packed = tq.tq_pack_weights(desc, torch.from_numpy(fl.codes).to(DEV), dev16(fl.scale), dev16(fl.zero),
                                torch.from_numpy(fl.A8).to(DEV), torch.from_numpy(fl.B8).to(DEV), sigma=dev16(fl.sigma))
    lg = torch.from_numpy(logits).to(DEV)
    y, idx, w = tq.tq_route_moe_forward(desc, packed, x_device(x, tq.TQ_ACT_BF16), lg, None)
    torch.cuda.synchronize()
    ref = oracle.moe_forward_fp8(cfg, fl.codes, fl.scale, fl.zero, fl.a8_list(), fl.b8_list(), fl.sigma, x, idx.cpu().numpy(),
                                 w.cpu().numpy())
    assert np.array_equal(idx.cpu().numpy(), oracle.route(logits, bias, cfg.k)[0])
    assert rel_err(y.float().cpu().numpy(), ref) <= REG_BF16


def test_fused_argument_checks():
    cfg = rcfg(984)
    layer = make_layer(cfg)
    packed = pack_layer_gpu(layer)
    desc = desc_of(cfg, tq.TQ_ACT_BF16)
    x = x_device(make_x(cfg), tq.TQ_ACT_BF16)
    logits, _ = make_logits(cfg)
    lg = torch.from_numpy(logits).to(DEV)
    with pytest.raises(tq.TqError) as ei:
        tq.tq_route_moe_forward(desc, packed, x, None, None)
    assert ei.value.status == 1      # TQ_ERR_NULL
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(tq.TqError) as ei:
        tq.tq_route_moe_forward(desc, packed, x, lg, None, workspace=small)
    assert ei.value.status == 5      # TQ_ERR_WORKSPACE


def test_fused_decode_full_shape():
    """Benchmark config 2 (Mixtral-shaped decode) through the one-call entry point, replayed from a HIP graph as
    bench.py does."""
    cfg = CONFIGS[2]
    print("route+forward config 2: generating", flush=True)
    layer = make_layer(cfg, workers=16)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    packed = pack_layer_gpu(layer)
    desc = desc_of(cfg, tq.TQ_ACT_BF16)
    lg = torch.from_numpy(logits).to(DEV)
    bs = None if bias is None else torch.from_numpy(bias).to(DEV)
    xd = x_device(x, tq.TQ_ACT_BF16)
    ws = torch.empty(tq.tq_moe_workspace_size(desc, cfg.T), dtype=torch.uint8, device=DEV)
    idx = torch.empty((cfg.T, cfg.k), dtype=torch.int32, device=DEV)
    w = torch.empty((cfg.T, cfg.k), dtype=torch.float32, device=DEV)
    y = torch.empty_like(xd)
    tq.tq_init()
    tq.tq_route_moe_forward(desc, packed, xd, lg, bs, idx, w, y, ws)
    torch.cuda.synchronize()
    y_eager = y.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            tq.tq_route_moe_forward(desc, packed, xd, lg, bs, idx, w, y, ws)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        y.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_eager.view(torch.int16))
    ridx, rw = oracle.route(logits, bias, cfg.k)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    ref = oracle.moe_forward_layer(layer, x, ridx, w.cpu().numpy())
    e = rel_err(y.float().cpu().numpy(), ref)
    print(f"route+forward config 2: rel err {e:.3e}", flush=True)
    assert e <= REG_BF16
