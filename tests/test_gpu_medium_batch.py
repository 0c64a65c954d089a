"""Medium batches on layers of few, wide experts (tens of rows per expert, a handful of row tiles): the tiled kernels'
pre-pass then cuts the contraction into slices summed by a second launch, and the 64-row tiling splits the down
projection over K into fp32 planes and deals the column blocks of every row tile to the XCDs.  Every path against the oracle on layers wide enough for several slices and
two planes; run-to-run determinism of the sliced sums; the same layers with fp8 factors and dense 3-bit codes.
Second part: small batches on layers of many experts, which the decode kernels take with a device-side deal of their
workgroups."""
import numpy as np
import pytest
import torch

import oracle
from synth import LayerConfig, make_layer, make_layer_fp8, make_x, make_logits
import paper_2605_09281_amd.binding as tq
from gpu_util import DEV, dev16, desc_of, pack_layer_gpu, x_device, rel_err

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


def wide(cfg_id, **kw):
    base = dict(name="wide", E=4, S=0, k=2, H=1024, F=4096, T=100, g=64, r=16, bits=4)
    base.update(kw)
    return LayerConfig(cfg_id, **base)


# gate/up: 1024 / 512 = 2 slices, down: 4096 / 512 = 8 slices; 4096 / 2048 = 2 planes on the 64-row tiling
WIDE = {
    "g64_r16_50_rows": wide(1201),
    "g64_r16_12_rows": wide(1202, T=24),
    "g128_r32_shared": wide(1203, g=128, r=32, E=5, S=1, k=2, T=160),
    "g32_r40": wide(1204, g=32, r=40, T=70),                    # three column tiles of t, chunks of 128 indices
    "g64_r64_6_experts": wide(1205, r=64, E=6, k=3, T=130),     # four column tiles of t in the gate/up pre-pass
    "rank0": wide(1206, r=0, T=90),                             # slices of group sums only, no second launch
    "ragged_last_chunk": wide(1207, H=1088, F=4160, T=80),      # 17 and 65 groups: a short last chunk in the last slice
    "11_column_blocks": wide(1208, H=512, F=1408, E=3, T=60),   # gate/up: 11 blocks of 4 column pairs over 8 XCDs
}

_cache = {}


def get_layer(cfg):
    if cfg.cfg_id not in _cache:
        _cache[cfg.cfg_id] = make_layer(cfg, workers=8)
    return _cache[cfg.cfg_id]


def run(cfg, flags):
    layer = get_layer(cfg)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    packed = pack_layer_gpu(layer)
    idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None if bias is None else torch.from_numpy(bias).to(DEV), cfg.k)
    desc = desc_of(cfg, tq.TQ_ACT_BF16, flags)
    ws = torch.empty(tq.tq_moe_workspace_size(desc, cfg.T), dtype=torch.uint8, device=DEV)
    ws.fill_(0x5A)
    y = tq.tq_moe_forward(desc, packed, x_device(x, tq.TQ_ACT_BF16), idx, w, workspace=ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    ref = oracle.moe_forward_layer(layer, x, idx.cpu().numpy(), w.cpu().numpy())
    return y, ref


@pytest.mark.parametrize("flags", [tq.TQ_FLAG_FORCE_SMALL_TILE, tq.TQ_FLAG_FORCE_LARGE_TILE, 0],
                         ids=["tile32", "tile_large", "auto"])
@pytest.mark.parametrize("name", list(WIDE))
def test_wide_experts_medium_batch(name, flags):
    print(f"medium batch {name} flags {flags}", flush=True)
    y, ref = run(WIDE[name], flags)
    assert rel_err(y.float().cpu().numpy(), ref) <= TOL_BF16


@pytest.mark.parametrize("flags", [tq.TQ_FLAG_FORCE_SMALL_TILE, tq.TQ_FLAG_FORCE_LARGE_TILE], ids=["tile32", "tile_large"])
def test_sliced_sums_are_run_to_run_deterministic(flags):
    cfg = WIDE["g64_r16_50_rows"]
    a, _ = run(cfg, flags)
    b, _ = run(cfg, flags)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("flags", [tq.TQ_FLAG_FORCE_SMALL_TILE, tq.TQ_FLAG_FORCE_LARGE_TILE], ids=["tile32", "tile_large"])
def test_wide_experts_fp8_factors(flags):
    cfg = wide(1210, T=110, r=32)
    fl = make_layer_fp8(cfg)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    desc = tq.make_desc(cfg.E, cfg.S, cfg.k, cfg.H, cfg.F, cfg.g, cfg.bits, cfg.r, tq.TQ_ACT_BF16, tq.TQ_FLAG_FP8_FACTORS | flags)
    packed = tq.tq_pack_weights(desc, torch.from_numpy(fl.codes).to(DEV), dev16(fl.scale), dev16(fl.zero),
                                torch.from_numpy(fl.A8).to(DEV), torch.from_numpy(fl.B8).to(DEV), sigma=dev16(fl.sigma))
    idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None, cfg.k)
    y = tq.tq_moe_forward(desc, packed, x_device(x, tq.TQ_ACT_BF16), idx, w)
    torch.cuda.synchronize()
    ref = oracle.moe_forward_fp8(cfg, fl.codes, fl.scale, fl.zero, fl.a8_list(), fl.b8_list(), fl.sigma, x, idx.cpu().numpy(),
                                 w.cpu().numpy())
    assert rel_err(y.float().cpu().numpy(), ref) <= TOL_BF16


@pytest.mark.parametrize("flags", [tq.TQ_FLAG_FORCE_SMALL_TILE, tq.TQ_FLAG_FORCE_LARGE_TILE], ids=["tile32", "tile_large"])
def test_wide_experts_dense_3bit(flags):
    y, ref = run(wide(1211, bits=3, dense=True, T=100), flags)
    assert rel_err(y.float().cpu().numpy(), ref) <= TOL_BF16


# ------------------------------------------------------------------ small batches on layers of many experts
# The decode kernels on layers of more than 32 experts: their workgroups share out the row tiles that exist (most
# experts receive no row), wave slices of 256 contraction indices up to a contraction of 2048 and of 512 beyond.
MANY = {
    "40_experts_10_tokens": wide(1301, E=40, k=4, H=256, F=384, T=10),
    "70_experts_shared": wide(1302, E=70, S=1, k=6, H=256, F=320, g=32, r=24, T=9),
    "36_experts_skewed_tall_tiles": wide(1303, E=36, k=2, H=192, F=256, T=100, zipf_s=1.3),     # hot experts hold several 16-row tiles
    "wave_slices_of_512": wide(1304, E=33, k=3, H=2304, F=2176, g=128, r=16, T=8),             # 4.5 and 4.25 slices of 512
    "more_tiles_than_cus": wide(1305, E=300, k=1, H=128, F=128, r=0, T=290),                    # one workgroup per tile, some tiles without any
}


@pytest.mark.parametrize("flags", [tq.TQ_FLAG_FORCE_SKINNY, 0], ids=["tile16", "auto"])
@pytest.mark.parametrize("name", list(MANY))
def test_many_experts_small_batch(name, flags):
    print(f"many experts {name} flags {flags}", flush=True)
    y, ref = run(MANY[name], flags)
    assert rel_err(y.float().cpu().numpy(), ref) <= TOL_BF16


def test_many_experts_run_to_run_deterministic():
    cfg = MANY["36_experts_skewed_tall_tiles"]
    a, _ = run(cfg, tq.TQ_FLAG_FORCE_SKINNY)
    b, _ = run(cfg, tq.TQ_FLAG_FORCE_SKINNY)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("name,flags", [("g128_r32_shared", tq.TQ_FLAG_FORCE_LARGE_TILE), ("g64_r16_50_rows", tq.TQ_FLAG_FORCE_SMALL_TILE),
                                        ("40_experts_10_tokens", 0)], ids=["large_split", "tile32_sliced", "many_experts_decode"])
def test_replayed_from_a_hip_graph(name, flags):
    """The launches these batches add (slice sums, split planes, one-workgroup permutation, device-side deal) captured
    in a HIP graph: every replay, with eager work in between, equals the eager result bit for bit."""
    cfg = WIDE.get(name) or MANY[name]
    layer = get_layer(cfg)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    packed = pack_layer_gpu(layer)
    desc = desc_of(cfg, tq.TQ_ACT_BF16, flags)
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
        ws.fill_(0x3C)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_eager.view(torch.int16))


def test_blob_of_another_layer_in_a_mid_sized_batch():
    """400 assignments (two chunks: the one-workgroup permutation) with a blob whose header does not match the
    descriptor: flag bit 1 is set and the tile counts are cleared, so that no later kernel indexes the blob."""
    cfg = wide(1401, H=128, F=192, T=200, r=8)
    other = wide(1402, H=128, F=256, T=200, r=8)
    layer = get_layer(cfg)
    packed = pack_layer_gpu(layer)
    logits, bias = make_logits(cfg)
    idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None, cfg.k)
    desc = desc_of(other, tq.TQ_ACT_BF16, 0)
    big = torch.zeros(tq.tq_packed_size(desc), dtype=torch.uint8, device=DEV)
    big[:packed.numel()] = packed                      # readable at the other layer's size, wrong header
    ws = torch.empty(tq.tq_moe_workspace_size(desc, cfg.T), dtype=torch.uint8, device=DEV)
    ws.fill_(0x11)
    tq.tq_moe_forward(desc, big, x_device(make_x(cfg), tq.TQ_ACT_BF16), idx, w, workspace=ws)
    torch.cuda.synchronize()
    ctrl = ws[:24].view(torch.int32).cpu().numpy()
    assert ctrl[0] & 2
    assert ctrl[1] == 0 and ctrl[2] == 0 and ctrl[3] == 0 and ctrl[4] == 0 and ctrl[5] == 0

