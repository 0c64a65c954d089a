"""GPU parity at the corners of what the descriptor allows: smallest dimensions, largest supported rank, groups of
32 and 256 on every tile path, a single expert, all experts selected, shared experts on the decode path, and a
workspace reused across batch sizes.  Same bar as the other parity tests."""
import numpy as np
import pytest
import torch

import oracle
from synth import LayerConfig, make_layer, make_x, make_logits
import paper_2605_09281_amd.binding as tq
from gpu_util import DEV, desc_of, pack_layer_gpu, x_device, rel_err

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
TOL_FP32 = 1e-5
FLAGS = {"auto": 0, "tile32": tq.TQ_FLAG_FORCE_SMALL_TILE, "tile_large": tq.TQ_FLAG_FORCE_LARGE_TILE,
         "tile16": tq.TQ_FLAG_FORCE_SKINNY}


def corner(cfg_id, **kw):
    base = dict(name="c", E=4, S=0, k=2, H=128, F=128, T=40, g=64, r=8, bits=4)
    base.update(kw)
    return LayerConfig(cfg_id, **base)


CORNERS = {
    "min_dims_g32": corner(501, H=64, F=64, g=32, r=4, T=9),
    "min_dims_g64_rank0": corner(502, H=64, F=64, g=64, r=0, T=70),
    "one_group_per_row": corner(503, H=128, F=128, g=128, r=16, T=33),
    "g32_many_rows": corner(504, H=128, F=192, g=32, r=8, E=4, T=300),
    "g256": corner(505, H=256, F=512, g=256, r=16, E=4, T=40),
    "g256_many_rows": corner(506, H=256, F=512, g=256, r=16, E=3, k=2, T=260),
    "rank128": corner(507, H=256, F=256, g=64, r=128, E=3, T=50),
    "rank1": corner(508, H=128, F=192, g=64, r=1, T=20),
    "one_expert": corner(509, E=1, k=1, T=70),
    "all_experts": corner(510, E=6, k=6, T=33),
    "shared_decode": corner(511, E=8, S=2, k=2, T=3),
    "int3_g256": corner(512, H=256, F=256, g=256, bits=3, r=8, T=25),
}

_layers = {}


def forward(cfg, act, flags, ws=None, T=None):
    if cfg.cfg_id not in _layers:
        _layers[cfg.cfg_id] = (make_layer(cfg, workers=8), make_x(cfg), make_logits(cfg))
    layer, x, (logits, bias) = _layers[cfg.cfg_id]
    if T is not None:
        x, logits = x[:T], logits[:T]
    n = x.shape[0]
    packed = pack_layer_gpu(layer)
    idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None if bias is None else torch.from_numpy(bias).to(DEV), cfg.k)
    desc = desc_of(cfg, act, flags)
    if ws is None:
        ws = torch.empty(tq.tq_moe_workspace_size(desc, n), dtype=torch.uint8, device=DEV)
    y = tq.tq_moe_forward(desc, packed, x_device(x, act), idx, w, workspace=ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    ridx, _ = oracle.route(logits, bias, cfg.k)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    ref = oracle.moe_forward_layer(layer, x, ridx, w.cpu().numpy())
    return y.float().cpu().numpy(), ref


@pytest.mark.parametrize("flag", list(FLAGS))
@pytest.mark.parametrize("name", list(CORNERS))
def test_corner_bf16(name, flag):
    print(f"corner {name} flag {flag}", flush=True)
    got, ref = forward(CORNERS[name], tq.TQ_ACT_BF16, FLAGS[flag])
    assert rel_err(got, ref) <= TOL_BF16


@pytest.mark.parametrize("name", ["min_dims_g32", "g256", "rank128", "one_expert", "shared_decode", "int3_g256"])
def test_corner_fp32(name):
    print(f"corner {name} fp32", flush=True)
    got, ref = forward(CORNERS[name], tq.TQ_ACT_FP32, 0)
    assert rel_err(got, ref) <= TOL_FP32


def test_rank_above_the_bf16_limit_is_refused_not_mangled():
    """The bf16 kernels carry at most 128 rank columns: a larger rank returns TQ_ERR_UNSUPPORTED (6) before any launch;
    the fp32 debug path takes it."""
    cfg = corner(520, H=128, F=128, g=64, r=130, E=2, k=1, T=6)
    with pytest.raises(tq.TqError) as ei:
        forward(cfg, tq.TQ_ACT_BF16, 0)
    assert ei.value.status == 6
    got, ref = forward(cfg, tq.TQ_ACT_FP32, 0)
    assert rel_err(got, ref) <= TOL_FP32


def test_workspace_sized_for_a_large_batch_serves_smaller_ones():
    cfg = corner(521, H=128, F=192, g=64, r=8, E=5, k=2, T=150)
    desc = desc_of(cfg, tq.TQ_ACT_BF16, 0)
    ws = torch.empty(tq.tq_moe_workspace_size(desc, cfg.T), dtype=torch.uint8, device=DEV)
    for T in (150, 7, 64, 1):
        print(f"workspace reuse T={T}", flush=True)
        got, ref = forward(cfg, tq.TQ_ACT_BF16, 0, ws=ws, T=T)
        assert rel_err(got, ref) <= TOL_BF16


def test_workspace_serves_smaller_batches_across_the_path_thresholds():
    """Sized for a batch on the tiled path (more than 4096 assignment rows), then used for batches that take the
    split-K planes (at most 4096 rows) and the decode scratch (at most 1024 rows)."""
    cfg = corner(522, H=128, F=192, g=64, r=8, E=6, k=3, T=1500)
    desc = desc_of(cfg, tq.TQ_ACT_BF16, 0)
    ws = torch.empty(tq.tq_moe_workspace_size(desc, cfg.T), dtype=torch.uint8, device=DEV)
    for T in (1500, 1300, 300, 5):
        print(f"workspace reuse across thresholds T={T}", flush=True)
        assert tq.tq_moe_workspace_size(desc, T) <= ws.numel()
        got, ref = forward(cfg, tq.TQ_ACT_BF16, 0, ws=ws, T=T)
        assert rel_err(got, ref) <= TOL_BF16


def test_many_rows_small_layer():
    """Tens of thousands of tokens on a small layer: thousands of row tiles per expert, multi-chunk permutation,
    persistent workgroups walking long item lists; sampled tokens against the oracle, all tokens finite."""
    cfg = corner(530, H=128, F=128, g=64, r=8, E=4, k=2, T=60000)
    layer = make_layer(cfg, workers=8)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    packed = pack_layer_gpu(layer)
    idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None, cfg.k)
    desc = desc_of(cfg, tq.TQ_ACT_BF16, 0)
    ws = torch.empty(tq.tq_moe_workspace_size(desc, cfg.T), dtype=torch.uint8, device=DEV)
    y = tq.tq_moe_forward(desc, packed, x_device(x, tq.TQ_ACT_BF16), idx, w, workspace=ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    assert bool(torch.isfinite(y.float()).all())
    rng = np.random.default_rng(530)
    tok = np.unique(np.concatenate([[0, cfg.T - 1], rng.integers(0, cfg.T, 400)])).astype(np.int32)
    ref = oracle.moe_forward_layer(layer, x, idx.cpu().numpy(), w.cpu().numpy(), tokens=tok)
    got = y[torch.from_numpy(tok.astype(np.int64)).to(DEV)].float().cpu().numpy()
    assert rel_err(got, ref) <= TOL_BF16

