"""The layer on SHARED 2D-tiled factors (Section 3.1, Eq. 4; tq_pack_weights_shared): the blob byte for byte against
oracle/pack_ref.py, the forward on every kernel family against the oracle's shared-factor layer, and, in the
degenerate tiling where every expert owns its tile, equality with the per-expert format's output bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from oracle import pack_ref
from synth import CONFIGS, LayerConfig, make_layer, make_shared_layer, make_x, make_logits
import paper_2605_09281_amd.binding as tq
from gpu_util import DEV, dev16, desc_of, pack_layer_gpu, x_device, rel_err

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
REG_BF16 = 4 * 2.0 ** -9
TOL_FP32 = 1e-5


def scfg(cfg_id, **kw):
    base = dict(name="sh", E=6, S=0, k=2, H=128, F=192, T=9, g=64, r=8, bits=4)
    base.update(kw)
    return LayerConfig(cfg_id, **base)


# name -> (config, M, N); None = the near-square grid of the paper
CASES = {
    "grid2x3": (scfg(851), 2, 3),
    "grid3x3_shared_expert_r32": (scfg(852, E=7, S=1, k=3, H=256, F=384, g=128, r=32, T=40), None, None),
    "grid1x1_all_share": (scfg(853, E=4, r=16, T=70), 1, 1),
    "grid2x2_fewer_tiles_than_experts": (scfg(854, E=8, k=2, g=32, r=20, T=33), 2, 2),
    "grid4x2_r48_int3": (scfg(855, E=8, k=2, H=256, F=128, bits=3, r=48, T=300), 4, 2),
    "dense3_grid2x2": (scfg(856, E=4, bits=3, dense=True, T=11), 2, 2),
}
_cache = {}


def get(name):
    if name not in _cache:
        cfg, M, N = CASES[name]
        _cache[name] = (make_shared_layer(cfg, M, N), make_x(cfg), make_logits(cfg))
    return _cache[name]


def shared_desc(sl, act=tq.TQ_ACT_BF16, flags=0):
    c = sl.cfg
    if c.dense:
        flags |= tq.TQ_FLAG_DENSE_CODES
    return tq.make_desc(c.E, c.S, c.k, c.H, c.F, c.g, c.bits, c.r, act, flags, tiles_m=sl.M, tiles_n=sl.N)


def pack_shared_gpu(sl, act=tq.TQ_ACT_BF16, phi=None):
    err = torch.zeros(1, dtype=torch.int32, device=DEV)
    packed = tq.tq_pack_weights_shared(shared_desc(sl, act), torch.from_numpy(sl.codes).to(DEV), dev16(sl.scale), dev16(sl.zero),
                                       [dev16(a) for a in sl.us], [dev16(a) for a in sl.v],
                                       torch.from_numpy(sl.phi if phi is None else phi).to(DEV), err_flag=err)
    torch.cuda.synchronize()
    return packed, int(err.item())


@pytest.mark.parametrize("name", list(CASES))
def test_shared_pack_is_byte_exact(name):
    sl, _, _ = get(name)
    packed, err = pack_shared_gpu(sl)
    assert err == 0
    ref = pack_ref.pack_layer_shared(sl)
    body = packed.cpu().numpy()[256:]
    assert body.size == ref.size == tq.tq_packed_size(shared_desc(sl)) - 256
    assert np.array_equal(body, ref)
    # unpack returns the per-expert residual (codes, scale, zero)
    codes = torch.full(sl.codes.shape, 255, dtype=torch.uint8, device=DEV)
    scale = torch.zeros(sl.scale.shape, dtype=torch.int16, device=DEV)
    zero = torch.zeros_like(scale)
    tq.tq_unpack_weights(shared_desc(sl), packed, codes, scale, zero)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), sl.codes)
    assert np.array_equal(scale.cpu().numpy().view(np.uint16), sl.scale)
    assert np.array_equal(zero.cpu().numpy().view(np.uint16), sl.zero)


def test_phi_outside_the_grid_sets_the_flag():
    sl, _, _ = get("grid2x3")
    phi = sl.phi.copy()
    phi[1, 1] = 3
    _, err = pack_shared_gpu(sl, phi=phi)
    assert err & 1
    phi = sl.phi.copy()
    phi[0, 0] = -1
    _, err = pack_shared_gpu(sl, phi=phi)
    assert err & 1


def run_forward(desc, packed, x, idx, w, act):
    ws = torch.empty(tq.tq_moe_workspace_size(desc, x.shape[0]), dtype=torch.uint8, device=DEV)
    y = tq.tq_moe_forward(desc, packed, x_device(x, act), idx, w, workspace=ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    return y.float().cpu().numpy()


PATHS = {"auto": 0, "small_tile": tq.TQ_FLAG_FORCE_SMALL_TILE, "large_tile": tq.TQ_FLAG_FORCE_LARGE_TILE,
         "decode": tq.TQ_FLAG_FORCE_SKINNY}


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("name", list(CASES))
def test_shared_forward_bf16(name, path):
    print(f"shared bf16 {name} {path}", flush=True)
    sl, x, (logits, bias) = get(name)
    cfg = sl.cfg
    packed, err = pack_shared_gpu(sl)
    assert err == 0
    idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None if bias is None else torch.from_numpy(bias).to(DEV), cfg.k)
    got = run_forward(shared_desc(sl, flags=PATHS[path]), packed, x, idx, w, tq.TQ_ACT_BF16)
    ref = oracle.moe_forward_shared(sl, x, idx.cpu().numpy(), w.cpu().numpy())
    e = rel_err(got, ref)
    print(f"   rel err {e:.3e}", flush=True)
    assert e <= TOL_BF16
    assert e <= REG_BF16


@pytest.mark.parametrize("name", list(CASES))
def test_shared_forward_fp32(name):
    print(f"shared fp32 {name}", flush=True)
    sl, x, (logits, bias) = get(name)
    cfg = sl.cfg
    packed, err = pack_shared_gpu(sl, tq.TQ_ACT_FP32)
    assert err == 0
    idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None if bias is None else torch.from_numpy(bias).to(DEV), cfg.k)
    got = run_forward(shared_desc(sl, tq.TQ_ACT_FP32), packed, x, idx, w, tq.TQ_ACT_FP32)
    ref = oracle.moe_forward_shared(sl, x, idx.cpu().numpy(), w.cpu().numpy())
    assert rel_err(got, ref) <= TOL_FP32


@pytest.mark.parametrize("path", list(PATHS))
def test_degenerate_tiling_equals_the_per_expert_format_bit_for_bit(path):
    """M = N = E+S, phi(e) = (e, e), tile e's factors = expert e's: same kernels, same operands, other addresses."""
    print(f"shared degenerate {path}", flush=True)
    cfg = scfg(860, E=5, S=1, k=2, H=128, F=256, r=24, T=150)
    layer = make_layer(cfg)
    sl = make_shared_layer(cfg, layer=layer, degenerate=True)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None, cfg.k)
    packed_s, err = pack_shared_gpu(sl)
    assert err == 0
    y_s = run_forward(shared_desc(sl, flags=PATHS[path]), packed_s, x, idx, w, tq.TQ_ACT_BF16)
    y_e = run_forward(desc_of(cfg, flags=PATHS[path]), pack_layer_gpu(layer), x, idx, w, tq.TQ_ACT_BF16)
    assert np.array_equal(y_s, y_e)


def test_blob_of_the_other_format_is_refused_by_the_forward():
    sl, x, (logits, _) = get("grid2x3")
    cfg = sl.cfg
    packed, _ = pack_shared_gpu(sl)
    idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None, cfg.k)
    desc = desc_of(cfg)           # per-expert descriptor, shared blob (which is larger: sizes pass)
    ws = torch.empty(tq.tq_moe_workspace_size(desc, x.shape[0]), dtype=torch.uint8, device=DEV)
    tq.tq_moe_forward(desc, packed, x_device(x, tq.TQ_ACT_BF16), idx, w, workspace=ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) & 2


def test_shared_full_shape_decode_layer():
    """The Mixtral-shaped decode layer (benchmark config 2) on a 3 x 3 grid of shared factors."""
    cfg = CONFIGS[2].replace(cfg_id=870)
    print("shared config 2: generating", flush=True)
    sl = make_shared_layer(cfg, workers=16)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    packed, err = pack_shared_gpu(sl)
    assert err == 0
    idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None if bias is None else torch.from_numpy(bias).to(DEV), cfg.k)
    got = run_forward(shared_desc(sl), packed, x, idx, w, tq.TQ_ACT_BF16)
    ref = oracle.moe_forward_shared(sl, x, idx.cpu().numpy(), w.cpu().numpy())
    e = rel_err(got, ref)
    print(f"shared config 2: rel err {e:.3e}", flush=True)
    assert e <= REG_BF16
