"""tq_moe_forward_static (the entry point for callers that cannot allocate) against tq_moe_forward: same kernels,
the library's static scratch array instead of a caller workspace.  Two calls in a row, the second on a smaller
batch, each compared with the workspace entry point bit for bit and with the oracle within the parity bound;
then a batch that needs more scratch than the array holds is refused before any launch."""
import numpy as np
import pytest
import torch

import oracle
from synth import CONFIGS, LayerConfig, make_layer, make_x, make_logits
import paper_2605_09281_amd.binding as tq
from gpu_util import DEV, desc_of, pack_layer_gpu, x_device, rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("act", [tq.TQ_ACT_BF16, tq.TQ_ACT_FP32], ids=["bf16", "fp32"])
def test_static_scratch_entry_point_matches_the_workspace_entry_point(act):
    cfg = CONFIGS[1]
    layer = make_layer(cfg, workers=4)
    x_all = make_x(cfg)
    logits_all, bias = make_logits(cfg)
    packed = pack_layer_gpu(layer, act)
    desc = desc_of(cfg, act, 0)
    tq.tq_init()
    err = torch.full((1,), 77, dtype=torch.int32, device=DEV)
    for T in (cfg.T, 21):                      # the second call is smaller and finds the first call's leftovers
        print(f"static scratch: T={T}", flush=True)
        x, logits = x_all[:T], logits_all[:T]
        assert tq.tq_moe_workspace_size(desc, T) <= tq.TQ_STATIC_SCRATCH_MAX
        idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None, cfg.k)
        xd = x_device(x, act)
        y_ws = tq.tq_moe_forward(desc, packed, xd, idx, w)
        y_st = torch.full_like(xd, float("nan"))
        tq.tq_moe_forward_static(desc, packed, xd, idx, w, y_st, err_flag=err)
        torch.cuda.synchronize()
        assert int(err.item()) == 0
        a = y_ws.view(torch.int16 if act == tq.TQ_ACT_BF16 else torch.int32)
        b = y_st.view(torch.int16 if act == tq.TQ_ACT_BF16 else torch.int32)
        assert torch.equal(a, b)
        ref = oracle.moe_forward_layer(layer, x, idx.cpu().numpy(), w.cpu().numpy())
        assert rel_err(y_st.float().cpu().numpy(), ref) <= (4 * 2.0 ** -9 if act == tq.TQ_ACT_BF16 else 1e-5)
    # an out-of-range expert index reaches the caller's flag
    idx_bad = idx.clone()
    idx_bad[3, 0] = cfg.E
    tq.tq_moe_forward_static(desc, packed, xd, idx_bad, w, y_st, err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 1


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    cfg = LayerConfig(990, "big", E=8, S=0, k=2, H=4096, F=14336, T=4096, g=128, r=32, bits=4)
    desc = desc_of(cfg, tq.TQ_ACT_BF16, 0)
    assert tq.tq_moe_workspace_size(desc, cfg.T) > tq.TQ_STATIC_SCRATCH_MAX
    fake = torch.zeros(256, dtype=torch.uint8, device=DEV)
    x = torch.zeros((cfg.T, cfg.H), dtype=torch.bfloat16, device=DEV)
    idx = torch.zeros((cfg.T, cfg.k), dtype=torch.int32, device=DEV)
    w = torch.zeros((cfg.T, cfg.k), dtype=torch.float32, device=DEV)
    with pytest.raises(tq.TqError) as ei:
        tq.tq_moe_forward_static(desc, fake, x, idx, w, torch.empty_like(x))
    assert ei.value.status == 5
