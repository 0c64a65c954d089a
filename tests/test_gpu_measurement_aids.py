"""The measurement aids of the boundary (not part of the method): argument checks and what they leave behind."""
import numpy as np
import pytest
import torch

import paper_2605_09281_amd.binding as tq
from gpu_util import DEV

pytestmark = pytest.mark.gpu


def test_debug_stream_copies_and_checks_its_arguments():
    n = 1 << 20
    src = torch.arange(n, dtype=torch.int32, device=DEV).view(torch.uint8)
    dst = torch.zeros_like(src)
    tq.tq_debug_stream(src, dst, src.numel(), 0)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    small = torch.zeros(16, dtype=torch.uint8, device=DEV)
    for mode in (1, 2):                      # read-only modes leave the 16-byte destination alone
        tq.tq_debug_stream(src, small, src.numel(), mode)
    torch.cuda.synchronize()
    assert int(small.sum()) == 0
    with pytest.raises(tq.TqError):
        tq.tq_debug_stream(src, dst, 24, 0)              # not a multiple of 16
    with pytest.raises(tq.TqError):
        tq.tq_debug_stream(src, dst, 32, 3)              # no such mode


@pytest.mark.parametrize("level", [0, 1, 2, 3, 4])
def test_issue_probe_reports_plausible_counters(level):
    scratch = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    scratch[256:512].view(torch.float32).fill_(0.5)
    iters = 500
    tq.tq_debug_issue_probe(level, iters, scratch)
    torch.cuda.synchronize()
    cycles, ticks = scratch[:16].view(torch.int64).cpu().tolist()
    mfmas = 32 * iters
    # an MFMA of this shape holds the matrix unit for 32 cycles and two waves share it: between 32 and 200 cycles
    # per MFMA of one wave, at a clock between 1 and 3 GHz (the wall clock ticks at 100 MHz)
    assert 32 * mfmas <= cycles <= 400 * mfmas, (cycles, mfmas)
    assert ticks > 0 and 1.0 <= cycles / (ticks * 10.0) <= 3.0


def test_issue_probe_checks_its_arguments():
    scratch = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    with pytest.raises(tq.TqError):
        tq.tq_debug_issue_probe(5, 10, scratch)
    with pytest.raises(tq.TqError):
        tq.tq_debug_issue_probe(0, 0, scratch)
    with pytest.raises(tq.TqError):
        tq.tq_debug_issue_probe(0, 10, scratch[:1024])


def test_stage_events_are_recorded_in_order():
    """tq_set_profile_events: the forward records the events it is given at its stage boundaries, on its stream."""
    from synth import CONFIGS, make_layer, make_x, make_logits
    from gpu_util import pack_layer_gpu, desc_of, x_device
    cfg = CONFIGS[1]
    layer = make_layer(cfg, workers=4)
    packed = pack_layer_gpu(layer)
    logits, bias = make_logits(cfg)
    idx, w = tq.tq_route(torch.from_numpy(logits).to(DEV), None, cfg.k)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(7)]
    for e in evs:
        e.record()                       # creates the underlying HIP events
    torch.cuda.synchronize()
    try:
        tq.tq_set_profile_events([e.cuda_event for e in evs])
        tq.tq_moe_forward(desc_of(cfg), packed, x_device(make_x(cfg), tq.TQ_ACT_BF16), idx, w)
        torch.cuda.synchronize()
    finally:
        tq.tq_set_profile_events([])
    total = evs[0].elapsed_time(evs[6])
    parts = [evs[i].elapsed_time(evs[i + 1]) for i in range(6)]
    assert all(p >= 0.0 for p in parts) and total > 0.0
    assert abs(sum(parts) - total) <= 0.05 * total + 0.01
