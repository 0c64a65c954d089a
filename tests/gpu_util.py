"""Shared plumbing of the GPU parity tests: host arrays -> device tensors, and the library calls."""
import numpy as np
import torch

import oracle
from synth import make_layer, make_x, make_logits, f32_to_bf16_bits
import paper_2605_09281_amd.binding as tq

DEV = "cuda:0"


def dev16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV)


def desc_of(cfg, act=tq.TQ_ACT_BF16, flags=0):
    if getattr(cfg, "dense", False):
        flags |= tq.TQ_FLAG_DENSE_CODES
    return tq.make_desc(cfg.E, cfg.S, cfg.k, cfg.H, cfg.F, cfg.g, cfg.bits, cfg.r, act, flags)


def pack_layer_gpu(layer, act=tq.TQ_ACT_BF16):
    c = layer.cfg
    desc = desc_of(c, act)
    err = torch.zeros(1, dtype=torch.int32, device=DEV)
    packed = tq.tq_pack_weights(desc, torch.from_numpy(layer.codes).to(DEV), dev16(layer.scale), dev16(layer.zero),
                                dev16(layer.A) if c.r else None, dev16(layer.B) if c.r else None, err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    return packed


def x_device(x: np.ndarray, act):
    if act == tq.TQ_ACT_FP32:
        return torch.from_numpy(x).to(DEV)
    return torch.from_numpy(f32_to_bf16_bits(x).view(np.int16)).to(DEV).view(torch.bfloat16)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    return float(np.max(np.abs(got.astype(np.float64) - ref)) / np.max(np.abs(ref)))
