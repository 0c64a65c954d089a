"""ctypes binding of libtileq.so: same names as the C ABI, torch tensors in and out.

Marshalling only.  Every step of the path runs in the library's kernels; torch is used for
device allocations and for the current stream.  Fails loudly when the library is missing.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from .build import library_path

TQ_OK = 0
TQ_ACT_BF16, TQ_ACT_FP32 = 0, 1
TQ_FLAG_FORCE_SMALL_TILE, TQ_FLAG_FORCE_LARGE_TILE, TQ_FLAG_FORCE_SKINNY = 1, 2, 4
TQ_FLAG_DENSE_CODES = 32
TQ_FLAG_FP8_FACTORS = 64
TQ_LOTILE_FP8 = 1
STATUS_NAMES = {0: "TQ_OK", 1: "TQ_ERR_NULL", 2: "TQ_ERR_SHAPE", 3: "TQ_ERR_ALIGN", 4: "TQ_ERR_RANGE",
                5: "TQ_ERR_WORKSPACE", 6: "TQ_ERR_UNSUPPORTED", 7: "TQ_ERR_HIP", 8: "TQ_ERR_BLOB"}

EXPORTS = ["tq_init", "tq_status_str", "tq_packed_size", "tq_pack_weights", "tq_pack_weights_shared", "tq_unpack_weights", "tq_route",
           "tq_permute_workspace_size", "tq_permute", "tq_moe_workspace_size", "tq_moe_forward", "tq_route_moe_forward", "tq_moe_forward_static",
           "tq_set_profile_events", "tq_debug_stream", "tq_debug_issue_probe", "tq_sketch_workspace_size", "tq_sketch_lowrank", "tq_lotile_packed_size", "tq_lotile_pack", "tq_lotile_pack_fp8",
           "tq_lotile_workspace_size", "tq_lotile_forward", "tq_lotile_grid", "tq_lotile_place"]


class TqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)}")


class LayerDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_experts", "n_shared", "top_k", "hidden", "ffn", "group", "bits", "rank", "act_dtype", "flags",
                 "tiles_m", "tiles_n")]


class LoTileDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_experts", "tiles_m", "tiles_n", "n_in", "n_out", "rank", "top_k", "flags")]


class _WeightsPtrs(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("scale", ctypes.c_void_p), ("zero", ctypes.c_void_p),
                ("A", ctypes.c_void_p), ("B", ctypes.c_void_p), ("sigma", ctypes.c_void_p)]


class _SharedPtrs(ctypes.Structure):
    _fields_ = [("us", ctypes.c_void_p * 3), ("v", ctypes.c_void_p * 3), ("phi", ctypes.c_void_p),
                ("sigma", ctypes.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is not built: run __graft_entry__.build() (there is no fallback path)")
        L = ctypes.CDLL(path)
        L.tq_init.restype = ctypes.c_int
        L.tq_init.argtypes = []
        L.tq_status_str.restype = ctypes.c_char_p
        L.tq_status_str.argtypes = [ctypes.c_int]
        L.tq_packed_size.restype = ctypes.c_size_t
        L.tq_packed_size.argtypes = [ctypes.POINTER(LayerDesc)]
        L.tq_moe_workspace_size.restype = ctypes.c_size_t
        L.tq_moe_workspace_size.argtypes = [ctypes.POINTER(LayerDesc), ctypes.c_int32]
        L.tq_permute_workspace_size.restype = ctypes.c_size_t
        L.tq_permute_workspace_size.argtypes = [ctypes.c_int32] * 3
        L.tq_pack_weights.restype = ctypes.c_int
        L.tq_pack_weights.argtypes = [ctypes.POINTER(LayerDesc), ctypes.POINTER(_WeightsPtrs), ctypes.c_void_p,
                                      ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        L.tq_pack_weights_shared.restype = ctypes.c_int
        L.tq_pack_weights_shared.argtypes = [ctypes.POINTER(LayerDesc), ctypes.POINTER(_WeightsPtrs),
                                             ctypes.POINTER(_SharedPtrs), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                             ctypes.c_void_p]
        L.tq_unpack_weights.restype = ctypes.c_int
        L.tq_unpack_weights.argtypes = [ctypes.POINTER(LayerDesc), ctypes.c_void_p, ctypes.POINTER(_WeightsPtrs),
                                        ctypes.c_void_p]
        L.tq_route.restype = ctypes.c_int
        L.tq_route.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.tq_permute.restype = ctypes.c_int
        L.tq_permute.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                 ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                 ctypes.c_size_t, ctypes.c_void_p]
        L.tq_moe_forward.restype = ctypes.c_int
        L.tq_moe_forward.argtypes = [ctypes.POINTER(LayerDesc), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_size_t, ctypes.c_void_p]
        L.tq_route_moe_forward.restype = ctypes.c_int
        L.tq_route_moe_forward.argtypes = [ctypes.POINTER(LayerDesc), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.tq_moe_forward_static.restype = ctypes.c_int
        L.tq_moe_forward_static.argtypes = [ctypes.POINTER(LayerDesc), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_void_p]
        L.tq_sketch_workspace_size.restype = ctypes.c_size_t
        L.tq_sketch_workspace_size.argtypes = [ctypes.c_int64, ctypes.c_int64]
        L.tq_sketch_lowrank.restype = ctypes.c_int
        L.tq_sketch_lowrank.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_size_t, ctypes.c_void_p]
        L.tq_debug_issue_probe.restype = ctypes.c_int
        L.tq_debug_issue_probe.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.tq_debug_stream.restype = ctypes.c_int
        L.tq_debug_stream.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_void_p]
        L.tq_set_profile_events.restype = ctypes.c_int
        L.tq_set_profile_events.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32]
        L.tq_lotile_packed_size.restype = ctypes.c_size_t
        L.tq_lotile_packed_size.argtypes = [ctypes.POINTER(LoTileDesc)]
        L.tq_lotile_workspace_size.restype = ctypes.c_size_t
        L.tq_lotile_workspace_size.argtypes = [ctypes.POINTER(LoTileDesc), ctypes.c_int32]
        L.tq_lotile_pack.restype = ctypes.c_int
        L.tq_lotile_pack.argtypes = [ctypes.POINTER(LoTileDesc), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        L.tq_lotile_pack_fp8.restype = ctypes.c_int
        L.tq_lotile_pack_fp8.argtypes = [ctypes.POINTER(LoTileDesc), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                         ctypes.c_void_p]
        L.tq_lotile_forward.restype = ctypes.c_int
        L.tq_lotile_forward.argtypes = [ctypes.POINTER(LoTileDesc), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_size_t, ctypes.c_void_p]
        L.tq_lotile_grid.restype = ctypes.c_int
        L.tq_lotile_grid.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        L.tq_lotile_place.restype = ctypes.c_int
        L.tq_lotile_place.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        _lib = L
    return _lib


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    return t.data_ptr()


def _check(rc: int, where: str) -> None:
    if rc != TQ_OK:
        raise TqError(rc, where)


def make_desc(E, S, k, H, F, g, bits, r, act_dtype=TQ_ACT_BF16, flags=0, tiles_m=0, tiles_n=0) -> LayerDesc:
    return LayerDesc(E, S, k, H, F, g, bits, r, act_dtype, flags, tiles_m, tiles_n)


def tq_init() -> None:
    """Per-device set-up for the current device (optional, see include/tileq.h)."""
    _check(lib().tq_init(), "tq_init")


def tq_status_str(status: int) -> str:
    return lib().tq_status_str(status).decode()


def tq_packed_size(desc: LayerDesc) -> int:
    return int(lib().tq_packed_size(ctypes.byref(desc)))


def tq_moe_workspace_size(desc: LayerDesc, T: int) -> int:
    return int(lib().tq_moe_workspace_size(ctypes.byref(desc), T))


def tq_pack_weights(desc: LayerDesc, codes, scale, zero, A=None, B=None, packed=None, err_flag=None, sigma=None):
    """Canonical device tensors (uint8 codes, int16/uint16 fp16-bit scale/zero/A/B) -> packed uint8 blob.  With
    TQ_FLAG_FP8_FACTORS A and B are uint8 E4M3 codes and sigma the fp16-bit tensor [E+S, 3, r]."""
    n = tq_packed_size(desc)
    if n == 0:
        raise TqError(2, "tq_packed_size")
    if packed is None:
        packed = torch.empty(n, dtype=torch.uint8, device=codes.device)
    src = _WeightsPtrs(_ptr(codes), _ptr(scale), _ptr(zero), _ptr(A), _ptr(B), _ptr(sigma))
    rc = lib().tq_pack_weights(ctypes.byref(desc), ctypes.byref(src), _ptr(packed), packed.numel(),
                               _ptr(err_flag), _stream())
    _check(rc, "tq_pack_weights")
    return packed


def tq_pack_weights_shared(desc: LayerDesc, codes, scale, zero, us, v, phi, packed=None, err_flag=None, sigma=None):
    """As tq_pack_weights for shared 2D-tiled factors: us / v are 3-lists (gate, up, down) of fp16-bit tensors
    [M, K_p, r] / [N, r, N_p] (uint8 E4M3 codes with TQ_FLAG_FP8_FACTORS, then sigma is the fp16-bit tensor [3, r]),
    phi int32 [E+S, 2]."""
    n = tq_packed_size(desc)
    if n == 0:
        raise TqError(2, "tq_packed_size")
    if packed is None:
        packed = torch.empty(n, dtype=torch.uint8, device=codes.device)
    src = _WeightsPtrs(_ptr(codes), _ptr(scale), _ptr(zero), None, None, None)
    sh = _SharedPtrs((ctypes.c_void_p * 3)(*[_ptr(t) for t in us]), (ctypes.c_void_p * 3)(*[_ptr(t) for t in v]), _ptr(phi),
                     _ptr(sigma))
    rc = lib().tq_pack_weights_shared(ctypes.byref(desc), ctypes.byref(src), ctypes.byref(sh), _ptr(packed), packed.numel(),
                                      _ptr(err_flag), _stream())
    _check(rc, "tq_pack_weights_shared")
    return packed


def tq_unpack_weights(desc: LayerDesc, packed, codes, scale, zero, A=None, B=None, sigma=None) -> None:
    dst = _WeightsPtrs(_ptr(codes), _ptr(scale), _ptr(zero), _ptr(A), _ptr(B), _ptr(sigma))
    _check(lib().tq_unpack_weights(ctypes.byref(desc), _ptr(packed), ctypes.byref(dst), _stream()),
           "tq_unpack_weights")


def tq_route(logits, bias, k: int, topk_idx=None, topk_w=None):
    T, E = logits.shape
    if topk_idx is None:
        topk_idx = torch.empty((T, k), dtype=torch.int32, device=logits.device)
    if topk_w is None:
        topk_w = torch.empty((T, k), dtype=torch.float32, device=logits.device)
    _check(lib().tq_route(_ptr(logits), _ptr(bias), T, E, k, _ptr(topk_idx), _ptr(topk_w), _stream()), "tq_route")
    return topk_idx, topk_w


def tq_permute(topk_idx, E: int, err_flag=None):
    T, k = topk_idx.shape
    dev = topk_idx.device
    offsets = torch.empty(E + 1, dtype=torch.int32, device=dev)
    slot_of = torch.empty(T * k, dtype=torch.int32, device=dev)
    src_of = torch.empty(T * k, dtype=torch.int32, device=dev)
    nws = int(lib().tq_permute_workspace_size(T, E, k))
    ws = torch.empty(max(nws, 256), dtype=torch.uint8, device=dev)
    _check(lib().tq_permute(_ptr(topk_idx), T, E, k, _ptr(offsets), _ptr(slot_of), _ptr(src_of), _ptr(err_flag),
                            _ptr(ws), ws.numel(), _stream()), "tq_permute")
    return offsets, slot_of, src_of


def tq_moe_forward(desc: LayerDesc, packed, x, topk_idx, topk_w, y=None, workspace=None):
    T = x.shape[0]
    if y is None:
        y = torch.empty_like(x)
    if workspace is None:
        workspace = torch.empty(max(tq_moe_workspace_size(desc, T), 256), dtype=torch.uint8, device=x.device)
    _check(lib().tq_moe_forward(ctypes.byref(desc), _ptr(packed), _ptr(x), _ptr(topk_idx), _ptr(topk_w), T, _ptr(y),
                                _ptr(workspace), workspace.numel(), _stream()), "tq_moe_forward")
    return y


def tq_route_moe_forward(desc: LayerDesc, packed, x, logits, bias, topk_idx=None, topk_w=None, y=None, workspace=None):
    """tq_route + tq_moe_forward in one call; returns (y, topk_idx, topk_w)."""
    T = x.shape[0]
    if topk_idx is None:
        topk_idx = torch.empty((T, desc.top_k), dtype=torch.int32, device=x.device)
    if topk_w is None:
        topk_w = torch.empty((T, desc.top_k), dtype=torch.float32, device=x.device)
    if y is None:
        y = torch.empty_like(x)
    if workspace is None:
        workspace = torch.empty(max(tq_moe_workspace_size(desc, T), 256), dtype=torch.uint8, device=x.device)
    _check(lib().tq_route_moe_forward(ctypes.byref(desc), _ptr(packed), _ptr(x), _ptr(logits), _ptr(bias), T, _ptr(topk_idx),
                                      _ptr(topk_w), _ptr(y), _ptr(workspace), workspace.numel(), _stream()),
           "tq_route_moe_forward")
    return y, topk_idx, topk_w


TQ_STATIC_SCRATCH_MAX = 32 << 20


def tq_moe_forward_static(desc: LayerDesc, packed, x, topk_idx, topk_w, y, err_flag=None):
    """tq_moe_forward on the library's static scratch array: allocates nothing (y is the caller's)."""
    _check(lib().tq_moe_forward_static(ctypes.byref(desc), _ptr(packed), _ptr(x), _ptr(topk_idx), _ptr(topk_w),
                                       x.shape[0], _ptr(y), _ptr(err_flag), _stream()), "tq_moe_forward_static")
    return y


def tq_set_profile_events(events) -> None:
    """events: list of raw hipEvent_t handles (ints), or an empty list to switch stage events off."""
    n = len(events)
    arr = (ctypes.c_void_p * max(n, 1))(*events)
    _check(lib().tq_set_profile_events(arr, n), "tq_set_profile_events")


def tq_sketch_lowrank(W, r: int, it: int, sketch, workspace=None):
    """Rank-r sketch decomposition of the fp32 device matrix W [rows, cols] (OVERWRITTEN with the residual).
    sketch: fp32 [r, cols].  Returns (U [r, rows], sigma [r], V [r, cols])."""
    rows, cols = W.shape
    n = int(lib().tq_sketch_workspace_size(rows, cols))
    if n == 0:
        raise TqError(2, "tq_sketch_workspace_size")
    if workspace is None:
        workspace = torch.empty(n, dtype=torch.uint8, device=W.device)
    U = torch.empty((r, rows), dtype=torch.float32, device=W.device)
    sigma = torch.empty(r, dtype=torch.float32, device=W.device)
    V = torch.empty((r, cols), dtype=torch.float32, device=W.device)
    _check(lib().tq_sketch_lowrank(_ptr(W), rows, cols, r, it, _ptr(sketch), _ptr(U), _ptr(sigma), _ptr(V), _ptr(workspace),
                                   workspace.numel(), _stream()), "tq_sketch_lowrank")
    return U, sigma, V


def tq_debug_issue_probe(level: int, iters: int, scratch) -> None:
    """Measurement aid: see include/tileq.h.  scratch: uint8 device tensor of at least 4096 bytes."""
    _check(lib().tq_debug_issue_probe(level, iters, _ptr(scratch), scratch.numel() * scratch.element_size(), _stream()),
           "tq_debug_issue_probe")


def tq_debug_stream(src, dst, nbytes: int, mode: int) -> None:
    """Streaming copy (mode 0), read (mode 1) or non-temporal read (mode 2) of nbytes with 16-byte accesses: a
    measurement aid."""
    _check(lib().tq_debug_stream(_ptr(src), _ptr(dst), nbytes, mode, _stream()), "tq_debug_stream")


def make_lotile_desc(E, M, N, n_in, n_out, r, k, flags=0) -> LoTileDesc:
    return LoTileDesc(E, M, N, n_in, n_out, r, k, flags)


def tq_lotile_packed_size(desc: LoTileDesc) -> int:
    return int(lib().tq_lotile_packed_size(ctypes.byref(desc)))


def tq_lotile_workspace_size(desc: LoTileDesc, T: int) -> int:
    return int(lib().tq_lotile_workspace_size(ctypes.byref(desc), T))


def tq_lotile_pack(desc: LoTileDesc, us, v, phi, packed=None, err_flag=None):
    """us [M, in, r], v [N, r, out] (fp16 bit patterns, int16/uint16), phi int32 [E, 2] -> packed uint8 blob."""
    n = tq_lotile_packed_size(desc)
    if n == 0:
        raise TqError(2, "tq_lotile_packed_size")
    if packed is None:
        packed = torch.empty(n, dtype=torch.uint8, device=us.device)
    _check(lib().tq_lotile_pack(ctypes.byref(desc), _ptr(us), _ptr(v), _ptr(phi), _ptr(packed), packed.numel(),
                                _ptr(err_flag), _stream()), "tq_lotile_pack")
    return packed


def tq_lotile_pack_fp8(desc: LoTileDesc, u8, sigma, v8, phi, packed=None, err_flag=None):
    """u8 [M, in, r], v8 [N, r, out] fp8 E4M3 bytes (uint8), sigma [r] fp16 bit patterns -> packed uint8 blob."""
    n = tq_lotile_packed_size(desc)
    if n == 0:
        raise TqError(2, "tq_lotile_packed_size")
    if packed is None:
        packed = torch.empty(n, dtype=torch.uint8, device=u8.device)
    _check(lib().tq_lotile_pack_fp8(ctypes.byref(desc), _ptr(u8), _ptr(sigma), _ptr(v8), _ptr(phi), _ptr(packed),
                                    packed.numel(), _ptr(err_flag), _stream()), "tq_lotile_pack_fp8")
    return packed


def tq_lotile_forward(desc: LoTileDesc, packed, x, topk_idx, topk_w, y=None, workspace=None):
    T = x.shape[0]
    if y is None:
        y = torch.empty((T, desc.n_out), dtype=x.dtype, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(tq_lotile_workspace_size(desc, T), 256), dtype=torch.uint8, device=x.device)
    _check(lib().tq_lotile_forward(ctypes.byref(desc), _ptr(packed), _ptr(x), _ptr(topk_idx), _ptr(topk_w), T,
                                   _ptr(y), _ptr(workspace), workspace.numel(), _stream()), "tq_lotile_forward")
    return y


def tq_lotile_grid(n_experts: int):
    """Host-only helper: the near-square tile grid (M, N) for n_experts."""
    m, n = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().tq_lotile_grid(n_experts, ctypes.byref(m), ctypes.byref(n)), "tq_lotile_grid")
    return int(m.value), int(n.value)


def tq_lotile_place(ideal, tiles_m: int, tiles_n: int):
    """Host-only helper: greedy placement of experts on the M x N grid.  ideal: int32 numpy array [E, 2] (host)."""
    import numpy as np
    ideal = np.ascontiguousarray(ideal, dtype=np.int32)
    phi = np.empty_like(ideal)
    _check(lib().tq_lotile_place(ideal.ctypes.data_as(ctypes.c_void_p), ideal.shape[0], tiles_m, tiles_n,
                                 phi.ctypes.data_as(ctypes.c_void_p)), "tq_lotile_place")
    return phi

