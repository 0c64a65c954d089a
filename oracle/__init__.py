"""ctypes front end of the CPU oracle (``tileq_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
cpu_baseline leg.  The product package never imports this module and shares no code with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "tileq_oracle.c")
_LIB = os.path.join(_DIR, "libtileq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


class OrcLayer(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_experts", "n_shared", "top_k", "hidden", "ffn", "group", "bits", "rank")]


class OrcWeights(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("scale", ctypes.c_void_p), ("zero", ctypes.c_void_p),
                ("A", ctypes.c_void_p), ("B", ctypes.c_void_p)]


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.orc_half_to_double.restype = ctypes.c_double
        L.orc_half_to_double.argtypes = [ctypes.c_uint16]
        L.orc_silu_export.restype = ctypes.c_double
        L.orc_silu_export.argtypes = [ctypes.c_double]
        L.orc_moe_forward.restype = ctypes.c_int32
        L.orc_num_threads.restype = ctypes.c_int32
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_num_threads(n: int) -> None:
    lib().orc_set_num_threads(ctypes.c_int32(n))


def half_to_double(bits: int) -> float:
    return float(lib().orc_half_to_double(ctypes.c_uint16(bits)))


def silu(v: float) -> float:
    return float(lib().orc_silu_export(ctypes.c_double(v)))


def route(logits: np.ndarray, bias: Optional[np.ndarray], k: int):
    """Top-k routing.  Returns (idx int32 [T,k], w fp32 [T,k])."""
    logits = _c(logits, np.float32)
    T, E = logits.shape
    b = None if bias is None else _c(bias, np.float32)
    idx = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float32)
    lib().orc_route(_p(logits), _p(b), ctypes.c_int32(T), ctypes.c_int32(E), ctypes.c_int32(k),
                    _p(idx), _p(w))
    return idx, w


def permute(idx: np.ndarray, E: int):
    """Returns (offsets int32 [E+1], slot_of int32 [T*k], src_of int32 [T*k])."""
    idx = _c(idx, np.int32)
    T, k = idx.shape
    offsets = np.empty(E + 1, dtype=np.int32)
    slot_of = np.empty(T * k, dtype=np.int32)
    src_of = np.empty(T * k, dtype=np.int32)
    lib().orc_permute(_p(idx), ctypes.c_int32(T), ctypes.c_int32(E), ctypes.c_int32(k),
                      _p(offsets), _p(slot_of), _p(src_of))
    return offsets, slot_of, src_of


def dequant(codes: np.ndarray, scale_bits: np.ndarray, zero_bits: np.ndarray, g: int) -> np.ndarray:
    """codes uint8 [N,K], scale/zero fp16 bit patterns [N,K/g] -> float64 [N,K]."""
    codes = _c(codes, np.uint8)
    N, K = codes.shape
    s = _c(scale_bits, np.uint16)
    z = _c(zero_bits, np.uint16)
    assert s.size == N * (K // g) and z.size == s.size
    W = np.empty((N, K), dtype=np.float64)
    lib().orc_dequant(_p(codes), _p(s), _p(z), ctypes.c_int32(N), ctypes.c_int32(K), ctypes.c_int32(g), _p(W))
    return W


def project(v: np.ndarray, codes: np.ndarray, scale_bits: np.ndarray, zero_bits: np.ndarray,
            A_bits: Optional[np.ndarray], B_bits: Optional[np.ndarray], g: int) -> np.ndarray:
    """One projection of one vector: v [K] float64 -> [N] float64.  A [K,r], B [r,N] fp16 bits or None."""
    codes = _c(codes, np.uint8)
    N, K = codes.shape
    v = _c(v, np.float64)
    assert v.shape == (K,)
    s = _c(scale_bits, np.uint16)
    z = _c(zero_bits, np.uint16)
    r = 0
    A = B = None
    if A_bits is not None and A_bits.size:
        A = _c(A_bits, np.uint16)
        B = _c(B_bits, np.uint16)
        r = A.size // K
        assert A.size == K * r and B.size == r * N
    out = np.empty(N, dtype=np.float64)
    lib().orc_project(_p(v), _p(codes), _p(s), _p(z), _p(A), _p(B), ctypes.c_int32(N), ctypes.c_int32(K),
                      ctypes.c_int32(g), ctypes.c_int32(r), _p(out))
    return out


def moe_forward(E: int, S: int, k: int, H: int, F: int, g: int, bits: int, r: int,
                codes: np.ndarray, scale: np.ndarray, zero: np.ndarray,
                A: Optional[np.ndarray], B: Optional[np.ndarray],
                x: np.ndarray, idx: np.ndarray, w: np.ndarray,
                tokens: Optional[np.ndarray] = None) -> np.ndarray:
    """The whole layer on canonical weight arrays.  x fp32 [T,H]; returns float64 [n_tokens, H]."""
    x = _c(x, np.float32)
    T = x.shape[0]
    assert x.shape == (T, H)
    idx = _c(idx, np.int32)
    w = _c(w, np.float32)
    assert idx.shape == (T, k) and w.shape == (T, k)
    ne, HF = E + S, H * F
    codes = _c(codes, np.uint8)
    scale = _c(scale, np.uint16)
    zero = _c(zero, np.uint16)
    assert codes.size == ne * 3 * HF and scale.size == ne * 3 * HF // g and zero.size == scale.size
    if r > 0:
        A = _c(A, np.uint16)
        B = _c(B, np.uint16)
        assert A.size == ne * (2 * H + F) * r and B.size == ne * (2 * F + H) * r
    else:
        A = B = None
    tok = None if tokens is None else _c(tokens, np.int32)
    n = T if tok is None else tok.size
    y = np.empty((n, H), dtype=np.float64)
    L = OrcLayer(E, S, k, H, F, g, bits, r)
    Wt = OrcWeights(_p(codes), _p(scale), _p(zero), _p(A), _p(B))
    rc = lib().orc_moe_forward(ctypes.byref(L), ctypes.byref(Wt), _p(x), _p(idx), _p(w), ctypes.c_int32(T),
                               _p(tok), ctypes.c_int32(n), _p(y))
    if rc != 0:
        raise ValueError("oracle: expert or token index out of range")
    return y


def moe_forward_layer(layer, x: np.ndarray, idx: np.ndarray, w: np.ndarray,
                      tokens: Optional[np.ndarray] = None) -> np.ndarray:
    """Convenience wrapper over an object with .cfg (E,S,k,H,F,g,bits,r) and canonical arrays."""
    c = layer.cfg
    return moe_forward(c.E, c.S, c.k, c.H, c.F, c.g, c.bits, c.r, layer.codes, layer.scale, layer.zero,
                       layer.A if c.r else None, layer.B if c.r else None, x, idx, w, tokens)


class OrcShared(ctypes.Structure):
    _fields_ = [("us", ctypes.c_void_p * 3), ("v", ctypes.c_void_p * 3), ("phi", ctypes.c_void_p),
                ("M", ctypes.c_int32), ("N", ctypes.c_int32)]


def moe_forward_shared(slayer, x: np.ndarray, idx: np.ndarray, w: np.ndarray,
                       tokens: Optional[np.ndarray] = None) -> np.ndarray:
    """The layer on shared 2D-tiled factors.  slayer: object with .cfg, canonical .codes/.scale/.zero, .us / .v
    (3-lists of fp16-bit arrays [M, K_p, r] / [N, r, N_p]) and .phi int32 [E+S, 2].  Returns float64 [n_tokens, H]."""
    c = slayer.cfg
    x = _c(x, np.float32)
    T = x.shape[0]
    idx = _c(idx, np.int32)
    w = _c(w, np.float32)
    assert x.shape == (T, c.H) and idx.shape == (T, c.k) and w.shape == (T, c.k) and c.r > 0
    codes, scale, zero = _c(slayer.codes, np.uint8), _c(slayer.scale, np.uint16), _c(slayer.zero, np.uint16)
    us = [_c(a, np.uint16) for a in slayer.us]
    v = [_c(a, np.uint16) for a in slayer.v]
    phi = _c(slayer.phi, np.int32)
    M, N = us[0].shape[0], v[0].shape[0]
    for p, (K, Nout) in enumerate(((c.H, c.F), (c.H, c.F), (c.F, c.H))):
        assert us[p].shape == (M, K, c.r) and v[p].shape == (N, c.r, Nout)
    assert phi.shape == (c.E + c.S, 2)
    tok = None if tokens is None else _c(tokens, np.int32)
    n = T if tok is None else tok.size
    y = np.empty((n, c.H), dtype=np.float64)
    L = OrcLayer(c.E, c.S, c.k, c.H, c.F, c.g, c.bits, c.r)
    Wt = OrcWeights(_p(codes), _p(scale), _p(zero), None, None)
    Sh = OrcShared((ctypes.c_void_p * 3)(*[a.ctypes.data for a in us]), (ctypes.c_void_p * 3)(*[a.ctypes.data for a in v]),
                   _p(phi), M, N)
    lb = lib()
    lb.orc_moe_forward_shared.restype = ctypes.c_int32
    rc = lb.orc_moe_forward_shared(ctypes.byref(L), ctypes.byref(Wt), ctypes.byref(Sh), _p(x), _p(idx), _p(w),
                                   ctypes.c_int32(T), _p(tok), ctypes.c_int32(n), _p(y))
    if rc != 0:
        raise ValueError("oracle: expert, token or tile index out of range")
    return y


def moe_forward_fp8(cfg, codes, scale, zero, a8, b8, sigma, x, idx, w, phi=None, tokens=None) -> np.ndarray:
    """The layer with fp8 E4M3 factors and an fp16 Sigma.  a8 / b8: 3-lists (gate, up, down) of uint8 arrays
    [nA, K_p, r] / [nB, r, N_p].  phi None: per-expert factors (nA = nB = E+S, sigma fp16 bits [E+S, 3, r]);
    phi int32 [E+S, 2]: shared tiled factors (sigma [3, r]).  Returns float64 [n_tokens, H]."""
    c = cfg
    x = _c(x, np.float32)
    T = x.shape[0]
    idx = _c(idx, np.int32)
    w = _c(w, np.float32)
    codes, scale, zero = _c(codes, np.uint8), _c(scale, np.uint16), _c(zero, np.uint16)
    a8 = [_c(a, np.uint8) for a in a8]
    b8 = [_c(b, np.uint8) for b in b8]
    sigma = _c(sigma, np.uint16)
    dims = ((c.H, c.F), (c.H, c.F), (c.F, c.H))
    nA, nB = a8[0].shape[0], b8[0].shape[0]
    for p, (K, No) in enumerate(dims):
        assert a8[p].shape == (nA, K, c.r) and b8[p].shape == (nB, c.r, No)
    if phi is None:
        assert nA == nB == c.E + c.S and sigma.shape == (c.E + c.S, 3, c.r)
    else:
        phi = _c(phi, np.int32)
        assert phi.shape == (c.E + c.S, 2) and sigma.shape == (3, c.r)
    tok = None if tokens is None else _c(tokens, np.int32)
    n = T if tok is None else tok.size
    y = np.empty((n, c.H), dtype=np.float64)
    L = OrcLayer(c.E, c.S, c.k, c.H, c.F, c.g, c.bits, c.r)
    pa = (ctypes.c_void_p * 3)(*[a.ctypes.data for a in a8])
    pb = (ctypes.c_void_p * 3)(*[b.ctypes.data for b in b8])
    lb = lib()
    lb.orc_moe_forward_fp8.restype = ctypes.c_int32
    rc = lb.orc_moe_forward_fp8(ctypes.byref(L), _p(codes), _p(scale), _p(zero), pa, pb, _p(sigma), _p(phi),
                                ctypes.c_int32(nA), ctypes.c_int32(nB), _p(x), _p(idx), _p(w), ctypes.c_int32(T), _p(tok),
                                ctypes.c_int32(n), _p(y))
    if rc != 0:
        raise ValueError("oracle: expert, token or tile index out of range")
    return y


def lotile_forward(x: np.ndarray, us_bits: np.ndarray, v_bits: np.ndarray, phi: np.ndarray,
                   idx: np.ndarray, w: np.ndarray) -> np.ndarray:
    """LoTileMoE of Section 3.2 (three-dimensional accumulator form).  x [T, in] fp32; us_bits [M, in, r] and
    v_bits [N, r, out] fp16 bit patterns; phi [E, 2] int32; idx, w [T, k].  Returns y [T, out] fp64."""
    L = lib()
    if not getattr(L, "_lotile_ready", False):
        L.orc_lotile_forward.restype = None
        L.orc_lotile_forward.argtypes = [ctypes.c_int32] * 7 + [ctypes.c_void_p] * 7
        L._lotile_ready = True
    x = _c(x, np.float32)
    us_bits = _c(us_bits, np.uint16)
    v_bits = _c(v_bits, np.uint16)
    phi = _c(phi, np.int32)
    idx = _c(idx, np.int32)
    w = _c(w, np.float32)
    T, n_in = x.shape
    M, _, r = us_bits.shape
    N, _, n_out = v_bits.shape
    k = idx.shape[1]
    y = np.zeros((T, n_out), dtype=np.float64)
    L.orc_lotile_forward(T, n_in, n_out, M, N, r, k, _p(x), _p(us_bits), _p(v_bits), _p(phi), _p(idx), _p(w), _p(y))
    return y


def fp8_e4m3_to_double(bits: int) -> float:
    L = lib()
    L.orc_fp8_e4m3_to_double.restype = ctypes.c_double
    L.orc_fp8_e4m3_to_double.argtypes = [ctypes.c_uint8]
    return float(L.orc_fp8_e4m3_to_double(ctypes.c_uint8(bits)))


def lotile_forward_fp8(x: np.ndarray, u8: np.ndarray, sigma_bits: np.ndarray, v8: np.ndarray, phi: np.ndarray,
                       idx: np.ndarray, w: np.ndarray) -> np.ndarray:
    """LoTileMoE on mixed-precision factors (end of Section 3.1): u8 [M, in, r] and v8 [N, r, out] fp8 E4M3 bytes,
    sigma_bits [r] fp16 bit patterns.  Returns y [T, out] fp64."""
    L = lib()
    if not getattr(L, "_lotile_fp8_ready", False):
        L.orc_lotile_forward_fp8.restype = None
        L.orc_lotile_forward_fp8.argtypes = [ctypes.c_int32] * 7 + [ctypes.c_void_p] * 8
        L._lotile_fp8_ready = True
    x = _c(x, np.float32)
    u8 = _c(u8, np.uint8)
    v8 = _c(v8, np.uint8)
    sigma_bits = _c(sigma_bits, np.uint16)
    phi = _c(phi, np.int32)
    idx = _c(idx, np.int32)
    w = _c(w, np.float32)
    T, n_in = x.shape
    M, _, r = u8.shape
    N, _, n_out = v8.shape
    assert sigma_bits.shape == (r,)
    k = idx.shape[1]
    y = np.zeros((T, n_out), dtype=np.float64)
    L.orc_lotile_forward_fp8(T, n_in, n_out, M, N, r, k, _p(x), _p(u8), _p(sigma_bits), _p(v8), _p(phi), _p(idx), _p(w),
                             _p(y))
    return y
