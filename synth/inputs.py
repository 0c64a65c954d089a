"""Seeded synthetic inputs with the shapes and value distributions of the five benchmark layers.

Everything here is input manufacture: counter-based random draws (numpy Philox), bf16/fp16
rounding of the drawn values, and a plain round-to-nearest group quantiser that turns a random
fp32 weight matrix into (codes, scale, zero).  The forward pass itself (dequantisation,
projections, routing, packing) lives elsewhere, once in ``oracle/`` and once in the HIP library.

Canonical (unpacked) weight layout, expert-major, ``p`` in {0: gate, 1: up, 2: down}:

  codes  uint8  [E+S, 3, N*K]      one code per byte, row-major [N, K]
                                   (gate/up: N=F, K=H; down: N=H, K=F)
  scale  fp16   [E+S, 3, N*K/g]    row-major [N, K/g]
  zero   fp16   [E+S, 3, N*K/g]    row-major [N, K/g]
  A      fp16   [E+S, (2H+F)*r]    per expert: gate [H, r] | up [H, r] | down [F, r]
  B      fp16   [E+S, (2F+H)*r]    per expert: gate [r, F] | up [r, F] | down [r, H]

Experts 0..E-1 are routed, E..E+S-1 are the always-on shared experts.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Optional

import numpy as np

SEED_BASE = 0x71170000

# tensor ids that are mixed into the Philox key
_TID_X, _TID_LOGITS, _TID_ZIPF, _TID_WEIGHT, _TID_FACTOR, _TID_OUTLIER = 0, 1, 2, 3, 4, 5


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    cfg_id: int
    name: str
    E: int          # routed experts
    S: int          # always-on shared experts
    k: int          # top-k
    H: int          # hidden
    F: int          # expert FFN width
    T: int          # tokens
    g: int          # quantisation group size along the contraction dim
    r: int          # rank of the low-rank factors
    bits: int       # 4, or 3 (codes 0..7 stored in 4-bit slots); with dense: 3 or 2, stored densely
    outlier_frac: float = 0.0   # fraction of input channels drawn heavy-tailed (Student-t, df=3)
    zipf_s: float = 0.0         # expert bias -s*ln(rank) added to the router logits
    w_std: float = 0.02
    f_std: float = 0.01
    dense: bool = False         # codes stored at `bits` bits each (the packed format's dense layouts)

    @property
    def qmax(self) -> int:
        return (1 << self.bits) - 1

    @property
    def n_exp(self) -> int:
        return self.E + self.S

    @property
    def a_tot(self) -> int:
        return self.T * (self.k + self.S)

    def replace(self, **kw) -> "LayerConfig":
        return dataclasses.replace(self, **kw)


CONFIGS = {
    1: LayerConfig(1, "tiny", E=8, S=0, k=2, H=256, F=512, T=64, g=64, r=8, bits=4),
    2: LayerConfig(2, "mixtral_decode", E=8, S=0, k=2, H=4096, F=14336, T=16, g=128, r=32, bits=4,
                   outlier_frac=0.05),
    3: LayerConfig(3, "dsv2lite_prefill", E=64, S=2, k=6, H=2048, F=1408, T=4096, g=128, r=16, bits=4,
                   zipf_s=1.1),
    4: LayerConfig(4, "qwenmoe_mixed", E=60, S=0, k=4, H=2048, F=1408, T=1024, g=64, r=64, bits=3),
    5: LayerConfig(5, "large_finegrained", E=128, S=0, k=8, H=4096, F=1536, T=8192, g=128, r=32, bits=4,
                   zipf_s=1.1),
}


def _rng(cfg_id: int, tensor_id: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[SEED_BASE + 16 * cfg_id + tensor_id, sub]))


# ----------------------------------------------------------------------------- bf16 helpers
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even.  Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16, returned as fp32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


# ----------------------------------------------------------------------------- activations / router
def make_x(cfg: LayerConfig) -> np.ndarray:
    """Activations ~N(0,1), rounded to bf16, returned as fp32 [T, H] (exactly bf16-representable)."""
    x = _rng(cfg.cfg_id, _TID_X).standard_normal((cfg.T, cfg.H), dtype=np.float32)
    return bf16_round(x)


def make_logits(cfg: LayerConfig):
    """Router logits ~N(0,1) fp32 [T, E] and the optional Zipf expert bias fp32 [E] (or None)."""
    logits = _rng(cfg.cfg_id, _TID_LOGITS).standard_normal((cfg.T, cfg.E), dtype=np.float32)
    bias = None
    if cfg.zipf_s > 0.0:
        rank = _rng(cfg.cfg_id, _TID_ZIPF).permutation(cfg.E) + 1
        bias = (-cfg.zipf_s * np.log(rank.astype(np.float64))).astype(np.float32)
    return logits, bias


# ----------------------------------------------------------------------------- quantiser
def rtn_quantize(w: np.ndarray, g: int, qmax: int):
    """Asymmetric round-to-nearest group quantiser for a [N, K] fp32 matrix, groups along K.

    Per (row, group): lo=min(w,0), hi=max(w,0), scale=fp16((hi-lo)/qmax) (1 where that is 0),
    zero=fp16(clip(rint(-lo/scale), 0, qmax)), code=clip(rint(w/scale)+zero, 0, qmax);
    rint rounds half to even.  Returns (codes uint8 [N,K], scale fp16 [N,K/g], zero fp16 [N,K/g]).
    """
    N, K = w.shape
    assert K % g == 0
    wg = w.reshape(N, K // g, g)
    lo = np.minimum(wg.min(axis=-1), 0.0)
    hi = np.maximum(wg.max(axis=-1), 0.0)
    scale = ((hi - lo) / np.float32(qmax)).astype(np.float16)
    scale[scale == 0] = np.float16(1.0)
    sf = scale.astype(np.float32)
    zero = np.clip(np.rint(-lo / sf), 0, qmax).astype(np.float16)
    q = np.rint(wg / sf[..., None])
    q += zero.astype(np.float32)[..., None]
    np.clip(q, 0, qmax, out=q)
    return q.astype(np.uint8).reshape(N, K), scale, zero


def _outlier_channels(cfg: LayerConfig, p: int, K: int) -> Optional[np.ndarray]:
    """The heavy-tailed input channels of projection p: one seeded subset shared by all experts."""
    if cfg.outlier_frac <= 0.0:
        return None
    n = int(round(cfg.outlier_frac * K))
    if n == 0:
        return None
    return np.sort(_rng(cfg.cfg_id, _TID_OUTLIER, p).choice(K, size=n, replace=False))


def _gen_matrix(cfg: LayerConfig, e: int, p: int, N: int, K: int, cols: Optional[np.ndarray],
                codes_out: np.ndarray, scale_out: np.ndarray, zero_out: np.ndarray) -> None:
    rng = _rng(cfg.cfg_id, _TID_WEIGHT, 3 * e + p)
    rows_per_chunk = max(1, min(N, (1 << 22) // K))
    G = K // cfg.g
    for r0 in range(0, N, rows_per_chunk):
        r1 = min(N, r0 + rows_per_chunk)
        w = rng.standard_normal((r1 - r0, K), dtype=np.float32)
        w *= np.float32(cfg.w_std)
        if cols is not None:
            nz = rng.standard_normal((r1 - r0, cols.size), dtype=np.float32)
            chi = rng.chisquare(3.0, size=(r1 - r0, cols.size)).astype(np.float32)
            w[:, cols] = np.float32(cfg.w_std) * nz / np.sqrt(chi / np.float32(3.0))
        q, s, z = rtn_quantize(w, cfg.g, cfg.qmax)
        codes_out[r0 * K:r1 * K] = q.reshape(-1)
        scale_out[r0 * G:r1 * G] = s.view(np.uint16).reshape(-1)
        zero_out[r0 * G:r1 * G] = z.view(np.uint16).reshape(-1)


@dataclasses.dataclass
class Layer:
    cfg: LayerConfig
    codes: np.ndarray   # uint8  [E+S, 3, H*F]
    scale: np.ndarray   # uint16 (fp16 bits) [E+S, 3, H*F/g]
    zero: np.ndarray    # uint16 (fp16 bits) [E+S, 3, H*F/g]
    A: np.ndarray       # uint16 (fp16 bits) [E+S, (2H+F)*r]
    B: np.ndarray       # uint16 (fp16 bits) [E+S, (2F+H)*r]

    def shapes(self, p: int):
        """(N, K) of projection p."""
        c = self.cfg
        return (c.F, c.H) if p < 2 else (c.H, c.F)

    def a_offset(self, p: int) -> int:
        c = self.cfg
        return (0, c.H * c.r, 2 * c.H * c.r)[p]

    def b_offset(self, p: int) -> int:
        c = self.cfg
        return (0, c.F * c.r, 2 * c.F * c.r)[p]

    def codes_matrix(self, e: int, p: int) -> np.ndarray:
        N, K = self.shapes(p)
        return self.codes[e, p].reshape(N, K)

    def scale_matrix(self, e: int, p: int) -> np.ndarray:
        N, K = self.shapes(p)
        return self.scale[e, p].view(np.float16).reshape(N, K // self.cfg.g)

    def zero_matrix(self, e: int, p: int) -> np.ndarray:
        N, K = self.shapes(p)
        return self.zero[e, p].view(np.float16).reshape(N, K // self.cfg.g)

    def a_matrix(self, e: int, p: int) -> np.ndarray:
        N, K = self.shapes(p)
        o = self.a_offset(p)
        return self.A[e, o:o + K * self.cfg.r].view(np.float16).reshape(K, self.cfg.r)

    def b_matrix(self, e: int, p: int) -> np.ndarray:
        N, K = self.shapes(p)
        o = self.b_offset(p)
        return self.B[e, o:o + N * self.cfg.r].view(np.float16).reshape(self.cfg.r, N)


def make_layer(cfg: LayerConfig, workers: int = 8) -> Layer:
    """All expert weights of one layer: random fp32 weights -> RTN codes/scale/zero, random fp16 factors."""
    assert cfg.H % cfg.g == 0 and cfg.F % cfg.g == 0
    ne, HF = cfg.n_exp, cfg.H * cfg.F
    codes = np.empty((ne, 3, HF), dtype=np.uint8)
    scale = np.empty((ne, 3, HF // cfg.g), dtype=np.uint16)
    zero = np.empty((ne, 3, HF // cfg.g), dtype=np.uint16)
    A = np.empty((ne, (2 * cfg.H + cfg.F) * cfg.r), dtype=np.uint16)
    B = np.empty((ne, (2 * cfg.F + cfg.H) * cfg.r), dtype=np.uint16)
    cols = [_outlier_channels(cfg, p, cfg.H if p < 2 else cfg.F) for p in range(3)]

    def one(e: int) -> None:
        for p in range(3):
            N, K = (cfg.F, cfg.H) if p < 2 else (cfg.H, cfg.F)
            _gen_matrix(cfg, e, p, N, K, cols[p], codes[e, p], scale[e, p], zero[e, p])
        if cfg.r > 0:
            rng = _rng(cfg.cfg_id, _TID_FACTOR, e)
            a = rng.standard_normal(A.shape[1], dtype=np.float32) * np.float32(cfg.f_std)
            b = rng.standard_normal(B.shape[1], dtype=np.float32) * np.float32(cfg.f_std)
            A[e] = a.astype(np.float16).view(np.uint16)
            B[e] = b.astype(np.float16).view(np.uint16)

    if workers > 1 and ne > 1:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(one, range(ne)))
    else:
        for e in range(ne):
            one(e)
    return Layer(cfg, codes, scale, zero, A, B)


# ----------------------------------------------------------------------------- shared 2D-tiled factors
_TID_LOTILE = 11
_TID_SHARED_LAYER = 13


@dataclasses.dataclass
class SharedLayer:
    """A layer whose low-rank factors are shared over a 2D grid of tiles: codes / scale / zero as in Layer, and per
    projection p (gate, up, down) us[p] [M, K_p, r], v[p] [N, r, N_p] (fp16 bit patterns), phi [E+S, 2] -> (m, n)."""
    cfg: LayerConfig
    codes: np.ndarray
    scale: np.ndarray
    zero: np.ndarray
    us: list
    v: list
    phi: np.ndarray

    @property
    def M(self) -> int:
        return self.us[0].shape[0]

    @property
    def N(self) -> int:
        return self.v[0].shape[0]

    def expanded(self) -> "Layer":
        """The same layer with the factors copied out per expert (A_e = us[m(e)], B_e = v[n(e)]): array gathers only."""
        c = self.cfg
        m, n = self.phi[:, 0], self.phi[:, 1]
        A = np.concatenate([self.us[p][m].reshape(c.n_exp, -1) for p in range(3)], axis=1)
        B = np.concatenate([self.v[p][n].reshape(c.n_exp, -1) for p in range(3)], axis=1)
        return Layer(c, self.codes, self.scale, self.zero, np.ascontiguousarray(A), np.ascontiguousarray(B))


def make_shared_layer(cfg: LayerConfig, M: Optional[int] = None, N: Optional[int] = None, layer: Optional["Layer"] = None,
                      degenerate: bool = False, workers: int = 8) -> SharedLayer:
    """Codes as make_layer (or taken from `layer`), factors ~N(0, f_std) per tile on the near-square grid of the
    paper (M = round(sqrt(E+S)), N = ceil((E+S) / M)) unless given, phi a seeded permutation of the tiles (drawn
    with replacement when there are fewer tiles than experts).  degenerate: M = N = E+S, phi(e) = (e, e), and the
    factors of tile e are the per-expert factors of `layer` (the per-expert format as a special case)."""
    if layer is None:
        layer = make_layer(cfg, workers=workers)
    ne = cfg.n_exp
    dims = ((cfg.H, cfg.F), (cfg.H, cfg.F), (cfg.F, cfg.H))
    if degenerate:
        us = [np.stack([layer.a_matrix(e, p).view(np.uint16) for e in range(ne)]) for p in range(3)]
        v = [np.stack([layer.b_matrix(e, p).view(np.uint16) for e in range(ne)]) for p in range(3)]
        phi = np.stack([np.arange(ne), np.arange(ne)], axis=1).astype(np.int32)
        return SharedLayer(cfg, layer.codes, layer.scale, layer.zero, us, v, phi)
    if M is None or N is None:
        M, N = lotile_grid(ne)
    rng = _rng(cfg.cfg_id, _TID_SHARED_LAYER)
    us = [(rng.standard_normal((M, K, cfg.r), dtype=np.float32) * cfg.f_std).astype(np.float16).view(np.uint16) for K, _ in dims]
    v = [(rng.standard_normal((N, cfg.r, No), dtype=np.float32) * cfg.f_std).astype(np.float16).view(np.uint16) for _, No in dims]
    tiles = rng.permutation(M * N)[:ne] if M * N >= ne else rng.integers(0, M * N, ne)
    phi = np.stack([tiles // N, tiles % N], axis=1).astype(np.int32)
    return SharedLayer(cfg, layer.codes, layer.scale, layer.zero, us, v, phi)


_TID_FP8 = 15


@dataclasses.dataclass
class Fp8Layer:
    """A layer whose low-rank factors are fp8 E4M3 codes with an fp16 diagonal Sigma: A8 uint8 [E+S, (2H+F) r] and
    B8 uint8 [E+S, (2F+H) r] in the shapes of Layer.A / Layer.B, sigma uint16 (fp16 bits) [E+S, 3, r]."""
    cfg: LayerConfig
    codes: np.ndarray
    scale: np.ndarray
    zero: np.ndarray
    A8: np.ndarray
    B8: np.ndarray
    sigma: np.ndarray

    def a8_list(self):
        c = self.cfg
        o = (0, c.H * c.r, 2 * c.H * c.r, (2 * c.H + c.F) * c.r)
        return [np.ascontiguousarray(self.A8[:, o[p]:o[p + 1]]).reshape(c.n_exp, -1, c.r) for p in range(3)]

    def b8_list(self):
        c = self.cfg
        o = (0, c.F * c.r, 2 * c.F * c.r, (2 * c.F + c.H) * c.r)
        return [np.ascontiguousarray(self.B8[:, o[p]:o[p + 1]]).reshape(c.n_exp, c.r, -1) for p in range(3)]


def make_layer_fp8(cfg: LayerConfig, layer: Optional["Layer"] = None, sigma_pow2: bool = False, workers: int = 8) -> Fp8Layer:
    """Codes as make_layer (or taken from `layer`); factors: fp8 codes of N(0, 1) draws (unit scale, as the columns of a
    normalised factorisation are stored) and sigma = f_std^2 / (1 + rho / 4) per rank component, a decaying spectrum
    (sigma_pow2: rounded down to powers of two, so that fp8 * sigma is exact in fp16)."""
    assert cfg.r > 0
    if layer is None:
        layer = make_layer(cfg, workers=workers)
    rng = _rng(cfg.cfg_id, _TID_FP8)
    ne = cfg.n_exp
    A8 = fp8_e4m3_encode(rng.standard_normal((ne, (2 * cfg.H + cfg.F) * cfg.r), dtype=np.float32))
    B8 = fp8_e4m3_encode(rng.standard_normal((ne, (2 * cfg.F + cfg.H) * cfg.r), dtype=np.float32))
    sg = (cfg.f_std ** 2 / (1.0 + np.arange(cfg.r) / 4.0)) * (1.0 + 0.25 * rng.random((ne, 3, cfg.r)))
    if sigma_pow2:
        sg = 2.0 ** np.floor(np.log2(sg))
    return Fp8Layer(cfg, layer.codes, layer.scale, layer.zero, A8, B8, sg.astype(np.float16).view(np.uint16))


_TID_PLANTED = 14


def make_planted_experts(cfg_id: int, n_exp: int, K: int, Nout: int, M: int, N: int, r_true: int, noise: float = 0.02,
                         strength: float = 0.05, phi: Optional[np.ndarray] = None):
    """Expert matrices with a planted 2D-tiled structure, standing in for trained experts that resemble each other
    along rows and columns: W_e [K, Nout] fp32 = L_m(e) R_n(e) + noise * N(0, 1), with M left blocks L_m [K, r_true] and
    N right blocks R_n [r_true, Nout] ~ N(0, strength / sqrt(r_true)) and a seeded collision-free placement phi (needs
    M N >= n_exp), or the placement given.  Returns (W [n_exp, K, Nout], phi int32 [n_exp, 2])."""
    assert M * N >= n_exp
    rng = _rng(cfg_id, _TID_PLANTED)
    L = rng.standard_normal((M, K, r_true), dtype=np.float32) * np.float32(np.sqrt(strength / np.sqrt(r_true)))
    R = rng.standard_normal((N, r_true, Nout), dtype=np.float32) * np.float32(np.sqrt(strength / np.sqrt(r_true)))
    tiles = rng.permutation(M * N)[:n_exp]
    if phi is None:
        phi = np.stack([tiles // N, tiles % N], axis=1).astype(np.int32)
    W = np.stack([L[phi[e, 0]] @ R[phi[e, 1]] for e in range(n_exp)])
    W += rng.standard_normal(W.shape, dtype=np.float32) * np.float32(noise)
    return W.astype(np.float32), phi


def tile_matrix(W: np.ndarray, phi: np.ndarray, M: int, N: int) -> np.ndarray:
    """Experts W [n_exp, K, Nout] placed on the M x N grid by phi (the tiled matrix of Eq. 11; empty cells are zero)."""
    n_exp, K, Nout = W.shape
    big = np.zeros((M * K, N * Nout), dtype=np.float32)
    for e in range(n_exp):
        m, n = int(phi[e, 0]), int(phi[e, 1])
        big[m * K:(m + 1) * K, n * Nout:(n + 1) * Nout] = W[e]
    return big


def lotile_grid(E: int):
    """The paper's near-square tile grid for E experts: M = round(sqrt(E)), N = ceil(E / M)."""
    M = max(1, int(round(float(np.sqrt(E)))))
    N = (E + M - 1) // M
    return M, N


def make_lotile(cfg: LayerConfig, n_in: int, n_out: int, M: Optional[int] = None, N: Optional[int] = None):
    """Shared factors for one linear map of a layer shaped like `cfg`: us [M, n_in, r] and v [N, r, n_out] as fp16
    bit patterns (values ~N(0, f_std)), and a placement phi [E, 2] that puts every expert on its own tile of the
    M x N grid (a seeded permutation of the tiles); with fewer tiles than experts the placement draws tiles with
    replacement, so experts share them.  Inputs only: no forward arithmetic."""
    if M is None or N is None:
        M, N = lotile_grid(cfg.E)
    rng = _rng(cfg.cfg_id, _TID_LOTILE)
    us = (rng.standard_normal((M, n_in, cfg.r), dtype=np.float32) * cfg.f_std).astype(np.float16).view(np.uint16)
    v = (rng.standard_normal((N, cfg.r, n_out), dtype=np.float32) * cfg.f_std).astype(np.float16).view(np.uint16)
    tiles = rng.permutation(M * N)[:cfg.E] if M * N >= cfg.E else rng.integers(0, M * N, cfg.E)
    phi = np.stack([tiles // N, tiles % N], axis=1).astype(np.int32)
    return us, v, phi


def fp8_e4m3_encode(a: np.ndarray) -> np.ndarray:
    """fp32 -> fp8 E4M3 bytes (round to nearest even; the library conversion of torch on the CPU).  Input
    generation only."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def make_lotile_fp8(cfg: LayerConfig, n_in: int, n_out: int, M: Optional[int] = None, N: Optional[int] = None):
    """Mixed-precision shared factors: u8 [M, n_in, r] and v8 [N, r, n_out] fp8 E4M3 bytes of N(0, 1) draws (unit
    scale, as the columns of a normalised factorisation would be stored), sigma [r] fp16 bit patterns carrying the
    magnitude (f_std^2 / (1 + rho / 4): a decaying spectrum), and phi as make_lotile."""
    if M is None or N is None:
        M, N = lotile_grid(cfg.E)
    rng = _rng(cfg.cfg_id, _TID_LOTILE + 1)
    u8 = fp8_e4m3_encode(rng.standard_normal((M, n_in, cfg.r), dtype=np.float32))
    v8 = fp8_e4m3_encode(rng.standard_normal((N, cfg.r, n_out), dtype=np.float32))
    sigma = (cfg.f_std ** 2 / (1.0 + np.arange(cfg.r) / 4.0)).astype(np.float16).view(np.uint16)
    tiles = rng.permutation(M * N)[:cfg.E] if M * N >= cfg.E else rng.integers(0, M * N, cfg.E)
    phi = np.stack([tiles // N, tiles % N], axis=1).astype(np.int32)
    return u8, sigma, v8, phi
