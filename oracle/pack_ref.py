"""Independent packer for the library's weight blob, written from the layout prose in
``include/tileq.h`` with numpy reshapes/transposes (no code shared with the HIP packer).

TEST INFRASTRUCTURE ONLY: used to check tq_pack_weights byte for byte.
Returns the blob body (everything after the 256-byte header).
"""
from __future__ import annotations

import numpy as np


def _bf16_rne(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bits, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def _zero_coeff_parts(scale_bits: np.ndarray, zero_bits: np.ndarray, g16: int):
    """[N, G] fp16 bit patterns -> (hi, lo) bf16 bit patterns [N, 16*g16] of c = -scale * (128 + zero),
    evaluated in fp32 as the header specifies; groups beyond G are zero."""
    s = scale_bits.view(np.float16).astype(np.float32)
    z = zero_bits.view(np.float16).astype(np.float32)
    c = (-s) * (np.float32(128.0) + z)
    hi = _bf16_rne(c)
    hi_f = (hi.astype(np.uint32) << 16).view(np.float32)
    lo = _bf16_rne(c - hi_f)
    N, G = s.shape
    out_hi = np.zeros((N, 16 * g16), dtype=np.uint16)
    out_lo = np.zeros_like(out_hi)
    out_hi[:, :G] = hi
    out_lo[:, :G] = lo
    return out_hi, out_lo


def _zc_part(hi: np.ndarray, lo: np.ndarray) -> np.ndarray:
    """[N, 16*g16] -> [N, g16 (block), 2 (which), 2 (hf), 8 (i)]: which 0 = hi, which 1 = lo."""
    N = hi.shape[0]
    h = hi.reshape(N, -1, 2, 8)
    l = lo.reshape(N, -1, 2, 8)
    return np.stack([h, l], axis=2)


_NIBBLE_POS = [(i // 2) + 4 * (i % 2) for i in range(8)]


def _words(codes_nk: np.ndarray) -> np.ndarray:
    """[N, K] codes -> [N, K/64 (chunk), 4 (word), 2 (hf)] uint32 words of 8 codes each."""
    N, K = codes_nk.shape
    c = codes_nk.reshape(N, K // 64, 4, 2, 8).astype(np.uint32) & 15
    out = np.zeros(c.shape[:-1], dtype=np.uint32)
    for i in range(8):
        out |= c[..., i] << np.uint32(4 * _NIBBLE_POS[i])
    return out


def _dense_words(codes_nk: np.ndarray, bits: int) -> np.ndarray:
    """[N, K] codes -> [N, K/64 (chunk), bits (word), 2 (hf)] uint32: the dense 2- / 3-bit layout.  Slot P = 4 w + j of a
    (lane, chunk) holds lo = q[w][2j] and hi = q[w][2j+1] sixteen bit positions apart."""
    N, K = codes_nk.shape
    fm = (1 << bits) - 1
    c = codes_nk.reshape(N, K // 64, 4, 2, 4, 2).astype(np.uint32) & fm       # [n, chunk, w, hf, j, lo/hi]
    slot = c[..., 0] | (c[..., 1] << np.uint32(16))                             # [n, chunk, w, hf, j]
    slot = slot.transpose(0, 1, 3, 2, 4).reshape(N, K // 64, 2, 16)             # [n, chunk, hf, P]
    out = np.zeros((N, K // 64, 2, bits), dtype=np.uint32)                      # [n, chunk, hf, word]
    if bits == 2:
        for P in range(16):
            out[..., P // 8] |= slot[..., P] << np.uint32(2 * (P % 8))
    else:
        for P in range(15):
            out[..., P // 5] |= slot[..., P] << np.uint32(3 * (P % 5))
        last = slot[..., 15]
        for b in range(3):
            out[..., b] |= (((last >> np.uint32(b)) & 1) << np.uint32(15)) | (((last >> np.uint32(16 + b)) & 1) << np.uint32(31))
    return out.transpose(0, 1, 3, 2)                                            # [n, chunk, word, hf]


def _pad_rows(a: np.ndarray, rows: int) -> np.ndarray:
    if a.shape[0] == rows:
        return a
    out = np.zeros((rows,) + a.shape[1:], dtype=a.dtype)
    out[:a.shape[0]] = a
    return out


def _pad_cols(a: np.ndarray, cols: int) -> np.ndarray:
    if a.shape[1] == cols:
        return a
    out = np.zeros((a.shape[0], cols), dtype=a.dtype)
    out[:, :a.shape[1]] = a
    return out


def _bfrag_gu(B0, B1, r16, pairs) -> bytes:
    """Right factors of gate and up, [r, F] each -> [pairs, step, tile, hf, col, i]."""
    b = np.stack([_pad_rows(Bp, r16).reshape(r16 // 16, 2, 8, pairs, 32) for Bp in (B0, B1)], axis=0)
    # [tile, step, hf, i, pairs, col] -> [pairs, step, tile, hf, col, i]
    return np.ascontiguousarray(b.transpose(4, 1, 0, 2, 5, 3)).tobytes()


def _afrag_gu(A0, A1, r16, K) -> bytes:
    """Left factors of gate and up, [H, r] each, side by side -> [ta, step, hf, col, i]."""
    acat = np.concatenate([_pad_cols(A0, r16), _pad_cols(A1, r16)], axis=1)   # [K, 2*r16]
    nat = (2 * r16 + 31) // 32
    acat = _pad_cols(acat, 32 * nat).reshape(K // 16, 2, 8, nat, 32)
    # [step, hf, i, ta, col] -> [ta, step, hf, col, i]
    return np.ascontiguousarray(acat.transpose(3, 0, 1, 4, 2)).tobytes()


def _bfrag_d(B2, r16, pairs) -> bytes:
    b = _pad_rows(B2, r16).reshape(r16 // 16, 2, 8, pairs, 2, 32)
    # [step, hf, i, pairs, tile, col] -> [pairs, step, tile, hf, col, i]
    return np.ascontiguousarray(b.transpose(3, 0, 4, 1, 5, 2)).tobytes()


def _afrag_d(A2, r16, K) -> bytes:
    nat = (r16 + 31) // 32
    a = _pad_cols(_pad_cols(A2, r16), 32 * nat).reshape(K // 16, 2, 8, nat, 32)
    return np.ascontiguousarray(a.transpose(3, 0, 1, 4, 2)).tobytes()


def _sig_part(sig_list, r16) -> bytes:
    """fp16 bit patterns [r] per projection -> fp32 [len(sig_list) * r16] (zero beyond r), padded to 256 bytes."""
    out = np.zeros((len(sig_list), r16), dtype=np.float32)
    for i, sg in enumerate(sig_list):
        out[i, :sg.size] = np.asarray(sg, dtype=np.uint16).view(np.float16).astype(np.float32)
    b = out.tobytes()
    return b + b"\0" * ((-len(b)) % 256)


def pack_expert(codes3, scale3, zero3, A3, B3, H, F, g, r, dense_bits=0, factors=True, sigma3=None) -> bytes:
    """codes3[p]: [N,K] uint8; scale3/zero3[p]: [N,K/g] uint16; A3[p]: [K,r] uint16; B3[p]: [r,N] uint16.
    dense_bits: 0 = codes in 4-bit slots; 2 or 3 = the dense layouts (no zc part).  factors=False: a record of the
    shared-factor format (no bfrag / afrag parts).  sigma3 (fp16 bits [r] per projection): fp8 factors, A3 / B3 are
    then uint8 E4M3 codes in the same layouts with 1-byte elements, followed by the fp32 sig part."""
    r16 = (r + 15) // 16 * 16
    parts = []

    def section(is_d: bool):
        if not is_d:
            K, pairs = H, F // 32
            # codes: [pairs, chunks, tile, hf, col, word]
            if dense_bits:
                w = np.stack([_dense_words(codes3[p], dense_bits).reshape(pairs, 32, K // 64, dense_bits, 2) for p in (0, 1)], axis=0)
                # [tile, pairs, col, chunk, word, hf] -> [pairs, chunk, tile, word, hf, col]
                parts.append(np.ascontiguousarray(w.transpose(1, 3, 0, 4, 5, 2)).tobytes())
            else:
                w = np.stack([_words(codes3[p]).reshape(pairs, 32, K // 64, 4, 2) for p in (0, 1)], axis=0)
                # w: [tile, pairs, col, chunk, word, hf] -> [pairs, chunk, tile, hf, col, word]
                parts.append(np.ascontiguousarray(w.transpose(1, 3, 0, 5, 2, 4)).tobytes())
            sz = np.stack([(scale3[p].astype(np.uint32) | (zero3[p].astype(np.uint32) << 16)).reshape(pairs, 32, K // g)
                           for p in (0, 1)], axis=0)          # [tile, pairs, col, G]
            parts.append(np.ascontiguousarray(sz.transpose(1, 3, 0, 2)).tobytes())
            g16 = (K // g + 15) // 16
            if not dense_bits:
                zc = np.stack([_zc_part(*_zero_coeff_parts(scale3[p], zero3[p], g16)).reshape(pairs, 32, g16, 2, 2, 8)
                               for p in (0, 1)], axis=0)
                # [tile, pairs, col, block, which, hf, i] -> [pairs, fragment = 2*block + which, tile, hf, col, i]
                parts.append(np.ascontiguousarray(zc.transpose(1, 3, 4, 0, 5, 2, 6)).tobytes())
            if r > 0 and factors:
                parts.append(_bfrag_gu(B3[0], B3[1], r16, pairs))
                parts.append(_afrag_gu(A3[0], A3[1], r16, K))
                if sigma3 is not None:
                    parts.append(_sig_part([sigma3[0], sigma3[1]], r16))
        else:
            K, pairs = F, H // 64
            if dense_bits:
                w = _dense_words(codes3[2], dense_bits).reshape(pairs, 2, 32, K // 64, dense_bits, 2)
                # [pairs, tile, col, chunk, word, hf] -> [pairs, chunk, tile, word, hf, col]
                parts.append(np.ascontiguousarray(w.transpose(0, 3, 1, 4, 5, 2)).tobytes())
            else:
                w = _words(codes3[2]).reshape(pairs, 2, 32, K // 64, 4, 2)
                # [pairs, tile, col, chunk, word, hf] -> [pairs, chunk, tile, hf, col, word]
                parts.append(np.ascontiguousarray(w.transpose(0, 3, 1, 5, 2, 4)).tobytes())
            sz = (scale3[2].astype(np.uint32) | (zero3[2].astype(np.uint32) << 16)).reshape(pairs, 2, 32, K // g)
            parts.append(np.ascontiguousarray(sz.transpose(0, 3, 1, 2)).tobytes())
            g16 = (K // g + 15) // 16
            if not dense_bits:
                zc = _zc_part(*_zero_coeff_parts(scale3[2], zero3[2], g16)).reshape(pairs, 2, 32, g16, 2, 2, 8)
                # [pairs, tile, col, block, which, hf, i] -> [pairs, step, tile, hf, col, i]
                parts.append(np.ascontiguousarray(zc.transpose(0, 3, 4, 1, 5, 2, 6)).tobytes())
            if r > 0 and factors:
                parts.append(_bfrag_d(B3[2], r16, pairs))
                parts.append(_afrag_d(A3[2], r16, K))
                if sigma3 is not None:
                    parts.append(_sig_part([sigma3[2]], r16))

    section(False)
    section(True)
    body = b"".join(parts)
    pad = (-len(body)) % 256
    return body + b"\0" * pad


def pack_layer(layer) -> np.ndarray:
    """Blob body (after the 256-byte header) for a synth.Layer-like object, as a uint8 array."""
    c = layer.cfg
    out = []
    for e in range(c.E + c.S):
        codes3 = [layer.codes_matrix(e, p) for p in range(3)]
        scale3 = [layer.scale_matrix(e, p).view(np.uint16) for p in range(3)]
        zero3 = [layer.zero_matrix(e, p).view(np.uint16) for p in range(3)]
        A3 = [layer.a_matrix(e, p).view(np.uint16) for p in range(3)] if c.r else [None] * 3
        B3 = [layer.b_matrix(e, p).view(np.uint16) for p in range(3)] if c.r else [None] * 3
        out.append(pack_expert(codes3, scale3, zero3, A3, B3, c.H, c.F, c.g, c.r,
                               dense_bits=c.bits if getattr(c, "dense", False) else 0))
    return np.frombuffer(b"".join(out), dtype=np.uint8)


def pack_layer_shared(sl) -> np.ndarray:
    """Blob body for a layer on shared 2D-tiled factors (object with .cfg, .codes/.scale/.zero, .us, .v, .phi): the
    per-expert records without factor parts, then the placement table int32 [E+S][2] (padded to 256 bytes), then
    for section GU the M left blocks (gate and up side by side, afrag layout) and the N right blocks (bfrag layout),
    then the same for section D; the whole padded to 256 bytes."""
    c = sl.cfg
    r16 = (c.r + 15) // 16 * 16
    out = []
    for e in range(c.E + c.S):
        codes3 = [sl.codes[e, p].reshape((c.F, c.H) if p < 2 else (c.H, c.F)) for p in range(3)]
        scale3 = [sl.scale[e, p].reshape(codes3[p].shape[0], -1) for p in range(3)]
        zero3 = [sl.zero[e, p].reshape(codes3[p].shape[0], -1) for p in range(3)]
        out.append(pack_expert(codes3, scale3, zero3, [None] * 3, [None] * 3, c.H, c.F, c.g, c.r,
                               dense_bits=c.bits if getattr(c, "dense", False) else 0, factors=False))
    phi = np.ascontiguousarray(sl.phi, dtype=np.int32).tobytes()
    out.append(phi + b"\0" * ((-len(phi)) % 256))
    M, N = sl.us[0].shape[0], sl.v[0].shape[0]
    sigma = getattr(sl, "sigma", None)          # fp8 factors: us / v are uint8 arrays and one Sigma [3, r] follows the pools
    out += [_afrag_gu(sl.us[0][m], sl.us[1][m], r16, c.H) for m in range(M)]
    out += [_bfrag_gu(sl.v[0][n], sl.v[1][n], r16, c.F // 32) for n in range(N)]
    if sigma is not None:
        out.append(_sig_part([sigma[0], sigma[1]], r16))
    out += [_afrag_d(sl.us[2][m], r16, c.F) for m in range(M)]
    out += [_bfrag_d(sl.v[2][n], r16, c.H // 64) for n in range(N)]
    if sigma is not None:
        out.append(_sig_part([sigma[2]], r16))
    body = b"".join(out)
    return np.frombuffer(body + b"\0" * ((-len(body)) % 256), dtype=np.uint8)


def pack_layer_fp8(fl) -> np.ndarray:
    """Blob body for a layer with fp8 factors (object with .cfg, .codes/.scale/.zero, .a8_list(), .b8_list(), .sigma)."""
    c = fl.cfg
    a8, b8 = fl.a8_list(), fl.b8_list()
    out = []
    for e in range(c.E + c.S):
        codes3 = [fl.codes[e, p].reshape((c.F, c.H) if p < 2 else (c.H, c.F)) for p in range(3)]
        scale3 = [fl.scale[e, p].reshape(codes3[p].shape[0], -1) for p in range(3)]
        zero3 = [fl.zero[e, p].reshape(codes3[p].shape[0], -1) for p in range(3)]
        out.append(pack_expert(codes3, scale3, zero3, [a8[p][e] for p in range(3)], [b8[p][e] for p in range(3)], c.H, c.F,
                               c.g, c.r, dense_bits=c.bits if getattr(c, "dense", False) else 0,
                               sigma3=[fl.sigma[e, p] for p in range(3)]))
    return np.frombuffer(b"".join(out), dtype=np.uint8)
