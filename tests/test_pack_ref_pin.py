"""CPU pin of oracle/pack_ref.py (the independent packer that the GPU packer is compared with byte for byte).

pack_ref builds the blob with numpy reshapes and transposes.  Here the same blob is written out element by
element, one scalar loop per part, straight from the layout text in include/tileq.h ("word w of (pair, chunk c,
tile, lane) carries the 8 codes of column (tile, lane%32) at kk = 64c + 16w + 8hf + i ..."), on the smallest
layers the descriptor allows, and the two must agree on every byte.  A transposed axis, a wrong nibble order, a
gate/up swap or a mis-sized part in pack_ref fails here without a GPU."""
import struct

import numpy as np
import pytest

from oracle import pack_ref
from synth import LayerConfig, make_layer


def _bf16_rne_scalar(f: float) -> int:
    u = struct.unpack("<I", struct.pack("<f", np.float32(f)))[0]
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF


def _bf16_to_f32(b: int) -> np.float32:
    return np.float32(struct.unpack("<f", struct.pack("<I", b << 16))[0])


def _align256(n):
    return (n + 255) // 256 * 256


def factor_parts_by_definition(sec, A, B, H, F, r, elem="<H"):
    """(bfrag, afrag) of one section from A[p] [K, r] and B[p] [r, N] (fp16 bit patterns, or fp8 codes with
    elem = "<B"), element by element."""
    r16 = (r + 15) // 16 * 16
    if sec == "GU":
        K, pairs, na = H, F // 32, 2 * r16
        col_of = lambda pair, tile, cc: (tile, 32 * pair + cc)
    else:
        K, pairs, na = F, H // 64, r16
        col_of = lambda pair, tile, cc: (2, 64 * pair + 32 * tile + cc)
    # ---- bfrag: fp16 [pairs][r16/16][2 tiles][64 lanes][8]
    bpart = bytearray()
    for pair in range(pairs):
        for s in range(r16 // 16):
            for tile in range(2):
                for lane in range(64):
                    p, n = col_of(pair, tile, lane % 32)
                    hf = lane // 32
                    for i in range(8):
                        rho = 16 * s + 8 * hf + i
                        bpart += struct.pack(elem, int(B[p][rho, n]) if rho < r else 0)
    # ---- afrag: fp16 [ceil(NA/32)][K/16][64 lanes][8]
    apart = bytearray()
    for ta in range((na + 31) // 32):
        for s in range(K // 16):
            for lane in range(64):
                hf = lane // 32
                cc = 32 * ta + lane % 32
                for i in range(8):
                    kk = 16 * s + 8 * hf + i
                    v = 0
                    if cc < na:
                        p, rho = (cc // r16, cc % r16) if sec == "GU" else (2, cc)
                        if rho < r:
                            v = int(A[p][kk, rho])
                    apart += struct.pack(elem, v)
    return bytes(bpart), bytes(apart)


def sig_part_by_definition(sec, sigma3, r):
    """fp32 Sigma of one section: gate then up (r16 each) in GU, r16 in D, zero beyond r, padded to 256 bytes."""
    r16 = (r + 15) // 16 * 16
    out = bytearray()
    for p in ((0, 1) if sec == "GU" else (2,)):
        for rho in range(r16):
            v = np.float32(np.asarray(sigma3[p][rho:rho + 1], dtype=np.uint16).view(np.float16)[0]) if rho < r else np.float32(0)
            out += struct.pack("<f", v)
    out += b"\0" * (_align256(len(out)) - len(out))
    return bytes(out)


def blob_by_definition(layer, with_factors=True, fp8=None) -> bytes:
    """fp8: an object with a8_list() / b8_list() / sigma whose factors replace the layer's fp16 ones."""
    c = layer.cfg
    H, F, g, r = c.H, c.F, c.g, c.r
    r16 = (r + 15) // 16 * 16
    out = bytearray()
    for e in range(c.E + c.S):
        rec = bytearray()
        for sec in ("GU", "D"):
            if sec == "GU":
                K, pairs = H, F // 32
                # pair j = (gate rows 32j..32j+31, up rows 32j..32j+31)
                col_of = lambda pair, tile, cc: (tile, 32 * pair + cc)          # (projection, row of that matrix)
                na = 2 * r16
            else:
                K, pairs = F, H // 64
                col_of = lambda pair, tile, cc: (2, 64 * pair + 32 * tile + cc)
                na = r16
            G = K // g
            codes = [layer.codes_matrix(e, p) for p in range(3)]
            scale = [layer.scale_matrix(e, p).view(np.uint16) for p in range(3)]
            zero = [layer.zero_matrix(e, p).view(np.uint16) for p in range(3)]
            dense_bits = c.bits if c.dense else 0
            # ---- codes: uint32 [pairs][K/64][2 tiles][64 lanes][4], or dense [pairs][K/64][2 tiles][bits][64 lanes]
            part = bytearray()
            for pair in range(pairs if dense_bits else 0):
                for ch in range(K // 64):
                    for tile in range(2):
                        for d in range(dense_bits):
                            for lane in range(64):
                                p, n = col_of(pair, tile, lane % 32)
                                hf = lane // 32
                                word = 0
                                for w in range(4):
                                    for j in range(4):
                                        P = 4 * w + j
                                        lo = int(codes[p][n, 64 * ch + 16 * w + 8 * hf + 2 * j])
                                        hi = int(codes[p][n, 64 * ch + 16 * w + 8 * hf + 2 * j + 1])
                                        if dense_bits == 2:
                                            if P // 8 == d:
                                                word |= (lo | (hi << 16)) << (2 * (P % 8))
                                        elif P < 15:
                                            if P // 5 == d:
                                                word |= (lo | (hi << 16)) << (3 * (P % 5))
                                        else:
                                            word |= (((lo >> d) & 1) << 15) | (((hi >> d) & 1) << 31)
                                part += struct.pack("<I", word)
            for pair in range(0 if dense_bits else pairs):
                for ch in range(K // 64):
                    for tile in range(2):
                        for lane in range(64):
                            p, n = col_of(pair, tile, lane % 32)
                            hf = lane // 32
                            for w in range(4):
                                word = 0
                                for i in range(8):
                                    kk = 64 * ch + 16 * w + 8 * hf + i
                                    word |= (int(codes[p][n, kk]) & 15) << (4 * ((i // 2) + 4 * (i % 2)))
                                part += struct.pack("<I", word)
            rec += part
            # ---- sz: uint32 [pairs][K/g][2 tiles][32]  low half scale, high half zero
            part = bytearray()
            for pair in range(pairs):
                for gi in range(G):
                    for tile in range(2):
                        for cc in range(32):
                            p, n = col_of(pair, tile, cc)
                            part += struct.pack("<I", int(scale[p][n, gi]) | (int(zero[p][n, gi]) << 16))
            rec += part
            # ---- zc: bf16 [pairs][2*ceil(G/16)][2 tiles][64 lanes][8]
            part = bytearray()
            for pair in range(0 if dense_bits else pairs):          # dense blobs carry no zc part
                for s in range(2 * ((G + 15) // 16)):
                    for tile in range(2):
                        for lane in range(64):
                            p, n = col_of(pair, tile, lane % 32)
                            hf = lane // 32
                            for i in range(8):
                                gi = 16 * (s // 2) + 8 * hf + i
                                v = 0
                                if gi < G:
                                    sc = np.float32(scale[p][n, gi:gi + 1].view(np.float16)[0])
                                    ze = np.float32(zero[p][n, gi:gi + 1].view(np.float16)[0])
                                    cf = np.float32(-sc) * np.float32(np.float32(128.0) + ze)
                                    hi = _bf16_rne_scalar(cf)
                                    v = hi if s % 2 == 0 else _bf16_rne_scalar(np.float32(cf - _bf16_to_f32(hi)))
                                part += struct.pack("<H", v)
            rec += part
            if r > 0 and with_factors and fp8 is None:
                A = [layer.a_matrix(e, p).view(np.uint16) for p in range(3)]
                B = [layer.b_matrix(e, p).view(np.uint16) for p in range(3)]
                bpart, apart = factor_parts_by_definition(sec, A, B, H, F, r)
                rec += bpart
                rec += apart
            elif r > 0 and with_factors:
                A = [fp8.a8_list()[p][e] for p in range(3)]
                B = [fp8.b8_list()[p][e] for p in range(3)]
                bpart, apart = factor_parts_by_definition(sec, A, B, H, F, r, elem="<B")
                rec += bpart
                rec += apart
                rec += sig_part_by_definition(sec, [fp8.sigma[e, p] for p in range(3)], r)
        rec += b"\0" * (_align256(len(rec)) - len(rec))
        out += rec
    return bytes(out)


CASES = {
    "smallest_g32_r4": LayerConfig(901, "p", E=1, S=0, k=1, H=64, F=64, T=1, g=32, r=4, bits=4),
    "rect_g64_r20_shared": LayerConfig(902, "p", E=2, S=1, k=1, H=128, F=64, T=1, g=64, r=20, bits=4),
    "rank0_int3": LayerConfig(903, "p", E=1, S=0, k=1, H=64, F=128, T=1, g=64, r=0, bits=3),
    "dense3_r4": LayerConfig(904, "p", E=1, S=1, k=1, H=64, F=128, T=1, g=64, r=4, bits=3, dense=True),
    "dense2_rank0": LayerConfig(905, "p", E=2, S=0, k=1, H=128, F=64, T=1, g=64, r=0, bits=2, dense=True),
}


@pytest.mark.parametrize("name", list(CASES))
def test_pack_ref_equals_the_layout_written_out_element_by_element(name):
    layer = make_layer(CASES[name], workers=1)
    # make the zero-points and scales irregular so that hi/lo parts and both halves of the sz word are exercised
    rng = np.random.default_rng(CASES[name].cfg_id)
    z = layer.zero.view(np.float16).astype(np.float32) + rng.uniform(-0.5, 0.5, layer.zero.shape).astype(np.float32)
    layer.zero = z.astype(np.float16).view(np.uint16)
    want = blob_by_definition(layer)
    got = pack_ref.pack_layer(layer).tobytes()
    assert len(got) == len(want)
    assert got == want


def test_pack_ref_size_is_the_storage_count_of_the_header():
    """Sizes of the five parts per section as include/tileq.h states them."""
    for cfg in CASES.values():
        layer = make_layer(cfg, workers=1)
        H, F, g, r = cfg.H, cfg.F, cfg.g, cfg.r
        r16 = (r + 15) // 16 * 16
        total = 0
        for K, pairs, na in ((H, F // 32, 2 * r16), (F, H // 64, r16)):
            G = K // g
            if cfg.dense:
                total += pairs * (K // 64) * 2 * 64 * 4 * cfg.bits + pairs * G * 2 * 32 * 4
            else:
                total += pairs * (K // 64) * 2 * 64 * 16 + pairs * G * 2 * 32 * 4 + pairs * 2 * ((G + 15) // 16) * 2 * 64 * 16
            if r:
                total += pairs * (r16 // 16) * 2 * 64 * 16 + ((na + 31) // 32) * (K // 16) * 64 * 16
        assert pack_ref.pack_layer(layer).size == (cfg.E + cfg.S) * _align256(total)


def shared_blob_by_definition(sl) -> bytes:
    """The shared-factor blob as include/tileq.h orders it: records without factor parts, the placement table,
    then per section the M left blocks and the N right blocks."""
    c = sl.cfg
    out = bytearray(blob_by_definition(sl.expanded(), with_factors=False))
    for e in range(c.E + c.S):
        out += struct.pack("<ii", int(sl.phi[e, 0]), int(sl.phi[e, 1]))
    out += b"\0" * (_align256(len(out)) - len(out))
    M, N = sl.us[0].shape[0], sl.v[0].shape[0]
    for sec in ("GU", "D"):
        # a left block reads only A, a right block only B: the other operand is a dummy of the right shape
        for m in range(M):
            A = [sl.us[p][m] for p in range(3)]
            out += factor_parts_by_definition(sec, A, [sl.v[p][0] for p in range(3)], c.H, c.F, c.r)[1]
        for n in range(N):
            B = [sl.v[p][n] for p in range(3)]
            out += factor_parts_by_definition(sec, [sl.us[p][0] for p in range(3)], B, c.H, c.F, c.r)[0]
    out += b"\0" * (_align256(len(out)) - len(out))
    return bytes(out)


SHARED_CASES = {
    "grid2x3_r4": (LayerConfig(911, "p", E=3, S=1, k=1, H=64, F=128, T=1, g=32, r=4, bits=4), 2, 3),
    "grid1x2_r20": (LayerConfig(912, "p", E=2, S=0, k=1, H=128, F=64, T=1, g=64, r=20, bits=4), 1, 2),
    "grid2x2_dense3": (LayerConfig(913, "p", E=3, S=0, k=1, H=64, F=64, T=1, g=64, r=8, bits=3, dense=True), 2, 2),
}


@pytest.mark.parametrize("name", list(SHARED_CASES))
def test_shared_pack_ref_equals_the_layout_written_out_element_by_element(name):
    from synth import make_shared_layer
    cfg, M, N = SHARED_CASES[name]
    sl = make_shared_layer(cfg, M, N, workers=1)
    want = shared_blob_by_definition(sl)
    got = pack_ref.pack_layer_shared(sl).tobytes()
    assert len(got) == len(want)
    assert got == want
    # the factors are stored once per tile: r16-padded fp16 blocks, counted from the header's part sizes
    r16 = (cfg.r + 15) // 16 * 16
    fact = 0
    for K, pairs, na in ((cfg.H, cfg.F // 32, 2 * r16), (cfg.F, cfg.H // 64, r16)):
        fact += M * ((na + 31) // 32) * (K // 16) * 1024 + N * pairs * (r16 // 16) * 2048
    rec = len(blob_by_definition(sl.expanded(), with_factors=False))
    assert len(got) == _align256(rec + _align256(8 * (cfg.E + cfg.S)) + fact)


FP8_CASES = {
    "fp8_r20": LayerConfig(921, "p", E=2, S=1, k=1, H=128, F=64, T=1, g=64, r=20, bits=4),
    "fp8_r4_g32": LayerConfig(922, "p", E=1, S=0, k=1, H=64, F=64, T=1, g=32, r=4, bits=4),
    "fp8_dense3_r33": LayerConfig(923, "p", E=2, S=0, k=1, H=64, F=128, T=1, g=64, r=33, bits=3, dense=True),
}


@pytest.mark.parametrize("name", list(FP8_CASES))
def test_fp8_factor_pack_ref_equals_the_layout_written_out_element_by_element(name):
    from synth import make_layer_fp8, Layer
    cfg = FP8_CASES[name]
    fl = make_layer_fp8(cfg, workers=1)
    dummy = Layer(cfg, fl.codes, fl.scale, fl.zero, None, None)
    want = blob_by_definition(dummy, fp8=fl)
    got = pack_ref.pack_layer_fp8(fl).tobytes()
    assert len(got) == len(want)
    assert got == want


def test_shared_fp8_pack_ref_equals_the_layout_written_out_element_by_element():
    """Shared tiled fp8 factors: byte pools in the afrag / bfrag layouts and one fp32 Sigma table per section."""
    from synth import make_shared_layer, fp8_e4m3_encode
    cfg, M, N = LayerConfig(931, "p", E=3, S=1, k=1, H=64, F=128, T=1, g=32, r=12, bits=4), 2, 3
    sl = make_shared_layer(cfg, M, N, workers=1)
    rng = np.random.default_rng(931)
    sl.us = [fp8_e4m3_encode(rng.standard_normal(a.shape).astype(np.float32)) for a in sl.us]
    sl.v = [fp8_e4m3_encode(rng.standard_normal(a.shape).astype(np.float32)) for a in sl.v]
    sl.sigma = (rng.random((3, cfg.r)) + 0.5).astype(np.float16).view(np.uint16)
    got = pack_ref.pack_layer_shared(sl).tobytes()
    # by definition: the records, the placement table, then per section M left blocks, N right blocks, Sigma
    from synth import Layer
    out = bytearray(blob_by_definition(Layer(cfg, sl.codes, sl.scale, sl.zero, None, None), with_factors=False))
    for e in range(cfg.E + cfg.S):
        out += struct.pack("<ii", int(sl.phi[e, 0]), int(sl.phi[e, 1]))
    out += b"\0" * (_align256(len(out)) - len(out))
    for sec in ("GU", "D"):
        for m in range(M):
            out += factor_parts_by_definition(sec, [sl.us[p][m] for p in range(3)], [sl.v[p][0] for p in range(3)], cfg.H, cfg.F,
                                              cfg.r, elem="<B")[1]
        for n in range(N):
            out += factor_parts_by_definition(sec, [sl.us[p][0] for p in range(3)], [sl.v[p][n] for p in range(3)], cfg.H, cfg.F,
                                              cfg.r, elem="<B")[0]
        out += sig_part_by_definition(sec, [sl.sigma[p] for p in range(3)], cfg.r)
    out += b"\0" * (_align256(len(out)) - len(out))
    assert got == bytes(out)
    desc_bytes = None
    import paper_2605_09281_amd.binding as tq
    d = tq.make_desc(cfg.E, cfg.S, cfg.k, cfg.H, cfg.F, cfg.g, cfg.bits, cfg.r, flags=tq.TQ_FLAG_FP8_FACTORS, tiles_m=M, tiles_n=N)
    assert tq.tq_packed_size(d) - 256 == len(got)
