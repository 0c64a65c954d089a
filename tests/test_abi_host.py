"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and its host-side
argument checks and size accounting behave as include/tileq.h says (no kernel is launched)."""
import ctypes
import os
import re

import pytest

import paper_2605_09281_amd.binding as tq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "tileq.h")).read()
    declared = sorted(set(re.findall(r"^(?:const char \*|size_t |tq_status )(tq_[a-z_0-9]+)\(", hdr, flags=re.M)))
    assert set(declared) == set(tq.EXPORTS), declared
    L = tq.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_status_strings():
    assert tq.tq_status_str(0) == "ok"
    for s in range(1, 9):
        assert tq.tq_status_str(s) not in ("ok", "unknown status")


@pytest.mark.parametrize("E,S,H,F,g,r", [(8, 0, 4096, 14336, 128, 32), (60, 0, 2048, 1408, 64, 64),
                                         (128, 0, 4096, 1536, 128, 32), (4, 1, 256, 512, 64, 32)])
def test_packed_size_closed_form(E, S, H, F, g, r):
    """Appendix A.3, per-expert low-rank storage: d = d_basic + r d_fp (1/i + 1/o) bits per weight, here with
    4-bit codes, a 16-bit scale and a 16-bit zero per group and 16-bit factors (no Sigma is stored)."""
    n = tq.tq_packed_size(tq.make_desc(E, S, 2, H, F, g, 4, r))
    # the blob also carries a derived part (bf16 hi and lo of the zero-point coefficient: 2 values per group, in
    # blocks of 16 groups); what remains is the paper's count
    derived = (E + S) * 2 * (2 * F * 2 * 16 * -(-(H // g) // 16) + H * 2 * 16 * -(-(F // g) // 16))
    bits = 8.0 * (n - 256 - derived) / (3 * H * F * (E + S))
    assert abs(bits - (4 + 32 / g + 16 * r * (1 / H + 1 / F))) < 1e-9
    with open(os.path.join(ROOT, "tests", "golden", "bits_per_weight.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            h, ff, gg, rr, val = line.split()
            if (int(h), int(ff), int(gg), int(rr)) == (H, F, g, r):
                assert abs(bits - float(val)) < 5e-7


@pytest.mark.parametrize("bits", [2, 3])
@pytest.mark.parametrize("E,S,H,F,g,r", [(8, 0, 4096, 14336, 128, 32), (60, 0, 2048, 1408, 64, 64)])
def test_packed_size_of_dense_codes_is_the_papers_count(bits, E, S, H, F, g, r):
    """Appendix A.3 with d = 2 or 3: d + 2 * 16 / g (scale and zero) + 16 r (1/i + 1/o) bits per weight, nothing else."""
    n = tq.tq_packed_size(tq.make_desc(E, S, 2, H, F, g, bits, r, flags=tq.TQ_FLAG_DENSE_CODES))
    bpw = 8.0 * (n - 256) / (3 * H * F * (E + S))
    assert abs(bpw - (bits + 32 / g + 16 * r * (1 / H + 1 / F))) < 1e-9


def test_dense_descriptor_limits():
    D = tq.TQ_FLAG_DENSE_CODES
    assert tq.tq_packed_size(tq.make_desc(4, 0, 2, 128, 128, 64, 4, 8, flags=D)) == 0       # 4 bits are not dense
    assert tq.tq_packed_size(tq.make_desc(4, 0, 2, 128, 128, 32, 3, 8, flags=D)) == 0       # groups of 64 and more
    assert tq.tq_packed_size(tq.make_desc(4, 0, 2, 128, 128, 64, 2, 8)) == 0                # 2 bits only densely
    a = tq.tq_packed_size(tq.make_desc(4, 0, 2, 128, 128, 64, 3, 8, flags=D))
    b = tq.tq_packed_size(tq.make_desc(4, 0, 2, 128, 128, 64, 3, 8))
    assert 0 < a < b


def test_packed_size_rank_padding_and_zero_rank():
    base = tq.tq_packed_size(tq.make_desc(4, 0, 2, 256, 512, 64, 4, 0))
    derived = 4 * 2 * (2 * 512 * 32 + 256 * 32)       # H/g = 4 and F/g = 8 groups: one block of 16 each
    assert (base - 256 - derived) * 8 == 4 * 3 * 256 * 512 * (4 + 32 / 64)
    n8 = tq.tq_packed_size(tq.make_desc(4, 0, 2, 256, 512, 64, 4, 8))
    n16 = tq.tq_packed_size(tq.make_desc(4, 0, 2, 256, 512, 64, 4, 16))
    assert n8 == n16 > base          # the rank is stored padded to a multiple of 16


@pytest.mark.parametrize("kw", [dict(E=0), dict(k=9), dict(H=100), dict(F=96), dict(g=48), dict(g=512), dict(bits=5),
                                dict(r=-1), dict(r=300), dict(S=-1), dict(H=192, g=128)])
def test_invalid_descriptors(kw):
    base = dict(E=8, S=0, k=2, H=256, F=512, g=64, bits=4, r=8)
    base.update(kw)
    d = tq.make_desc(base["E"], base["S"], base["k"], base["H"], base["F"], base["g"], base["bits"], base["r"])
    assert tq.tq_packed_size(d) == 0
    assert tq.tq_moe_workspace_size(d, 16) == 0


def test_argument_errors_are_reported_before_any_launch():
    L = tq.lib()
    d = tq.make_desc(8, 0, 2, 256, 512, 64, 4, 8)
    fake = ctypes.c_void_p(0x10000)       # aligned, never dereferenced on these paths
    odd = ctypes.c_void_p(0x10004)
    src = tq._WeightsPtrs(0x10000, 0x10000, 0x10000, 0x10000, 0x10000)
    assert L.tq_pack_weights(ctypes.byref(d), ctypes.byref(src), None, 1 << 30, None, None) == 1
    assert L.tq_pack_weights(ctypes.byref(d), ctypes.byref(src), fake, 16, None, None) == 5
    assert L.tq_pack_weights(ctypes.byref(d), ctypes.byref(src), odd, 1 << 30, None, None) == 3
    src_noA = tq._WeightsPtrs(0x10000, 0x10000, 0x10000, None, None)
    assert L.tq_pack_weights(ctypes.byref(d), ctypes.byref(src_noA), fake, 1 << 30, None, None) == 1
    bad = tq.make_desc(8, 0, 2, 250, 512, 64, 4, 8)
    assert L.tq_pack_weights(ctypes.byref(bad), ctypes.byref(src), fake, 1 << 30, None, None) == 2
    # route
    assert L.tq_route(None, None, 4, 8, 2, fake, fake, None) == 1
    assert L.tq_route(fake, None, 4, 8, 9, fake, fake, None) == 2
    assert L.tq_route(fake, None, 4, 2048, 2, fake, fake, None) == 6
    assert L.tq_route(fake, None, 0, 8, 2, fake, fake, None) == 0        # T == 0: nothing to do
    # forward
    ws = tq.tq_moe_workspace_size(d, 16)
    assert ws > 0 and ws % 256 == 0
    assert L.tq_moe_forward(ctypes.byref(d), fake, fake, fake, fake, 16, fake, None, ws, None) == 1
    assert L.tq_moe_forward(ctypes.byref(d), fake, fake, fake, fake, 16, fake, fake, ws - 1, None) == 5
    assert L.tq_moe_forward(ctypes.byref(d), fake, odd, fake, fake, 16, fake, fake, ws, None) == 3
    assert L.tq_moe_forward(ctypes.byref(d), fake, fake, fake, fake, -1, fake, fake, ws, None) == 2
    assert L.tq_moe_forward(ctypes.byref(d), fake, fake, fake, fake, 0, fake, fake, ws, None) == 0
    # permute
    assert L.tq_permute(fake, 4, 8, 2, fake, fake, fake, None, fake, 0, None) == 5
    assert L.tq_permute(fake, 4, 8, 9, fake, fake, fake, None, fake, 1 << 20, None) == 2


def test_workspace_grows_with_tokens():
    d = tq.make_desc(8, 0, 2, 256, 512, 64, 4, 8)
    a, b = tq.tq_moe_workspace_size(d, 16), tq.tq_moe_workspace_size(d, 4096)
    assert 0 < a < b


@pytest.mark.parametrize("E,S,k,H,F,g,r", [(16, 0, 8, 4096, 1536, 128, 32), (8, 0, 2, 4096, 14336, 128, 32),
                                           (64, 2, 6, 2048, 1408, 128, 16), (4, 0, 1, 64, 64, 32, 0)])
def test_workspace_size_never_shrinks_as_tokens_grow(E, S, k, H, F, g, r):
    """A workspace sized for T tokens must serve every smaller batch: the size is non-decreasing in T, in particular
    across the batch sizes where the split-K planes (4096 assignment rows), the decode scratch (1024) and the slices of
    the pre-pass (160 row tiles) are dropped."""
    d = tq.make_desc(E, S, k, H, F, g, 4, r)
    per = k + S
    slice_rows = 32 * (160 - (E + S)) + 31        # the most rows whose pre-pass may be cut over K (160 row tiles of 32)
    marks = sorted({1, 2, 1024 // per - 1, 1024 // per, 1024 // per + 1, 4096 // per - 1, 4096 // per, 4096 // per + 1,
                    slice_rows // per - 1, slice_rows // per, slice_rows // per + 1, slice_rows // per + 2,
                    2 * 4096 // per, 8192, 20000} - {0})
    sizes = [tq.tq_moe_workspace_size(d, T) for T in marks]
    assert all(b >= a > 0 for a, b in zip(sizes, sizes[1:])), list(zip(marks, sizes))
    if g >= 64:
        # dense codes: beyond the decode path the workspace also holds the derived zero-point coefficient fragments
        dd = tq.make_desc(E, S, k, H, F, g, 3, r, flags=tq.TQ_FLAG_DENSE_CODES)
        dsizes = [tq.tq_moe_workspace_size(dd, T) for T in marks]
        assert all(b >= a > 0 for a, b in zip(dsizes, dsizes[1:])), list(zip(marks, dsizes))
        zc = (E + S) * 2048 * (2 * -(-(H // g) // 16) * (F // 32) + 2 * -(-(F // g) // 16) * (H // 64))
        # batches the decode kernels take (a few rows per expert; on layers of more than 32 experts at most three, eight
        # with a hidden size up to 2048) need nothing extra
        extra_small = tq.tq_moe_workspace_size(dd, 2) - tq.tq_moe_workspace_size(d, 2)
        assert extra_small == 0
        if E + S > 32:
            t_mid = 9 * (E + S) // per + 1          # nine rows per expert: the tiled kernels
            assert tq.tq_moe_workspace_size(dd, t_mid) - tq.tq_moe_workspace_size(d, t_mid) == zc
        assert tq.tq_moe_workspace_size(dd, 20000) == tq.tq_moe_workspace_size(d, 20000) + zc


@pytest.mark.parametrize("E,S,k,H,F,g,r", [(8, 0, 2, 4096, 14336, 128, 32), (60, 0, 4, 2048, 1408, 64, 64), (128, 1, 8, 4096, 1536, 128, 32)])
def test_workspace_size_is_monotonic_over_every_batch_size(E, S, k, H, F, g, r):
    """Brute force over every T up to past the last threshold (4096 assignment rows)."""
    d = tq.make_desc(E, S, k, H, F, g, 4, r)
    last = 0
    for T in range(1, 4096 // (k + S) + 40):
        size = tq.tq_moe_workspace_size(d, T)
        assert size >= last > 0 or T == 1, (T, size, last)
        last = size


# ------------------------------------------------------------------ shared-factor low-rank operator (host side)
def test_lotile_packed_size_closed_form():
    """Appendix A.3, shared tiled factors: M in r + N r out 16-bit values (with r padded to a multiple of 16 and the
    reshaped left factor to whole 32-column tiles), plus the placement table and a header."""
    al = lambda n: (n + 255) // 256 * 256
    for E, M, N, n_in, n_out, r in [(8, 3, 3, 4096, 14336, 32), (64, 8, 8, 1408, 2048, 16), (6, 2, 3, 128, 192, 20)]:
        rp = (r + 15) // 16 * 16
        n = tq.tq_lotile_packed_size(tq.make_lotile_desc(E, M, N, n_in, n_out, r, 2))
        b1 = -(-(M * rp) // 32) * 32 * n_in * 2
        b2 = N * rp * n_out * 2
        assert n == 256 + al(E * 8) + al(b1) + al(b2)


@pytest.mark.parametrize("kw", [dict(E=0), dict(M=0), dict(N=0), dict(n_in=100), dict(n_out=16), dict(r=0), dict(r=257),
                                dict(k=0), dict(k=9), dict(flags=2)])
def test_lotile_invalid_descriptors(kw):
    a = dict(E=8, M=3, N=3, n_in=128, n_out=64, r=8, k=2, flags=0)
    a.update(kw)
    d = tq.make_lotile_desc(a["E"], a["M"], a["N"], a["n_in"], a["n_out"], a["r"], a["k"], a["flags"])
    assert tq.tq_lotile_packed_size(d) == 0
    assert tq.tq_lotile_workspace_size(d, 16) == 0
    L = tq.lib()
    assert L.tq_lotile_forward(ctypes.byref(d), 256, 256, 256, 256, 4, 256, 256, 1 << 20, None) == 2


def test_lotile_host_argument_checks():
    L = tq.lib()
    d = tq.make_lotile_desc(8, 3, 3, 128, 64, 8, 2)
    need = tq.tq_lotile_workspace_size(d, 4)
    assert need > 0 and need % 256 == 0
    assert tq.tq_lotile_workspace_size(d, -1) == 0
    assert L.tq_lotile_forward(ctypes.byref(d), None, 256, 256, 256, 4, 256, 256, need, None) == 1
    assert L.tq_lotile_forward(ctypes.byref(d), 256, 256, 256, 256, -1, 256, 256, need, None) == 2
    assert L.tq_lotile_forward(ctypes.byref(d), 128, 256, 256, 256, 4, 256, 256, need, None) == 3
    assert L.tq_lotile_forward(ctypes.byref(d), 256, 8, 256, 256, 4, 256, 256, need, None) == 3
    assert L.tq_lotile_forward(ctypes.byref(d), 256, 256, 256, 256, 4, 256, 256, need - 1, None) == 5
    assert L.tq_lotile_forward(ctypes.byref(d), 256, 256, 256, 256, 0, 256, 256, need, None) == 0     # T == 0: no-op
    assert L.tq_lotile_pack(ctypes.byref(d), 256, 256, None, 256, 1 << 30, None, None) == 1
    assert L.tq_lotile_pack(ctypes.byref(d), 256, 256, 256, 256, 16, None, None) == 5
    # the workspace grows with T and never shrinks
    assert tq.tq_lotile_workspace_size(d, 4096) > need


def test_lotile_fp8_packed_size_and_flag_checks():
    """Appendix A.3 with d_low = 8: one byte per factor entry (rank padded to 16, contraction to pairs of MFMA steps),
    an fp32 copy of Sigma, the placement table and a header; about half the bf16 form."""
    al = lambda n: (n + 255) // 256 * 256
    L = tq.lib()
    for E, M, N, n_in, n_out, r in [(8, 3, 3, 4096, 14336, 32), (64, 8, 8, 1408, 2048, 16), (6, 2, 3, 96, 160, 20)]:
        rp = (r + 15) // 16 * 16
        d8 = tq.make_lotile_desc(E, M, N, n_in, n_out, r, 2, tq.TQ_LOTILE_FP8)
        d16 = tq.make_lotile_desc(E, M, N, n_in, n_out, r, 2)
        n8, n16 = tq.tq_lotile_packed_size(d8), tq.tq_lotile_packed_size(d16)
        b1 = -(-(M * rp) // 32) * 32 * (-(-(n_in // 16) // 2) * 32)
        b2 = n_out * (-(-(N * rp // 16) // 2) * 32)
        assert n8 == 256 + al(E * 8) + al(rp * 4) + al(b1) + al(b2)
        assert n8 < 0.6 * n16
        assert tq.tq_lotile_workspace_size(d8, 64) == tq.tq_lotile_workspace_size(d16, 64)
        # each pack entry point accepts only its own storage form
        assert L.tq_lotile_pack(ctypes.byref(d8), 256, 256, 256, 256, 1 << 30, None, None) == 2
        assert L.tq_lotile_pack_fp8(ctypes.byref(d16), 256, 256, 256, 256, 256, 1 << 30, None, None) == 2
        assert L.tq_lotile_pack_fp8(ctypes.byref(d8), 256, None, 256, 256, 256, 1 << 30, None, None) == 1
        assert L.tq_lotile_pack_fp8(ctypes.byref(d8), 256, 256, 256, 256, 256, 16, None, None) == 5


# ------------------------------------------------------------------ offline tiling helpers (host only)
def test_lotile_grid_is_the_near_square_grid():
    """Appendix B, "Tiling-size": M = the integer closest to sqrt(E), N = ceil(E / M).  Hand-computed for the expert
    counts of the benchmark layers (8 -> 3 x 3, 60 -> 8 x 8, 64 -> 8 x 8, 128 -> 11 x 12), then the defining
    properties (|M - sqrt(E)| <= 1/2, N the smallest with M N >= E) and the oracle for every E below 700."""
    from oracle import placement
    for E, want in [(8, (3, 3)), (60, (8, 8)), (64, (8, 8)), (128, (11, 12)), (1, (1, 1)), (2, (1, 2)), (3, (2, 2))]:
        assert tq.tq_lotile_grid(E) == want
    for E in range(1, 700):
        M, N = tq.tq_lotile_grid(E)
        assert (M, N) == placement.grid(E)
        assert M * N >= E and abs(M - E ** 0.5) <= 0.5 + 1e-9 and (N - 1) * M < E


def test_lotile_place_worked_example():
    import numpy as np
    rows = [list(map(int, l.split())) for l in open(os.path.join(ROOT, "tests", "golden", "placement_example.txt"))
            if l.strip() and not l.startswith("#")]
    ideal = np.array([r[:2] for r in rows], dtype=np.int32)
    want = np.array([r[2:] for r in rows], dtype=np.int32)
    from oracle import placement
    assert placement.place(ideal, 3, 3) == [tuple(r) for r in want.tolist()]
    assert np.array_equal(tq.tq_lotile_place(ideal, 3, 3), want)


def test_lotile_place_matches_oracle_and_its_invariants():
    import numpy as np
    from oracle import placement
    rng = np.random.default_rng(7)
    for trial in range(60):
        M, N = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        E = int(rng.integers(1, M * N + 1))
        ideal = np.stack([rng.integers(-1, M + 2, E), rng.integers(-1, N + 2, E)], axis=1).astype(np.int32)
        phi = tq.tq_lotile_place(ideal, M, N)
        assert [tuple(r) for r in phi.tolist()] == placement.place(ideal, M, N)
        # no collisions, inside the grid; every expert sits at the smallest Chebyshev distance that was still free
        cells = {tuple(r) for r in phi.tolist()}
        assert len(cells) == E and all(0 <= m < M and 0 <= n < N for m, n in cells)
        taken = set()
        for k in range(E):
            am, an = min(max(ideal[k, 0], 0), M - 1), min(max(ideal[k, 1], 0), N - 1)
            d = max(abs(phi[k, 0] - am), abs(phi[k, 1] - an))
            best = min(max(abs(m - am), abs(n - an)) for m in range(M) for n in range(N) if (m, n) not in taken)
            assert d == best
            taken.add((int(phi[k, 0]), int(phi[k, 1])))
    # distinct ideal tiles inside the grid are kept: the objective of Eq. 9 is zero
    M, N = 4, 5
    perm = rng.permutation(M * N)[:13]
    ideal = np.stack([perm // N, perm % N], axis=1).astype(np.int32)
    assert np.array_equal(tq.tq_lotile_place(ideal, M, N), ideal)
    # fewer cells than experts is refused
    with pytest.raises(tq.TqError):
        tq.tq_lotile_place(np.zeros((5, 2), dtype=np.int32), 2, 2)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark is a one-GPU measurement: asked for more it says so and exits with an error, before touching a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
