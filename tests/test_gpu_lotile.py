"""GPU parity of the shared-factor low-rank operator (Section 3.2, Eq. 14-16) against the CPU oracle, through the
C ABI.  bf16 activations: max|gpu - oracle| / max|oracle| <= 2e-2."""
import numpy as np
import pytest
import torch

import oracle
from synth import LayerConfig, make_lotile, make_lotile_fp8, make_logits, bf16_round, CONFIGS
import paper_2605_09281_amd.binding as tq
from gpu_util import DEV, dev16, x_device, rel_err

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


def lt_cfg(cfg_id, **kw):
    base = dict(name="lt", E=6, S=0, k=3, H=128, F=192, T=37, g=64, r=8, bits=4)
    base.update(kw)
    return LayerConfig(cfg_id, **base)


def run_case(cfg, n_in, n_out, M=None, N=None, phi=None, idx=None, w=None, ref_idx=None, ref_w=None):
    us, v, phi0 = make_lotile(cfg, n_in, n_out, M, N)
    phi = phi0 if phi is None else phi
    x = bf16_round(np.random.default_rng(cfg.cfg_id).standard_normal((cfg.T, n_in), dtype=np.float32))
    if idx is None:
        logits, bias = make_logits(cfg)
        idx, w = oracle.route(logits, bias, cfg.k)
    desc = tq.make_lotile_desc(cfg.E, us.shape[0], v.shape[0], n_in, n_out, cfg.r, idx.shape[1])
    err = torch.zeros(1, dtype=torch.int32, device=DEV)
    packed = tq.tq_lotile_pack(desc, dev16(us), dev16(v), torch.from_numpy(phi).to(DEV), err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    ws = torch.empty(max(tq.tq_lotile_workspace_size(desc, cfg.T), 256), dtype=torch.uint8, device=DEV)
    y = tq.tq_lotile_forward(desc, packed, x_device(x, tq.TQ_ACT_BF16), torch.from_numpy(idx).to(DEV),
                             torch.from_numpy(w).to(DEV), workspace=ws)
    torch.cuda.synchronize()
    flag = int(ws[:4].view(torch.int32).item())
    ref = oracle.lotile_forward(x, us, v, phi, idx if ref_idx is None else ref_idx, w if ref_w is None else ref_w)
    return y.float().cpu().numpy(), ref, flag


CASES = {
    # name: (cfg, n_in, n_out, M, N)
    "base": (lt_cfg(301), 128, 192, None, None),
    "rank_not_16": (lt_cfg(302, r=20, E=7, k=2, T=21), 128, 96, 3, 3),
    "one_token": (lt_cfg(303, T=1, E=8, k=2), 128, 64, None, None),
    "ragged_rows": (lt_cfg(304, T=150, E=16, k=4, H=256, r=32), 256, 320, None, None),
    "long_k_split": (lt_cfg(305, T=5, E=9, k=3, H=2048, r=16), 2048, 128, None, None),   # planes > 1
    "wide_grid": (lt_cfg(306, T=70, E=60, k=4, H=256, r=64), 256, 160, None, None),
    "single_row_tile": (lt_cfg(307, T=33, E=5, k=5), 128, 128, 1, 5),
    "single_col_tile": (lt_cfg(308, T=33, E=4, k=2), 128, 128, 4, 1),
    "all_experts": (lt_cfg(309, T=40, E=6, k=6, r=4), 64, 32, None, None),
    "many_selections": (lt_cfg(313, T=19, E=300, k=270, r=8, H=128), 128, 64, None, None),   # selection table: one token per workgroup
    "many_selections_many_rows": (lt_cfg(314, T=700, E=40, k=33, r=16, H=128), 128, 96, None, None),
}


@pytest.mark.parametrize("name", list(CASES))
def test_lotile_forward_matches_oracle(name):
    cfg, n_in, n_out, M, N = CASES[name]
    got, ref, flag = run_case(cfg, n_in, n_out, M, N)
    assert flag == 0
    assert rel_err(got, ref) <= TOL_BF16


def test_lotile_shared_tiles_and_repeated_selection():
    """More experts than tiles (phi maps several experts to one tile) and tokens that list an expert twice: the
    selections add (Eq. 3 sums over them)."""
    cfg = lt_cfg(310, T=45, E=10, k=4)
    rng = np.random.default_rng(310)
    phi = np.stack([rng.integers(0, 2, cfg.E), rng.integers(0, 3, cfg.E)], axis=1).astype(np.int32)
    idx = rng.integers(0, cfg.E, size=(cfg.T, cfg.k)).astype(np.int32)
    w = rng.random((cfg.T, cfg.k)).astype(np.float32)
    got, ref, flag = run_case(cfg, 128, 96, 2, 3, phi=phi, idx=idx, w=w)
    assert flag == 0
    assert rel_err(got, ref) <= TOL_BF16


def test_lotile_invalid_expert_index_is_flagged_and_skipped():
    cfg = lt_cfg(311, T=20, E=6, k=3)
    logits, bias = make_logits(cfg)
    idx, w = oracle.route(logits, bias, cfg.k)
    bad = idx.copy()
    bad[3, 1] = cfg.E
    bad[7, 0] = -1
    w0 = w.copy()
    w0[3, 1] = 0.0
    w0[7, 0] = 0.0
    # the oracle sees the same selections with the two bad ones given weight zero on a valid index
    got, ref, flag = run_case(cfg, 128, 64, idx=bad, w=w, ref_idx=idx, ref_w=w0)
    assert flag == 1
    assert rel_err(got, ref) <= TOL_BF16


def test_lotile_pack_flags_placement_outside_grid():
    cfg = lt_cfg(312)
    us, v, phi = make_lotile(cfg, 128, 64)
    phi = phi.copy()
    phi[2, 0] = us.shape[0]
    desc = tq.make_lotile_desc(cfg.E, us.shape[0], v.shape[0], 128, 64, cfg.r, cfg.k)
    err = torch.zeros(1, dtype=torch.int32, device=DEV)
    tq.tq_lotile_pack(desc, dev16(us), dev16(v), torch.from_numpy(phi).to(DEV), err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 1


def test_lotile_is_reproducible_and_workspace_reusable():
    cfg, n_in, n_out, M, N = CASES["ragged_rows"]
    a, ref, _ = run_case(cfg, n_in, n_out, M, N)
    b, _, _ = run_case(cfg, n_in, n_out, M, N)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("cfg_id,T", [(2, 16), (3, 2048)])
def test_lotile_at_layer_shapes_sampled(cfg_id, T):
    """The down-projection shape of a benchmark layer (ffn -> hidden) with the paper's near-square grid, checked on
    sampled tokens the oracle computes one by one."""
    c = CONFIGS[cfg_id]
    cfg = lt_cfg(320 + cfg_id, E=c.E, k=c.k, T=T, H=c.H, F=c.F, r=c.r)
    us, v, phi = make_lotile(cfg, c.F, c.H)
    rng = np.random.default_rng(cfg.cfg_id)
    x = bf16_round(rng.standard_normal((T, c.F), dtype=np.float32))
    logits, bias = make_logits(cfg)
    idx, w = oracle.route(logits, bias, cfg.k)
    desc = tq.make_lotile_desc(cfg.E, us.shape[0], v.shape[0], c.F, c.H, cfg.r, cfg.k)
    packed = tq.tq_lotile_pack(desc, dev16(us), dev16(v), torch.from_numpy(phi).to(DEV))
    y = tq.tq_lotile_forward(desc, packed, x_device(x, tq.TQ_ACT_BF16), torch.from_numpy(idx).to(DEV),
                             torch.from_numpy(w).to(DEV))
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, 14)]))
    ref = oracle.lotile_forward(x[rows], us, v, phi, idx[rows], w[rows])
    assert rel_err(y[torch.from_numpy(rows).to(DEV)].float().cpu().numpy(), ref) <= TOL_BF16


# ------------------------------------------------------------------ mixed-precision factors (fp8 U, V; fp16 Sigma)
def run_case_fp8(cfg, n_in, n_out, M=None, N=None):
    u8, sigma, v8, phi = make_lotile_fp8(cfg, n_in, n_out, M, N)
    x = bf16_round(np.random.default_rng(cfg.cfg_id).standard_normal((cfg.T, n_in), dtype=np.float32))
    logits, bias = make_logits(cfg)
    idx, w = oracle.route(logits, bias, cfg.k)
    desc = tq.make_lotile_desc(cfg.E, u8.shape[0], v8.shape[0], n_in, n_out, cfg.r, cfg.k, tq.TQ_LOTILE_FP8)
    err = torch.zeros(1, dtype=torch.int32, device=DEV)
    packed = tq.tq_lotile_pack_fp8(desc, torch.from_numpy(u8).to(DEV), dev16(sigma), torch.from_numpy(v8).to(DEV),
                                   torch.from_numpy(phi).to(DEV), err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    ws = torch.empty(max(tq.tq_lotile_workspace_size(desc, cfg.T), 256), dtype=torch.uint8, device=DEV)
    y = tq.tq_lotile_forward(desc, packed, x_device(x, tq.TQ_ACT_BF16), torch.from_numpy(idx).to(DEV),
                             torch.from_numpy(w).to(DEV), workspace=ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    ref = oracle.lotile_forward_fp8(x, u8, sigma, v8, phi, idx, w)
    return y.float().cpu().numpy(), ref


FP8_CASES = {
    "base": (lt_cfg(401), 128, 192, None, None),
    "rank_not_16": (lt_cfg(402, r=20, E=7, k=2, T=21), 128, 96, 3, 3),
    "odd_step_count": (lt_cfg(403, r=16, E=3, k=2, T=9), 96, 64, 1, 3),          # 6 and 3 MFMA steps: a half-filled pair
    "one_token": (lt_cfg(404, T=1, E=8, k=2), 128, 64, None, None),
    "ragged_rows": (lt_cfg(405, T=150, E=16, k=4, H=256, r=32), 256, 320, None, None),
    "long_k_split": (lt_cfg(406, T=5, E=9, k=3, H=2048, r=16), 2048, 128, None, None),
    "wide_grid": (lt_cfg(407, T=70, E=60, k=4, H=256, r=64), 256, 160, None, None),
}


@pytest.mark.parametrize("name", list(FP8_CASES))
def test_lotile_fp8_forward_matches_oracle(name):
    cfg, n_in, n_out, M, N = FP8_CASES[name]
    got, ref = run_case_fp8(cfg, n_in, n_out, M, N)
    assert rel_err(got, ref) <= TOL_BF16


def test_lotile_fp8_every_code_survives_the_packed_form():
    """All 254 finite fp8 codes as entries of U (one per input channel, rank 1, identity-like V): the kernel's
    conversion must agree with the format for each, subnormals and the largest values included."""
    codes = np.array([b for b in range(256) if (b & 0x7F) != 0x7F], dtype=np.uint8)
    n_in = 256
    u8 = np.zeros((1, n_in, 1), dtype=np.uint8)
    u8[0, :codes.size, 0] = codes
    v8 = np.zeros((1, 1, 32), dtype=np.uint8)
    v8[0, 0, :] = 0x38                                   # 1.0
    sigma = np.array([1.0], dtype=np.float16).view(np.uint16)
    phi = np.zeros((1, 2), dtype=np.int32)
    T = n_in
    x = np.eye(T, n_in, dtype=np.float32)                # token b reads input channel b alone
    idx = np.zeros((T, 1), dtype=np.int32)
    w = np.ones((T, 1), dtype=np.float32)
    desc = tq.make_lotile_desc(1, 1, 1, n_in, 32, 1, 1, tq.TQ_LOTILE_FP8)
    packed = tq.tq_lotile_pack_fp8(desc, torch.from_numpy(u8).to(DEV), dev16(sigma), torch.from_numpy(v8).to(DEV),
                                   torch.from_numpy(phi).to(DEV))
    y = tq.tq_lotile_forward(desc, packed, x_device(x, tq.TQ_ACT_BF16), torch.from_numpy(idx).to(DEV),
                             torch.from_numpy(w).to(DEV))
    torch.cuda.synchronize()
    got = y.float().cpu().numpy()[:, 0]
    ref = oracle.lotile_forward_fp8(x, u8, sigma, v8, phi, idx, w)[:, 0]
    # every fp8 value is a bf16 value and nothing else is added to it: exact
    assert np.array_equal(got.astype(np.float64), ref)


@pytest.mark.parametrize("cfg_id,T", [(2, 16), (5, 1024)])
def test_lotile_fp8_at_layer_shapes_sampled(cfg_id, T):
    c = CONFIGS[cfg_id]
    cfg = lt_cfg(420 + cfg_id, E=c.E, k=c.k, T=T, H=c.H, F=c.F, r=c.r)
    u8, sigma, v8, phi = make_lotile_fp8(cfg, c.H, c.F)
    rng = np.random.default_rng(cfg.cfg_id)
    x = bf16_round(rng.standard_normal((T, c.H), dtype=np.float32))
    logits, bias = make_logits(cfg)
    idx, w = oracle.route(logits, bias, cfg.k)
    desc = tq.make_lotile_desc(cfg.E, u8.shape[0], v8.shape[0], c.H, c.F, cfg.r, cfg.k, tq.TQ_LOTILE_FP8)
    packed = tq.tq_lotile_pack_fp8(desc, torch.from_numpy(u8).to(DEV), dev16(sigma), torch.from_numpy(v8).to(DEV),
                                   torch.from_numpy(phi).to(DEV))
    y = tq.tq_lotile_forward(desc, packed, x_device(x, tq.TQ_ACT_BF16), torch.from_numpy(idx).to(DEV),
                             torch.from_numpy(w).to(DEV))
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, 10)]))
    ref = oracle.lotile_forward_fp8(x[rows], u8, sigma, v8, phi, idx[rows], w[rows])
    assert rel_err(y[torch.from_numpy(rows).to(DEV)].float().cpu().numpy(), ref) <= TOL_BF16
