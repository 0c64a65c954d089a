#!/usr/bin/env python3
"""Benchmark of the quantised-expert MoE forward (route + tq_moe_forward) on one MI355X.

One "step" is one pass of the whole hot path over one batch of seeded synthetic tokens whose inputs
(activations, router logits, packed weights) are already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1..5]

By default all five benchmark layers are timed in turn: the headline (`value`, `config`, `roofline`) is the
largest one (config 5, MFMA-bound prefill), and `per_config` carries step time, roofline fractions (decode: HBM),
error against the oracle and the oracle's own rate for each of configs 1-5.  --workload N times one layer only.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12          # B/s, MI355X published
MFMA_BF16_PEAK = 2.5e15    # FLOP/s dense bf16, MI355X published
# HBM bytes per launch of the dominant kernel (gate/up) from separate rocprofv3 FETCH_SIZE and WRITE_SIZE passes
# over this same command, scaled by the streaming-copy calibration: (bytes, file under profiles/ that holds the
# counter readings).  These are profiler runs of their own, not measurements of the present run; workloads that
# have not been counted report null.
TRAFFIC_FROM_PROFILES = {2: (548.1e6 + 1.0e6, "profiles/hbm_traffic_config2_skinny_kernels.txt"),
                         3: (757.1e6 + 92.3e6, "profiles/hbm_traffic_config3_config5_prefill_kernels.txt"),
                         5: (4928.0e6 + 201.3e6, "profiles/hbm_traffic_config3_config5_prefill_kernels.txt")}
STAGES = ["permute", "aug_gate_up", "gate_up", "aug_down", "down", "combine"]


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


class HipEvents:
    """Raw HIP events (ctypes on libamdhip64) so that they can be recorded on the library's stream."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.ev = []
        for _ in range(n):
            e = ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(e)) == 0
            self.ev.append(e)

    def handles(self):
        return [e.value for e in self.ev]

    def record(self, i, stream):
        assert self.hip.hipEventRecord(self.ev[i], ctypes.c_void_p(stream)) == 0

    def sync(self, i):
        assert self.hip.hipEventSynchronize(self.ev[i]) == 0

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        assert self.hip.hipEventElapsedTime(ctypes.byref(ms), self.ev[a], self.ev[b]) == 0
        return float(ms.value)


def algorithmic_work(cfg, idx_np, fp8=False):
    """Algorithmic bytes and flops of one forward, whole path and per dominant kernel: every expert that receives a
    token is read once (codes, scales, zeros, factors), every activation row once per stage."""
    import numpy as np
    H, F, g, r, T = cfg.H, cfg.F, cfg.g, cfg.r, cfg.T
    touched = int(np.unique(idx_np).size) + cfg.S
    a_tot = cfg.a_tot
    cb = cfg.bits if cfg.dense else 4                              # bits each code occupies in the blob
    fb = 1 if fp8 else 2                                           # bytes per factor element
    gu_w = 2 * F * H * cb // 8 + 2 * F * (H // g) * 4 + 2 * r * F * fb  # codes (2 matrices) + scale/zero + B factors
    gu_a = 2 * H * r * fb + (2 * r * 2 if fp8 else 0)              # A factors (read by the pre-pass), Sigma
    d_w = H * F * cb // 8 + H * (F // g) * 4 + r * H * fb
    d_a = F * r * fb + (r * 2 if fp8 else 0)
    w_bytes = touched * (gu_w + gu_a + d_w + d_a)
    act_bytes = T * H * 2 * 2                                      # x in, y out
    flops_gu = a_tot * (4 * H * F + 4 * r * (H + F))               # gate+up: 2 matrices x 2 flop, plus low-rank
    flops_d = a_tot * (2 * H * F + 2 * r * (H + F))
    return dict(touched=touched,
                path_bytes=w_bytes + act_bytes,
                gate_up_bytes=touched * gu_w + a_tot * H * 2 + a_tot * F * 2,
                down_bytes=touched * d_w + a_tot * F * 2 + a_tot * H * 4,
                path_flops=flops_gu + flops_d, gate_up_flops=flops_gu, down_flops=flops_d)


def bench_lotile(args, cfg, dev):
    """One step = tq_route + tq_lotile_forward on x [T, hidden] -> y [T, ffn] with factors resident in HBM."""
    import numpy as np
    import torch
    from synth import make_lotile, make_lotile_fp8, make_x, make_logits, f32_to_bf16_bits
    import paper_2605_09281_amd.binding as tq

    n_in, n_out = cfg.H, cfg.F
    fp8 = args.lotile_fp8
    d16 = lambda a: torch.from_numpy(a.view(np.int16)).to(dev)
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    n_copies = 2
    if fp8:
        u8, sigma, v8, phi = make_lotile_fp8(cfg, n_in, n_out)
        M, N, r = u8.shape[0], v8.shape[0], cfg.r
        desc = tq.make_lotile_desc(cfg.E, M, N, n_in, n_out, r, cfg.k, tq.TQ_LOTILE_FP8)
        packed = [tq.tq_lotile_pack_fp8(desc, torch.from_numpy(u8).to(dev), d16(sigma), torch.from_numpy(v8).to(dev),
                                        torch.from_numpy(phi).to(dev)) for _ in range(n_copies)]
    else:
        us, v, phi = make_lotile(cfg, n_in, n_out)
        M, N, r = us.shape[0], v.shape[0], cfg.r
        desc = tq.make_lotile_desc(cfg.E, M, N, n_in, n_out, r, cfg.k)
        packed = [tq.tq_lotile_pack(desc, d16(us), d16(v), torch.from_numpy(phi).to(dev)) for _ in range(n_copies)]
    fb = 1 if fp8 else 2      # bytes per stored factor entry
    logits_d = torch.from_numpy(logits).to(dev)
    bias_d = None if bias is None else torch.from_numpy(bias).to(dev)
    x_d = torch.from_numpy(f32_to_bf16_bits(x).view(np.int16)).to(dev).view(torch.bfloat16)
    idx_d = torch.empty((cfg.T, cfg.k), dtype=torch.int32, device=dev)
    w_d = torch.empty((cfg.T, cfg.k), dtype=torch.float32, device=dev)
    y_d = torch.empty((cfg.T, n_out), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(tq.tq_lotile_workspace_size(desc, cfg.T), dtype=torch.uint8, device=dev)

    def step(i):
        tq.tq_route(logits_d, bias_d, cfg.k, idx_d, w_d)
        tq.tq_lotile_forward(desc, packed[i % n_copies], x_d, idx_d, w_d, y=y_d, workspace=ws)

    for i in range(max(args.warmup, n_copies)):
        step(i)
    torch.cuda.synchronize()
    y_eager = y_d.clone()
    use_graph = not args.no_graph
    if use_graph:
        graphs = []
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for c in range(n_copies):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    step(c)
                graphs.append(g)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for i in range(args.warmup):
            graphs[i % n_copies].replay()
            torch.cuda.synchronize()
            assert torch.equal(y_d.view(torch.int16), y_eager.view(torch.int16)), "graph replay differs from eager"
        run = lambda i: graphs[i % n_copies].replay()
    else:
        run = step
    ev = HipEvents(2)
    stream = torch.cuda.current_stream().cuda_stream
    ev.record(0, stream)
    for i in range(args.steps):
        run(i)
    ev.record(1, stream)
    torch.cuda.synchronize()
    assert torch.equal(y_d.view(torch.int16), y_eager.view(torch.int16)), "timed run differs from the eager result"
    assert int(ws[:4].view(torch.int32).item()) == 0, "device error flag set"
    ms_per_step = ev.elapsed_ms(0, 1) / args.steps
    # per-kernel durations: the library records events at its stage boundaries on the same stream
    sev = HipEvents(4)
    tq.tq_set_profile_events(sev.handles())
    n_prof = max(1, min(args.steps, 50))
    st_ms = [0.0] * 3
    for i in range(n_prof):
        step(i)
        sev.sync(3)
        for q in range(3):
            st_ms[q] += sev.elapsed_ms(q, q + 1)
    tq.tq_set_profile_events([])
    stage_us = {n: st_ms[q] / n_prof * 1e3 for q, n in enumerate(("projection", "gather", "output"))}
    log("stage durations (us): " + ", ".join(f"{k}={v:.1f}" for k, v in stage_us.items()))
    rp = (r + 15) // 16 * 16
    # algorithmic work of the operator and of its two products (factors as stored, X_proj fp32, S bf16, each read or written once)
    alg_bytes = cfg.T * n_in * 2 + n_in * M * r * fb + N * r * n_out * fb + cfg.T * n_out * 2 + cfg.T * cfg.k * 8
    flops = 2.0 * cfg.T * (n_in * M * r + N * r * n_out)
    kern = {"projection": dict(name="lt_gemm_kernel<.,.,false> (X_proj = x (U Sigma)_reshape)",
                               bytes=cfg.T * n_in * 2 + n_in * M * r * fb + cfg.T * M * r * 4,
                               flops=2.0 * cfg.T * n_in * M * r),
            "output": dict(name="lt_gemm_kernel<.,.,true> (y = S V_flat)",
                           bytes=cfg.T * N * r * 2 + N * r * n_out * fb + cfg.T * n_out * 2,
                           flops=2.0 * cfg.T * N * r * n_out)}
    dom = max(kern, key=lambda q: stage_us[q])
    kd, t_dom = kern[dom], stage_us[dom] * 1e-6
    t = ms_per_step * 1e-3
    if kd["flops"] / kd["bytes"] < MFMA_BF16_PEAK / HBM_PEAK:
        roofline = dict(bound="hbm", kernel=kd["name"], achieved=round(kd["bytes"] / t_dom / 1e9, 1), peak=HBM_PEAK / 1e9,
                        unit="GB/s", frac=round(kd["bytes"] / t_dom / HBM_PEAK, 4), traffic=None,
                        algorithmic_bytes=kd["bytes"])
    else:
        roofline = dict(bound="mfma", kernel=kd["name"], achieved=round(kd["flops"] / t_dom / 1e12, 1),
                        peak=MFMA_BF16_PEAK / 1e12, unit="TFLOP/s", frac=round(kd["flops"] / t_dom / MFMA_BF16_PEAK, 4),
                        traffic=None)
    roofline["stage_us"] = {k: round(v, 2) for k, v in stage_us.items()}
    roofline["operator_algorithmic_bytes"] = alg_bytes
    roofline["operator_flops"] = flops
    roofline["path_hbm_frac"] = round(alg_bytes / t / HBM_PEAK, 4)
    roofline["path_mfma_frac"] = round(flops / t / MFMA_BF16_PEAK, 4)
    cpu_baseline = None
    max_rel_err = None
    if not args.no_cpu_baseline:
        import oracle
        ridx, rw = oracle.route(logits, bias, cfg.k)
        idx_np = idx_d.cpu().numpy()
        assert np.array_equal(ridx, idx_np), "routing indices differ from the oracle"
        n_tok = int(max(1, min(cfg.T, 3e9 // (n_in * M * r + cfg.k * r * n_out))))   # about 10-20 s, one thread
        tok = np.linspace(0, cfg.T - 1, n_tok).astype(np.int64)
        w_np = w_d.cpu().numpy()
        t1 = time.perf_counter()
        if fp8:
            y_ref = oracle.lotile_forward_fp8(x[tok], u8, sigma, v8, phi, idx_np[tok], w_np[tok])
        else:
            y_ref = oracle.lotile_forward(x[tok], us, v, phi, idx_np[tok], w_np[tok])
        cpu_s = time.perf_counter() - t1
        got = y_d.float().cpu().numpy()[tok].astype(np.float64)
        max_rel_err = float(np.max(np.abs(got - y_ref)) / np.max(np.abs(y_ref)))
        cpu_baseline = dict(value=round(n_tok / cpu_s, 3), unit="tokens/s", cores=1, kind="oracle",
                            sample=f"{n_tok} of {cfg.T} tokens of the same workload, {cpu_s:.2f} s")
        assert max_rel_err <= 2e-2, max_rel_err
    out = {
        "metric": "LoTileMoE tokens/s at 1 GPU (route + shared-factor low-rank operator, one linear map)",
        "value": round(cfg.T / t, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic", "launch": "hip_graph" if use_graph else "eager",
        "config": {"workload": f"config {cfg.cfg_id}: {cfg.name}, shared factors hidden -> ffn", "experts": cfg.E,
                   "top_k": cfg.k, "n_in": n_in, "n_out": n_out, "tokens": cfg.T, "rank": r, "tiles_m": M, "tiles_n": N,
                   "factors": "fp8 e4m3 + fp16 sigma" if fp8 else "bf16 (from fp16)"},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "max_rel_err_vs_oracle": max_rel_err,
    }
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=None, choices=[1, 2, 3, 4, 5],
                    help="time one benchmark layer only; default: all five in turn, headline on config 5")
    ap.add_argument("--dense-bits", type=int, default=0, choices=[0, 2, 3],
                    help="with --workload: re-quantise the layer's weights to 2 or 3 bits and store the codes densely "
                         "(decode workloads only)")
    ap.add_argument("--rank", type=int, default=None,
                    help="with --workload: override the rank of the low-rank factors (0 = quantised weights alone), for the "
                         "overhead of the low-rank path over the quantised forward")
    ap.add_argument("--tokens", type=int, default=None,
                    help="with --workload: the layer of that config at another batch size (the library picks the path)")
    ap.add_argument("--fp8-factors", action="store_true",
                    help="with --workload: store the low-rank factors as fp8 E4M3 codes with an fp16 diagonal Sigma")
    ap.add_argument("--separate-route", action="store_true",
                    help="a step calls tq_route and tq_moe_forward one after the other instead of tq_route_moe_forward")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch every step eagerly instead of replaying a captured HIP graph")
    ap.add_argument("--lotile", action="store_true",
                    help="instead of the layer: the shared-factor low-rank operator (tq_lotile_forward) on one linear "
                         "map hidden -> ffn of the workload, with the near-square tile grid")
    ap.add_argument("--lotile-fp8", action="store_true",
                    help="as --lotile with mixed-precision factors (fp8 E4M3 U and V, fp16 Sigma)")
    ap.add_argument("--stream-probe", action="store_true",
                    help="instead of the workload: time a plain 1 GiB streaming copy and read (counter calibration)")
    ap.add_argument("--sketch", action="store_true",
                    help="instead of the layer: the offline sketch decomposition (tq_sketch_lowrank) of the workload's tiled "
                         "gate matrix on the near-square grid, rank = the workload's, 2 power iterations")
    ap.add_argument("--issue-probe", action="store_true",
                    help="instead of the workload: the prefill main loop's instruction mix without memory traffic "
                         "(tq_debug_issue_probe), level by level")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path is a single-GPU kernel library with no collectives). "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from synth import CONFIGS, make_layer, make_x, make_logits, f32_to_bf16_bits
    import paper_2605_09281_amd.binding as tq

    cfg = CONFIGS[args.workload if args.workload is not None else 5]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.stream_probe:
        nbytes = 1 << 30
        bufs = [torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(3)]
        dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        stream = torch.cuda.current_stream().cuda_stream
        ev = HipEvents(2)
        res = {}
        for mode, name in ((0, "copy"), (1, "read"), (2, "read_nontemporal")):
            for i in range(3):
                tq.tq_debug_stream(bufs[i % 3], dst, nbytes, mode)
            torch.cuda.synchronize()
            ev.record(0, stream)
            for i in range(args.steps):
                tq.tq_debug_stream(bufs[i % 3], dst, nbytes, mode)
            ev.record(1, stream)
            torch.cuda.synchronize()
            us = ev.elapsed_ms(0, 1) / args.steps * 1e3
            moved = nbytes * (2 if mode == 0 else 1)
            res[name] = {"us": round(us, 1), "GB/s": round(moved / us / 1e3, 1)}
        print(json.dumps({"stream_probe": res, "bytes": nbytes}), flush=True)
        return
    if args.sketch:
        from synth import lotile_grid
        M, N = lotile_grid(cfg.n_exp)
        rows, cols, r, it = M * cfg.H, N * cfg.F, max(cfg.r, 1), 2
        gen = torch.Generator(device=dev).manual_seed(1234)
        W0 = torch.randn((rows, cols), dtype=torch.float32, device=dev, generator=gen) * 0.02
        S = torch.randn((r, cols), dtype=torch.float32, device=dev, generator=gen)
        ws = torch.empty(tq.lib().tq_sketch_workspace_size(rows, cols), dtype=torch.uint8, device=dev)
        stream = torch.cuda.current_stream().cuda_stream
        ev = HipEvents(2)
        times = []
        for i in range(1 + max(1, min(args.steps, 5))):
            W = W0.clone()
            torch.cuda.synchronize()
            ev.record(0, stream)
            tq.tq_sketch_lowrank(W, r, it, S, workspace=ws)
            ev.record(1, stream)
            torch.cuda.synchronize()
            if i:
                times.append(ev.elapsed_ms(0, 1))
        ms = sum(times) / len(times)
        moved = rows * cols * 4.0 * r * (2 * it + 3)           # per rank: 2 it + 2 reads and one write of the matrix
        print(json.dumps({"sketch": {"rows": rows, "cols": cols, "rank": r, "power_iterations": it, "ms": round(ms, 3),
                                     "ms_per_rank": round(ms / r, 3),
                                     "roofline": {"bound": "hbm", "achieved": round(moved / ms / 1e6, 1), "peak": 8000.0,
                                                  "unit": "GB/s", "frac": round(moved / ms / 1e6 / 8000.0, 4),
                                                  "algorithmic_bytes": moved}}}), flush=True)
        return
    if args.issue_probe:
        scratch = torch.zeros(4096, dtype=torch.uint8, device=dev)
        scratch[256:512].view(torch.float32).copy_(torch.linspace(0.001, 0.064, 64))
        stream = torch.cuda.current_stream().cuda_stream
        ev = HipEvents(2)
        iters = 4000
        n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
        names = {0: "mfma only", 1: "+ lds reads of A", 2: "+ unpack of B", 3: "+ fold (full mix)",
                 4: "+ tile store and barrier"}
        res = {}
        for rep in range(max(1, args.steps)):
            for level in range(5):
                tq.tq_debug_issue_probe(level, 200, scratch)            # spin-up
                torch.cuda.synchronize()
                ev.record(0, stream)
                tq.tq_debug_issue_probe(level, iters, scratch)
                ev.record(1, stream)
                torch.cuda.synchronize()
                ms = ev.elapsed_ms(0, 1)
                clk = scratch[:16].view(torch.int64).cpu().tolist()
                ns = ms * 1e6 / (iters * 32 * 2)                         # per MFMA and SIMD: two waves per SIMD
                ghz = clk[0] / (clk[1] * 10.0)
                pf = n_cu * 4 * 32768.0 / ns * 1e9 / 1e15
                r = res.setdefault(names[level], [])
                r.append({"ns_per_mfma_per_simd": round(ns, 2), "shader_clock_ghz": round(ghz, 3),
                          "cycles_per_mfma": round(ns * ghz, 1), "pflops": round(pf, 3),
                          "frac_of_2.5": round(pf / 2.5, 3)})
        print(json.dumps({"issue_probe": res, "mfmas_per_wave": iters * 32, "waves_per_simd": 2}), flush=True)
        return
    if args.lotile or args.lotile_fp8:
        return bench_lotile(args, cfg, dev)
    if args.workload is not None:
        wl = CONFIGS[args.workload]
        if args.dense_bits:
            wl = wl.replace(bits=args.dense_bits, dense=True)
        if args.rank is not None:
            wl = wl.replace(r=args.rank)
        if args.tokens is not None:
            if args.tokens < 1:
                print("bench.py: --tokens must be at least 1", file=sys.stderr)
                sys.exit(2)
            wl = wl.replace(T=args.tokens)
        res = bench_layer(args, wl, dev, oracle_macs=1.5e11, fp8=args.fp8_factors)
        print(json.dumps(headline(args, res, None)), flush=True)
        return
    # default: every benchmark layer in turn (configs 1-4 with a short oracle sample), the headline on the largest
    per = []
    for c in (1, 2, 3, 4):
        per.append(bench_layer(args, CONFIGS[c], dev, oracle_macs=2.5e10))
        torch.cuda.empty_cache()
        if c == 2:      # the decode layer once more at the paper's headline bit-width, stored densely
            per.append(bench_layer(args, CONFIGS[2].replace(bits=3, dense=True), dev, oracle_macs=2.5e10))
            torch.cuda.empty_cache()
    res5 = bench_layer(args, CONFIGS[5], dev, oracle_macs=1.5e11)
    per.append(res5)
    print(json.dumps(headline(args, res5, per)), flush=True)


def headline(args, res, per):
    """The one JSON line: the contract's keys from `res`, and the list of per-config summaries when all were run."""
    out = {
        "metric": "MoE-layer tokens/s at 1 GPU (route + quantised-expert forward); decode HBM % peak; prefill MFMA % peak",
        "value": res["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "ms_per_step_median": res["ms_per_step_median"],
        "ms_per_step_min": res["ms_per_step_min"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic", "launch": res["launch"], "untimed_spinup_steps": res["spinup_steps"],
        "config": res["config"], "roofline": res["roofline"], "cpu_baseline": res["cpu_baseline"],
        "max_rel_err_vs_oracle": res["max_rel_err"],
    }
    if per is not None:
        out["per_config"] = [
            {"workload": r["config"]["workload"], "tokens": r["config"]["tokens"], "ms_per_step": r["ms_per_step"],
             "ms_per_step_median": r["ms_per_step_median"], "ms_per_step_min": r["ms_per_step_min"],
             "tokens_per_s": r["tokens_per_s"], "bound": r["roofline"]["bound"], "kernel": r["roofline"]["kernel"],
             "frac": r["roofline"]["frac"], "path_frac": r["roofline"]["path_frac"],
             "hbm_path_frac": r["roofline"]["hbm_path_frac"], "mfma_path_frac": r["roofline"]["mfma_path_frac"],
             "stage_us": r["roofline"]["stage_us"], "max_rel_err_vs_oracle": r["max_rel_err"],
             "cpu_baseline": r["cpu_baseline"]} for r in per]
    return out


def bench_layer(args, cfg, dev, oracle_macs, fp8=False):
    """Times K steps of route + forward on one benchmark layer; returns a dict of results."""
    import numpy as np
    import torch
    from synth import make_layer, make_layer_fp8, make_x, make_logits, f32_to_bf16_bits
    import paper_2605_09281_amd.binding as tq

    t0 = time.time()
    layer = (make_layer_fp8 if fp8 else make_layer)(cfg, workers=min(16, os.cpu_count() or 8))
    x = make_x(cfg)
    logits, bias = make_logits(cfg)
    log(f"workload {cfg.cfg_id} ({cfg.name}): inputs generated in {time.time() - t0:.1f}s")

    def dev16(a):
        return torch.from_numpy(a.view(np.int16)).to(dev)

    desc = tq.make_desc(cfg.E, cfg.S, cfg.k, cfg.H, cfg.F, cfg.g, cfg.bits, cfg.r, tq.TQ_ACT_BF16,
                        (tq.TQ_FLAG_DENSE_CODES if cfg.dense else 0) | (tq.TQ_FLAG_FP8_FACTORS if fp8 else 0))
    codes_d = torch.from_numpy(layer.codes).to(dev)
    sc_d, ze_d = dev16(layer.scale), dev16(layer.zero)
    if fp8:
        A_d, B_d, sg_d = torch.from_numpy(layer.A8).to(dev), torch.from_numpy(layer.B8).to(dev), dev16(layer.sigma)
    else:
        A_d = dev16(layer.A) if cfg.r else None
        B_d = dev16(layer.B) if cfg.r else None
        sg_d = None
    n_copies = 2      # rotate weight copies so that no step finds its weights warm in the last-level cache
    packed = [tq.tq_pack_weights(desc, codes_d, sc_d, ze_d, A_d, B_d, sigma=sg_d) for _ in range(n_copies)]
    torch.cuda.synchronize()
    del codes_d, sc_d, ze_d, A_d, B_d, sg_d
    torch.cuda.empty_cache()
    logits_d = torch.from_numpy(logits).to(dev)
    bias_d = None if bias is None else torch.from_numpy(bias).to(dev)
    x_d = torch.from_numpy(f32_to_bf16_bits(x).view(np.int16)).to(dev).view(torch.bfloat16)
    idx_d = torch.empty((cfg.T, cfg.k), dtype=torch.int32, device=dev)
    w_d = torch.empty((cfg.T, cfg.k), dtype=torch.float32, device=dev)
    y_d = torch.empty_like(x_d)
    ws = torch.empty(tq.tq_moe_workspace_size(desc, cfg.T), dtype=torch.uint8, device=dev)
    tq.tq_init()

    def step(i):
        if args.separate_route:
            tq.tq_route(logits_d, bias_d, cfg.k, idx_d, w_d)
            tq.tq_moe_forward(desc, packed[i % n_copies], x_d, idx_d, w_d, y=y_d, workspace=ws)
        else:      # routing and forward in one call: decode batches route inside the permutation's launch
            tq.tq_route_moe_forward(desc, packed[i % n_copies], x_d, logits_d, bias_d, idx_d, w_d, y_d, ws)

    for i in range(max(args.warmup, n_copies)):
        step(i)
    torch.cuda.synchronize()
    y_eager = y_d.clone()
    ev = HipEvents(args.steps + 1 + 7)
    use_graph = not args.no_graph
    if use_graph:
        # the step is a short chain of kernels: replaying a captured HIP graph (one per weight copy) removes the
        # launch gaps between them.  The library records no memset nodes; every replay is checked below.
        graphs = []
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for c in range(n_copies):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    step(c)
                graphs.append(g)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for i in range(args.warmup):
            graphs[i % n_copies].replay()
            torch.cuda.synchronize()
            assert torch.equal(y_d.view(torch.int16), y_eager.view(torch.int16)), "graph replay differs from eager"
        run = lambda i: graphs[i % n_copies].replay()
    else:
        run = step
    stream = torch.cuda.current_stream().cuda_stream
    # Spin-up, untimed: the verification replays above synchronise after every step, which lets the clocks fall back;
    # the first ten to twenty steps after such a pause run up to 8 % slower.  Enough back-to-back steps to cover
    # about 30 ms go first, with no pause before the timed region.
    ev.record(0, stream)
    for i in range(3):
        run(i)
    ev.record(1, stream)
    torch.cuda.synchronize()
    est_ms = max(ev.elapsed_ms(0, 1) / 3, 1e-3)
    spinup = int(max(args.warmup, min(2000, 30.0 / est_ms)))
    for i in range(spinup):
        run(i)
    # the timed region: exactly K steps between two events (this gives `value`)
    ev.record(0, stream)
    for i in range(args.steps):
        run(i)
    ev.record(1, stream)
    torch.cuda.synchronize()
    assert torch.equal(y_d.view(torch.int16), y_eager.view(torch.int16)), "timed run differs from the eager result"
    ms_per_step = ev.elapsed_ms(0, 1) / args.steps
    # a second pass of K steps with an event at every step boundary: median and minimum step time
    ev.record(0, stream)
    for i in range(args.steps):
        run(i)
        ev.record(i + 1, stream)
    torch.cuda.synchronize()
    per_step_seq = [ev.elapsed_ms(i, i + 1) for i in range(args.steps)]
    if os.environ.get("TQ_BENCH_TRACE_STEPS"):
        log("per-step us: " + " ".join(f"{t * 1e3:.0f}" for t in per_step_seq))
    per_step = sorted(per_step_seq)
    ms_median, ms_min = per_step[len(per_step) // 2], per_step[0]
    log(f"timed {args.steps} steps after {spinup} spin-up steps: {ms_per_step * 1e3:.1f} us/step (events; median of a "
        f"second pass {ms_median * 1e3:.1f}, min {ms_min * 1e3:.1f})")
    assert int(ws[:4].view(torch.int32).item()) == 0, "device error flag set"

    # per-stage kernel durations: the library records events at its stage boundaries on the same stream
    so = args.steps + 1
    tq.tq_set_profile_events(ev.handles()[so:])
    n_prof = max(1, min(args.steps, 50))
    stage_ms = [0.0] * 6
    for i in range(n_prof):
        step(i)
        ev.sync(so + 6)
        for q in range(6):
            stage_ms[q] += ev.elapsed_ms(so + q, so + q + 1)
    tq.tq_set_profile_events([])
    stage_us = {name: stage_ms[q] / n_prof * 1e3 for q, name in enumerate(STAGES)}
    log("stage durations (us): " + ", ".join(f"{k}={v:.1f}" for k, v in stage_us.items()))

    idx_np = idx_d.cpu().numpy()
    work = algorithmic_work(cfg, idx_np, fp8)
    t_step = ms_per_step * 1e-3
    hbm_path = work["path_bytes"] / t_step / HBM_PEAK
    mfma_path = work["path_flops"] / t_step / MFMA_BF16_PEAK
    hbm_bound = work["path_flops"] / max(work["path_bytes"], 1) < MFMA_BF16_PEAK / HBM_PEAK
    t_gu = stage_us["gate_up"] * 1e-6
    ne = cfg.E + cfg.S
    decode_path = ((cfg.a_tot // ne <= (12 if ne <= 8 else 10)) if ne <= 32 else cfg.a_tot <= (8 if cfg.H <= 2048 else 3) * ne) and cfg.a_tot <= 1024   # the library's rule
    kname = ("gate/up stage (moe_skinny_kernel<0,.>)" if decode_path else
             "gate/up stage (moe_prefill_kernel<0,.>, or moe_mfma_kernel<.,.,0,.> where the layer does not qualify)")
    traffic, traffic_source = (None, None) if (cfg.dense or fp8) else TRAFFIC_FROM_PROFILES.get(cfg.cfg_id, (None, None))
    if hbm_bound:
        ach = work["gate_up_bytes"] / t_gu / 1e9
        roofline = dict(bound="hbm", kernel=kname, achieved=round(ach, 1), peak=HBM_PEAK / 1e9, unit="GB/s",
                        frac=round(ach / (HBM_PEAK / 1e9), 4), traffic=traffic, traffic_source=traffic_source,
                        algorithmic_bytes=work["gate_up_bytes"],
                        path_achieved=round(work["path_bytes"] / t_step / 1e9, 1), path_frac=round(hbm_path, 4))
    else:
        ach = work["gate_up_flops"] / t_gu / 1e12
        roofline = dict(bound="mfma", kernel=kname, achieved=round(ach, 1), peak=MFMA_BF16_PEAK / 1e12, unit="TFLOP/s",
                        frac=round(ach / (MFMA_BF16_PEAK / 1e12), 4), traffic=traffic, traffic_source=traffic_source,
                        algorithmic_flops=work["gate_up_flops"],
                        path_achieved=round(work["path_flops"] / t_step / 1e12, 1), path_frac=round(mfma_path, 4))
    roofline["hbm_path_frac"] = round(hbm_path, 4)
    roofline["mfma_path_frac"] = round(mfma_path, 4)
    roofline["gate_up_mfma_frac"] = round(work["gate_up_flops"] / t_gu / MFMA_BF16_PEAK, 4)
    roofline["gate_up_hbm_frac"] = round(work["gate_up_bytes"] / t_gu / HBM_PEAK, 4)
    roofline["stage_us"] = {k: round(v, 2) for k, v in stage_us.items()}
    roofline["stage_note"] = ("intervals between HIP events recorded at the library's stage boundaries in an eager pass; an "
                              "interval in which nothing is launched (aug_gate_up of a decode batch, whose pre-pass rides in the "
                              "permutation's launch) still reads ~5 us of event processing; ms_per_step is timed separately "
                              "over the replayed HIP graph")

    # the oracle beside it: a bounded token sample of the same workload, timed on this machine's host cores
    cpu_baseline = None
    max_rel_err = None
    if not args.no_cpu_baseline:
        import oracle
        ridx, rw = oracle.route(logits, bias, cfg.k)
        assert np.array_equal(ridx, idx_np), "routing indices differ from the oracle"
        pair_cost = 3.0 * cfg.H * cfg.F * (cfg.k + cfg.S)          # MACs per token
        n_tok = int(max(1, min(cfg.T, oracle_macs // pair_cost)))
        tok = np.linspace(0, cfg.T - 1, n_tok).astype(np.int32)
        w_np = w_d.cpu().numpy()
        t1 = time.perf_counter()
        if fp8:
            y_ref = oracle.moe_forward_fp8(cfg, layer.codes, layer.scale, layer.zero, layer.a8_list(), layer.b8_list(),
                                           layer.sigma, x, ridx, w_np, tokens=tok)
        else:
            y_ref = oracle.moe_forward_layer(layer, x, ridx, w_np, tokens=tok)
        cpu_s = time.perf_counter() - t1
        got = y_d.float().cpu().numpy()[tok].astype(np.float64)
        max_rel_err = float(np.max(np.abs(got - y_ref)) / np.max(np.abs(y_ref)))
        cpu_baseline = dict(value=round(n_tok / cpu_s, 3), unit="tokens/s", cores=oracle.num_threads(), kind="oracle",
                            sample=f"{n_tok} of {cfg.T} tokens of the same workload, {cpu_s:.1f} s")
        log(f"oracle: {n_tok} tokens in {cpu_s:.1f}s on {oracle.num_threads()} threads; max rel err {max_rel_err:.3e}")
        assert max_rel_err <= 2e-2, max_rel_err
    del packed, ws
    return dict(tokens_per_s=round(cfg.T / t_step, 1), ms_per_step=round(ms_per_step, 5),
                ms_per_step_median=round(ms_median, 5), ms_per_step_min=round(ms_min, 5),
                launch="hip_graph" if use_graph else "eager", spinup_steps=spinup,
                config={"workload": f"config {cfg.cfg_id}: {cfg.name}" + (f", codes re-quantised to {cfg.bits} bits, stored densely" if cfg.dense else "") + (", fp8 E4M3 factors with fp16 Sigma" if fp8 else ""), "experts": cfg.E, "shared": cfg.S, "top_k": cfg.k,
                        "hidden": cfg.H, "ffn": cfg.F, "tokens": cfg.T, "group": cfg.g, "rank": cfg.r, "bits": cfg.bits,
                        "touched_experts": work["touched"]},
                roofline=roofline, cpu_baseline=cpu_baseline, max_rel_err=max_rel_err)


if __name__ == "__main__":
    main()
