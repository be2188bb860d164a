#!/usr/bin/env python3
"""Benchmark of the fixed-routing MoE expert layer on one MI355X.

One step = the whole hot path once over configuration 3 (T=8192, d=2048, f=1408, E=64, top-6, Zipf(1.2)
routing): plan build, gate/up GEMMs + gate-weighted SiLU*up (rows of x gathered inside the GEMM), down GEMM,
combine, then the backward pass (dH + dSwiGLU, dW2, dW1/dW3, dXp, dX reduce; dY and x read in place).  Inputs are synthetic, seeded, and resident in HBM
before the timed region.  Prints ONE JSON line.

  value     algorithmic TFLOP/s of the step (forward 6*T*k*d*f + backward 12*T*k*d*f, App. M convention)
  roofline  the dominant kernel's achieved TFLOP/s (HIP events around each launch, on the launch stream)
            against the MI355X dense bf16 MFMA peak
  cpu_baseline  the CPU oracle timed on a bounded token sample of the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "config3_hbm_traffic.txt")


def measured_traffic(phase):
    """HBM bytes per launch of a phase's kernel from the committed rocprofv3 --pmc summary (None if absent)."""
    try:
        with open(TRAFFIC_FILE) as fh:
            for line in fh:
                parts = line.split()
                if len(parts) >= 2 and parts[0] == "traffic_bytes." + phase:
                    return float(parts[1])
    except OSError:
        pass
    return None



def phase_work(T, d, f, E, k):
    """Algorithmic work of each kernel phase per launch: ('mfma', FLOP) or ('hbm', bytes)."""
    N = T * k
    return {
        "gateup": ("mfma", 4.0 * N * d * f),
        "down": ("mfma", 2.0 * N * d * f),
        "dH": ("mfma", 2.0 * N * d * f),
        "dW2": ("mfma", 2.0 * N * d * f),
        "dW13": ("mfma", 4.0 * N * d * f),
        "dXp": ("mfma", 4.0 * N * d * f),
        "permute": ("hbm", 2.0 * T * d + 4.0 * N + 2.0 * N * d),
        "dO": ("hbm", 2.0 * T * d + 10.0 * N + 2.0 * N * d),
        "combine": ("hbm", 2.0 * N * d + 4.0 * N + 2.0 * T * d),
        "dX_reduce": ("hbm", 2.0 * N * d + 4.0 * N + 2.0 * T * d),
    }


def cpu_baseline(cfg, idx, gates, t, n_tok):
    """Time the oracle (forward + backward) on n_tok sampled tokens of the workload."""
    import numpy as np
    import torch

    import oracle
    from oracle.subproblem import token_subproblem

    rng = np.random.default_rng(0)
    sel = np.sort(rng.choice(cfg["T"], size=n_tok, replace=False))

    class Lazy:
        def __init__(self, ten):
            self.ten = ten

        def __getitem__(self, sel_e):
            s = torch.as_tensor(np.asarray(sel_e), device=self.ten.device, dtype=torch.long)
            return self.ten.index_select(0, s).float().cpu().numpy()

    x = t["x"].float().cpu().numpy()
    dY = t["dY"].float().cpu().numpy()
    sp = token_subproblem(sel, x, oracle.bf16_bits_to_f32(gates), idx, Lazy(t["W1"]), Lazy(t["W3"]), Lazy(t["W2"]), dY)
    t0 = time.perf_counter()
    oracle.moe_fwd(sp["x"], sp["w"], sp["idx"], sp["W1"], sp["W3"], sp["W2"], dtype=np.float32)
    oracle.moe_bwd(sp["x"], sp["w"], sp["idx"], sp["W1"], sp["W3"], sp["W2"], sp["dY"], dtype=np.float32)
    dt = time.perf_counter() - t0
    return n_tok / dt, dt, oracle.num_threads()


def routing_stats_bench(b, wl, dev, reps, cpu_samples):
    """Time the routing-statistics kernels on the corpus workload (ids resident in HBM); GB/s = id bytes read
    plus result bytes written, per launch.  The oracle is timed on a bounded sample of the same sequences."""
    import numpy as np
    import torch

    c = wl.CORPUS
    S, L, E, k, n_nodes = c["S"], c["L"], c["E"], c["k"], c["n_nodes"]
    idx = wl.draw_sequence_routing(S, L, E, k, c["n_topics"], seed=0, device=dev)
    nodes = wl.draw_expert_placement(E, n_nodes, seed=0)
    bits = np.zeros(E, dtype=np.uint64)
    for n, members in enumerate(nodes):
        bits[members] |= np.uint64(1) << np.uint64(n)
    bits_d = torch.from_numpy(bits.view(np.int64)).to(dev)
    counts = torch.empty((S, E), dtype=torch.int32, device=dev)
    ent = torch.empty(S, dtype=torch.float64, device=dev)
    loads = torch.empty(E, dtype=torch.int64, device=dev)
    mv = torch.empty(1, dtype=torch.float64, device=dev)
    comm = torch.empty((S, n_nodes), dtype=torch.int32, device=dev)
    best = torch.empty(S, dtype=torch.int32, device=dev)
    P = torch.empty((E, E), dtype=torch.int64, device=dev)
    grp = torch.empty(E, dtype=torch.int32, device=dev)
    flat = idx.view(S * L, k)

    def run():
        b.grouter_sample_stats(idx, E, counts, ent, loads, mv, bits_d, n_nodes, comm, best)   # both in one pass
        b.grouter_affinity(idx, E, counts, ent, loads, mv)
        b.grouter_sample_placement(idx, E, bits_d, n_nodes, comm, best)
        b.grouter_coactivation(flat, E, P)
        b.grouter_fold_groups(P, E // 4, grp)

    run()
    torch.cuda.synchronize()
    b.grouter_timing_enable(True)
    b.grouter_timing_read()
    for _ in range(reps):
        run()
    torch.cuda.synchronize()
    b.grouter_timing_enable(False)
    ph = b.grouter_timing_read()
    id_bytes = S * L * k
    alg = {"affinity": id_bytes + S * E * 4 + S * 8 + E * 8, "placement": id_bytes + S * n_nodes * 4 + S * 4,
           "sample_stats": id_bytes + S * E * 4 + S * 8 + E * 8 + S * n_nodes * 4 + S * 4,
           "coactivation": id_bytes + E * E * 8}
    out = {"workload": f"{S} packed sequences x {L} tokens, E={E}, top-{k}, uint8 ids ({id_bytes / 1e6:.1f} MB), "
                       f"{n_nodes} nodes, fold {E}->{E // 4}"}
    for name in ("sample_stats", "affinity", "placement", "coactivation", "fold"):
        ms, cnt = ph[name]
        if not cnt:
            continue
        e = {"avg_ms": round(ms / cnt, 5)}
        if name in alg:
            e["gbs"] = round(alg[name] / (ms / cnt * 1e-3) / 1e9, 1)
            e["frac_hbm_peak"] = round(e["gbs"] / PEAK_HBM_GBS, 4)
            e["tokens_per_s"] = round(S * L / (ms / cnt * 1e-3), 0)
        out[name] = e
    out["maxvio"] = round(float(mv.cpu()[0]), 4)
    out["frac_sequences_above_6.85_bits"] = round(float((ent > 6.85).double().mean().cpu()), 4)
    if cpu_samples > 0:
        from oracle import routing_stats as rs

        sub = idx[:cpu_samples].cpu().numpy()
        t0 = time.perf_counter()
        oc = rs.affinity_counts(sub, E)
        rs.entropy_bits(oc)
        rs.placement(sub, nodes, E)
        rs.coactivation(sub.reshape(-1, k), E)
        dt = time.perf_counter() - t0
        out["cpu_oracle"] = {"tokens_per_s": round(cpu_samples * L / dt, 0), "seconds": round(dt, 2), "kind": "oracle",
                             "sample": f"first {cpu_samples} of {S} sequences: affinity + entropy + placement + "
                                       f"co-activation (numpy)"}
    return out


def calibration_bench(b, dev, N, d, f):
    """What this machine sustains on the matrix cores, measured apart from the step: the library's MFMA instruction
    stream with no memory traffic (grouter_mfma_probe), and the vendor's dense bf16 GEMM (torch.matmul) on the
    dense counterparts of the layer's GEMM shapes."""
    import torch

    def avg_ms(fn, iters):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    out = {"mfma_probe": {}, "lds_read_probe": {}, "dense_matmul": {}}
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    wgs, iters = 2 * cus, 4000
    sink = torch.empty(wgs * 256, dtype=torch.float32, device=dev)
    for mode, name in ((0, "32x32x16 operands_in_registers"), (1, "32x32x16 operands_read_from_lds"),
                       (2, "16x16x32 operands_in_registers"), (3, "16x16x32 operands_read_from_lds"),
                       (6, "16x16x32 128x128 wave tile, one wave per SIMD, operands_in_registers"),
                       (7, "16x16x32 128x128 wave tile, one wave per SIMD, operands_read_from_lds")):
        n_wg, n_it = (wgs, iters) if mode < 6 else (cus, 2 * iters)     # the same number of MFMAs either way
        flop = b.grouter_mfma_probe(mode, n_it, n_wg, sink)
        ms = avg_ms(lambda: b.grouter_mfma_probe(mode, n_it, n_wg, sink), 10)
        tf = flop / (ms * 1e-3) / 1e12
        out["mfma_probe"][name] = {"avg_ms": round(ms, 4), "tflops": round(tf, 1),
                                   "frac_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4)}
    # the LDS fragment reads of the main loops alone (no MFMAs): what the LDS delivers per CU
    out["lds_read_probe"] = {}
    for mode, name in ((4, "16-byte reads"), (5, "pairs of transposing 8-byte reads")):
        b.grouter_mfma_probe(mode, iters, wgs, sink)
        ms = avg_ms(lambda: b.grouter_mfma_probe(mode, iters, wgs, sink), 10)
        gbs_cu = wgs * 4 * iters * 6 * 1024 / (ms * 1e-3) / 1e9 / cus
        out["lds_read_probe"][name] = {"avg_ms": round(ms, 4), "gb_per_s_per_cu": round(gbs_cu, 1)}
    g = torch.Generator(device=dev).manual_seed(7)
    shapes = [("gate_up", N, 2 * f, d), ("down", N, d, f), ("square", 8192, 8192, 8192)]
    for name, M, Nn, K in shapes:
        a = torch.randn(M, K, device=dev, dtype=torch.bfloat16, generator=g)
        for layout in ("B[K][N]", "B[N][K]"):
            w = torch.randn((K, Nn) if layout == "B[K][N]" else (Nn, K), device=dev, dtype=torch.bfloat16, generator=g)
            bm = w if layout == "B[K][N]" else w.t()
            c = torch.empty(M, Nn, device=dev, dtype=torch.bfloat16)
            ms = avg_ms(lambda: torch.matmul(a, bm, out=c), 10)
            tf = 2.0 * M * Nn * K / (ms * 1e-3) / 1e12
            out["dense_matmul"][f"{name} {M}x{Nn}x{K} {layout}"] = {"avg_ms": round(ms, 4), "tflops": round(tf, 1),
                                                                   "frac_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4)}
            del w, bm, c
        del a
    z = torch.zeros(8192, 8192, device=dev, dtype=torch.bfloat16)
    c = torch.empty_like(z)
    ms = avg_ms(lambda: torch.matmul(z, z, out=c), 10)
    tf = 2.0 * 8192 ** 3 / (ms * 1e-3) / 1e12
    out["dense_matmul"]["square 8192x8192x8192 all-zero operands"] = {"avg_ms": round(ms, 4), "tflops": round(tf, 1),
                                                                      "frac_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="named configuration to time (default: 3, the headline)")
    ap.add_argument("--cpu-tokens", type=int, default=4096, help="tokens in the CPU-oracle sample (0 = skip)")
    ap.add_argument("--no-kernel-events", action="store_true", help="do not bracket kernels with events")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB after the timed region, so that a "
                         "rocprofv3 --pmc run of this command can scale FETCH_SIZE / WRITE_SIZE against a known size")
    ap.add_argument("--no-routing-stats", action="store_true",
                    help="skip the routing-statistics kernels (timed after and apart from the step)")
    ap.add_argument("--calibrate", action="store_true",
                    help="after the timed region, also time the matrix-core probe (MFMA stream with no memory traffic) "
                         "and torch.matmul on the dense counterparts of the GEMM shapes; reported under 'calibration'")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2603_06626_amd import binding as b
    from paper_2603_06626_amd import workloads as wl

    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[args.config]
    T, d, f, E, k = cfg["T"], cfg["d"], cfg["f"], cfg["E"], cfg["k"]
    bwd = cfg["bwd"]
    n_layers = cfg["layers"]
    idx, gates = wl.make_routing(args.config)
    layers = [wl.make_tensors(args.config, layer=i, device=dev, need_bwd=True) for i in range(n_layers)]
    idx_d = torch.from_numpy(idx).to(dev)
    gw = torch.from_numpy(gates.view(np.int16)).to(dev).view(torch.bfloat16)
    plan = torch.empty(b.grouter_plan_bytes(T, k, E), dtype=torch.uint8, device=dev)
    if bwd:
        ctx = torch.empty(b.grouter_ctx_bytes(T, k, d, f), dtype=torch.uint8, device=dev)
        scr = torch.empty(b.grouter_bwd_scratch_bytes(T, k, d, f), dtype=torch.uint8, device=dev)
    else:
        ctx = torch.empty(b.grouter_fwd_only_bytes(T, k, d, f), dtype=torch.uint8, device=dev)
    y = torch.empty((T, d), dtype=torch.bfloat16, device=dev)
    dX = torch.empty_like(y)
    t0_ = layers[0]
    dW1, dW3, dW2 = torch.empty_like(t0_["W1"]), torch.empty_like(t0_["W3"]), torch.empty_like(t0_["W2"])

    def step():
        # the cached routing of a batch is its ids and its scores: both go into the plan, once for all layers
        b.grouter_plan_build(idx_d, E, plan)
        b.grouter_plan_set_gates(plan, E, gw)
        for t in layers:
            if not bwd:     # forward-only configurations: no saved context, rows gathered inside the gate/up GEMM
                b.grouter_moe_fwd_only(plan, t["x"], None, t["W1"], t["W3"], t["W2"], y, ctx, k=k)
                continue
            b.grouter_moe_fwd(plan, t["x"], None, t["W1"], t["W3"], t["W2"], y, ctx, k=k)
            if bwd:
                b.grouter_moe_bwd(plan, t["x"], None, t["W1"], t["W3"], t["W2"], t["dY"], ctx, dX, dW1, dW3, dW2, scr,
                                  k=k)

    for _ in range(args.warmup):
        step()
    b.grouter_plan_status(plan)
    torch.cuda.synchronize()
    b.grouter_timing_enable(not args.no_kernel_events)
    b.grouter_timing_read()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # on the stream the steps run on
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per_step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    b.grouter_timing_enable(False)
    phases = b.grouter_timing_read()
    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    # The same step replayed from a HIP graph (no per-kernel events, no launch gaps): extra information only,
    # `value` above stays the eagerly launched, event-instrumented step.
    # (extras never cost the main line: a failure in one of them is reported in its place)
    graph_replay = None
    if args.calibration_copy_mib == 0:
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
            for _ in range(3):
                graph.replay()
            torch.cuda.synchronize()
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            g0.record()
            for _ in range(args.steps):
                graph.replay()
            g1.record()
            torch.cuda.synchronize()
            g_ms = g0.elapsed_time(g1) / args.steps
            graph_replay = {"ms_per_step": round(g_ms, 4),
                            "tflops": round(wl.flops(T, d, f, k, bwd) * n_layers / (g_ms * 1e-3) / 1e12, 2)}
            del graph
        except Exception as ex:  # noqa: BLE001
            graph_replay = {"error": repr(ex)[:200]}

    # The row gather / weighted scatter kernels no longer run inside the step (the GEMMs read x and dY through
    # the plan's row map); they remain entry points of their own and are timed here, apart from the step.
    standalone = None
    if args.calibration_copy_mib == 0:
        try:
            rows = torch.empty((T * k, d), dtype=torch.bfloat16, device=dev)
            b.grouter_timing_enable(True)
            b.grouter_timing_read()
            for _ in range(10):
                b.grouter_permute(plan, T, k, E, layers[0]["x"], None, rows)
                b.grouter_permute(plan, T, k, E, layers[0]["x"], gw, rows)
            torch.cuda.synchronize()
            b.grouter_timing_enable(False)
            ph = b.grouter_timing_read()
            standalone = {}
            for name, label in (("permute", "permute (rows of x into expert-sorted order)"),
                                ("dO", "permute with gate weights")):
                ms, cnt = ph[name]
                amount = phase_work(T, d, f, E, k)[name][1]
                gbs = amount / (ms / cnt * 1e-3) / 1e9
                standalone[name] = {"what": label, "avg_ms": round(ms / cnt, 5), "gbs": round(gbs, 1),
                                    "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4)}
            del rows
        except Exception as ex:  # noqa: BLE001
            standalone = {"error": repr(ex)[:200]}

    stats = None
    if not args.no_routing_stats and args.calibration_copy_mib == 0:
        try:
            stats = routing_stats_bench(b, wl, dev, reps=10, cpu_samples=64 if args.cpu_tokens > 0 else 0)
        except Exception as ex:  # noqa: BLE001
            stats = {"error": repr(ex)[:200]}

    calib = None
    if args.calibrate:
        try:
            calib = calibration_bench(b, dev, T * k, d, f)
        except Exception as ex:  # noqa: BLE001
            calib = {"error": repr(ex)[:200]}

    flop_step = wl.flops(T, d, f, k, bwd) * n_layers
    ms_per_step = elapsed / args.steps * 1e3
    tflops = flop_step / (elapsed / args.steps) / 1e12
    work = phase_work(T, d, f, E, k)
    per_phase = {}
    gemm_ms = gemm_flop = 0.0
    for name, (ms, cnt) in phases.items():
        if cnt == 0:
            continue
        avg_ms = ms / cnt
        entry = {"avg_ms": round(avg_ms, 5), "launches": cnt}
        if name in work:
            kind, amount = work[name]
            if kind == "mfma":
                entry["tflops"] = round(amount / (avg_ms * 1e-3) / 1e12, 2)
                entry["frac_mfma_peak"] = round(entry["tflops"] / PEAK_BF16_TFLOPS, 4)
                gemm_ms += ms
                gemm_flop += amount * cnt
            else:
                entry["gbs"] = round(amount / (avg_ms * 1e-3) / 1e9, 1)
                entry["frac_hbm_peak"] = round(entry["gbs"] / PEAK_HBM_GBS, 4)
        per_phase[name] = entry
    roofline = None
    gemm = {n: e for n, e in per_phase.items() if "tflops" in e}
    if gemm:
        dom = max(gemm, key=lambda n: phases[n][0])
        roofline = {"bound": "mfma", "kernel": dom, "achieved": gemm[dom]["tflops"], "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(gemm[dom]["tflops"] / PEAK_BF16_TFLOPS, 4),
                    "traffic": measured_traffic(dom) if args.config == 3 else None,
                    "avg_launch_ms": gemm[dom]["avg_ms"],
                    "all_gemm_phases": {"tflops": round(gemm_flop / (gemm_ms * 1e-3) / 1e12, 2),
                                        "frac": round(gemm_flop / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                                        "ms_per_step": round(gemm_ms / args.steps, 4)}}

    cpu = None
    if args.cpu_tokens > 0:
        try:
            tok_s, dt, cores = cpu_baseline(cfg, idx, gates, layers[0], args.cpu_tokens)
            per_tok = wl.flops(1, d, f, k, bwd)
            cpu = {"value": round(tok_s * per_tok / 1e12, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                   "tokens_per_s": round(tok_s, 2), "seconds": round(dt, 2),
                   "sample": f"{args.cpu_tokens} of {T} tokens of configuration {args.config}, forward + backward "
                             f"(fp32 oracle, every expert those tokens touch)"}
        except Exception as ex:  # noqa: BLE001
            cpu = {"error": repr(ex)[:200], "kind": "oracle"}

    out = {
        "metric": "expert-layer fwd+bwd TFLOP/s and tokens/s at 1 MI355X; % bf16 MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(per_step_ms[len(per_step_ms) // 2], 4),
        "ms_per_step_min": round(per_step_ms[0], 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"configs[{args.config}]: T={T}, d_model={d}, d_ff={f}, E={E}, top-{k}, "
                               f"{cfg['routing']} routing, {'fwd+bwd' if bwd else 'fwd'}"
                               f"{', %d layers on one plan' % n_layers if n_layers > 1 else ''}; plan rebuilt every step",
                   "T": T, "d_model": d, "d_ff": f, "E": E, "k": k},
        "tokens_per_s": round(T * n_layers / (elapsed / args.steps), 1),
        "frac_mfma_peak_whole_step": round(tflops / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline, "cpu_baseline": cpu, "phases": per_phase, "graph_replay": graph_replay,
        "gather_kernels_standalone": standalone,
        "routing_stats": stats,
    }
    if calib is not None:
        out["calibration"] = calib
    print(json.dumps(out))


if __name__ == "__main__":
    main()
