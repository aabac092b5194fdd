#!/usr/bin/env python3
"""Benchmark of the fused projection + cross-entropy path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama3_8b]

A step is one flce_forward + one flce_backward (every kernel of the path) over one
batch of seeded synthetic input that is already resident in HBM.  Prints ONE JSON
line: whole-job tokens/s, the roofline figures of the dominant kernel class (timed
live with HIP events on the stream the kernels run on) and the CPU oracle timed on
a bounded row sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2516.6      # MI355X dense bf16: 256 CU x 4096 flop/clk x 2.4 GHz
F32_MFMA_PEAK_TFLOPS = 157.3

# Plain-ALU peaks of MI355X from its unit counts and clock: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations
# per second for ordinary fp32 vector instructions (an fma counts 2 flops: 78.6 T fma/s = 157.3 TFLOP/s), a quarter
# of that for the transcendental unit (v_exp_f32).
VALU_LANE_OPS_PER_S = 256 * 4 * 16 * 2.4e9
EXP_PER_S = VALU_LANE_OPS_PER_S / 4


def device_facts():
    """CU count and clocks of the GPU as the box reports them (rocminfo's record of the first GPU agent)."""
    import subprocess
    facts = {}
    try:
        txt = subprocess.run(["rocminfo"], capture_output=True, text=True, timeout=30).stdout
    except Exception:
        return facts
    for agent in txt.split("Agent ")[1:]:
        if "Device Type:             GPU" not in agent:
            continue
        for key, name in (("Marketing Name:", "marketing_name"), ("Name:", "gfx"), ("Compute Unit:", "compute_units"),
                          ("Max Clock Freq. (MHz):", "max_engine_clock_MHz"), ("SIMDs per CU:", "simds_per_cu"),
                          ("Wavefront Size:", "wavefront_size")):
            for line in agent.splitlines():
                if line.strip().startswith(key):
                    v = line.split(":", 1)[1].strip().split("(")[0].strip()
                    facts[name] = int(v) if v.isdigit() else v
                    break
        break
    return facts


def measured_traffic(workload, plan):
    """Fabric-side bytes per launch of each kernel class, from profiles/<workload>_pmc.txt (rocprofv3 FETCH_SIZE and
    WRITE_SIZE runs of this script, scaled by the same counters' reading for a plain copy).  The summary records
    the launch plan it was taken on; if that is not the plan of this run the figures do not apply: returns ({},
    reason) and the caller reports null."""
    path = os.path.join(ROOT, "profiles", f"{workload}_pmc.txt")
    if not os.path.exists(path):
        return {}, f"no {os.path.relpath(path, ROOT)}"
    rec_plan, out = None, {}
    for line in open(path):
        if line.startswith("plan: "):
            rec_plan = line[len("plan: "):].strip()
        elif line.startswith("traffic_bytes_per_launch "):
            f = line.split()
            kv = dict(t.split("=") for t in f[2:])
            out[f[1]] = float(kv["fetch"]) + float(kv["write"])
    if rec_plan != plan:
        return {}, f"{os.path.relpath(path, ROOT)} was taken on another plan ({rec_plan!r}, now {plan!r})"
    return out, None


def cpu_baseline(wl, x, rows):
    """The oracle as it stands, on the first `rows` rows of the workload (all of W)."""
    import numpy as np
    from oracle import flce_oracle as O
    from paper_2511_17599_amd import inputs as I
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    H = I.to_f64(x["H"][:rows])
    W = I.to_f64(x["W"])
    y = x["y"][:rows]
    t0 = time.perf_counter()
    f = O.forward(H, W, y, wl.ignore_index, wl.reduction)
    b = O.backward(H, W, y, wl.ignore_index, wl.reduction)
    dt = time.perf_counter() - t0
    assert np.isfinite(f["loss"]) and np.isfinite(b["dW"]).all()
    return {"value": rows / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"fp64 forward+backward of the first {rows} of {wl.N} rows against all {wl.V} vocabulary rows, "
                      f"{dt:.1f} s wall"}, f


# The paper's own evaluation grid (Table 1 / Table 2): d = 4096, bf16, B*T x V, with its latency (ms) and memory
# (MB) for the fused kernels on an NVIDIA GB200 -- another machine, quoted as context.  Table 2 does not say
# what the latency covers; its size says forward only.
PAPER_TABLE2 = {  # (N, V): (canonical_ms, proposed_ms, canonical_MB, proposed_MB)
    (1024, 32768): (0.73, 0.69, 1064, 280), (1024, 65536): (1.40, 0.97, 2088, 536),
    (1024, 131072): (2.76, 1.27, 4136, 1048), (1024, 262144): (5.46, 1.83, 8232, 2072),
    (4096, 32768): (1.66, 1.16, 1904, 304), (4096, 65536): (3.34, 1.69, 3696, 561),
    (4096, 131072): (6.78, 2.86, 7280, 1073), (4096, 262144): (13.70, 5.22, 14448, 2099),
    (8192, 32768): (2.93, 1.70, 3024, 337), (8192, 65536): (6.08, 2.90, 5840, 593),
    (8192, 131072): (13.25, 5.58, 11472, 1107), (8192, 262144): (27.77, 10.79, 22736, 2133),
    (16384, 32768): (5.62, 3.43, 5264, 401), (16384, 65536): (12.41, 6.61, 10128, 659),
    (16384, 131072): (26.67, 13.20, 19856, 1173), (16384, 262144): (50.15, 25.43, 39312, 2203),
    (32768, 32768): (11.42, 7.00, 9744, 531), (32768, 65536): (25.64, 13.80, 18704, 790),
    (32768, 131072): (50.24, 27.06, 36624, 1307), (32768, 262144): (96.52, 53.61, 72464, 2342),
}


def sweep_paper_grid(steps, warmup):
    """Forward-only and forward+backward latency and memory over the paper's grid; one JSON line per point."""
    import torch
    from paper_2511_17599_amd import binding as B
    from paper_2511_17599_amd import inputs as I
    from paper_2511_17599_amd.runner import Session, to_device

    d = 4096
    torch.cuda.set_device(0)
    Ns = sorted({k[0] for k in PAPER_TABLE2})
    Vs = sorted({k[1] for k in PAPER_TABLE2})
    Hfull = to_device(I.f32_to_bf16_bits(I.normal_f32(2001, I.STREAM_H, max(Ns) * d, 1.0)).reshape(max(Ns), d), "cuda")
    for V in Vs:
        W = to_device(I.f32_to_bf16_bits(I.normal_f32(2001, I.STREAM_W, V * d, 0.02)).reshape(V, d), "cuda")
        for N in Ns:
            y = I.targets_uniform(2001 + N, N, V)
            s = Session(N, d, V, "bf16", "mean", -100, Hfull[:N], W, y)

            def timed(fn):
                for _ in range(warmup):
                    fn()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    fn()
                torch.cuda.synchronize()
                return (time.perf_counter() - t0) / steps * 1e3

            fwd_ms = timed(lambda: s.forward())
            both_ms = timed(lambda: (s.forward(), s.backward()))
            st, nv = s.device_status()
            assert st == B.FLCE_OK and nv == N
            ref = PAPER_TABLE2[(N, V)]
            fwd_bytes = (N + V) * d * 2 + N * 8 + N * 4 + 4 + s.fwd_bytes
            print(json.dumps({
                "sweep": "paper_table2", "N": N, "d": d, "V": V, "dtype": "bf16",
                "forward_ms": fwd_ms, "forward_tflops_2NdV": 2.0 * N * d * V / fwd_ms / 1e9,
                "forward_backward_ms": both_ms, "forward_backward_tflops_8NdV": 8.0 * N * d * V / both_ms / 1e9,
                "forward_memory_MiB": fwd_bytes / 2**20, "forward_backward_memory_MiB": s.tensor_bytes() / 2**20,
                "naive_fp32_logits_MiB": N * V * 4 / 2**20, "loss": float(s.loss.item()),
                "paper_gb200": {"canonical_ms": ref[0], "proposed_ms": ref[1], "canonical_MB": ref[2],
                                "proposed_MB": ref[3]}}), flush=True)
            del s
        del W


def probe_main_loop(steps, warmup):
    """What the pieces of the tuned main loop sustain on their own (flce_probe): one JSON line per mode and K."""
    import torch
    from paper_2511_17599_amd import binding as B

    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
    g = torch.Generator(device="cuda").manual_seed(3001)
    wgs = 256
    for k, a_rows, b_rows, tiles in ((4096, 32768, 8192, 32), (768, 50176, 4096, 96)):
        A = (torch.randn(a_rows, k, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
        Bm = torch.randn(b_rows, k, device="cuda", generator=g).to(torch.bfloat16)
        BT = Bm.t().contiguous()
        sink = torch.empty(2 * wgs * 256, dtype=torch.float32, device="cuda")
        st = torch.cuda.current_stream()
        for mode, name in enumerate(B.PROBE_MODES):
            ms = []
            # the half-height-tile modes: twice the workgroups (two per CU) for the same total work
            launch_wgs = 2 * wgs if name.startswith("half") else wgs
            for it in range(warmup + steps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(st)
                rc = B.flce_probe(mode, A, Bm, BT, a_rows, b_rows, k, launch_wgs, tiles, sink, st)
                e1.record(st)
                assert rc == B.FLCE_OK, B.flce_status_string(rc)
                e1.synchronize()
                if it >= warmup:
                    ms.append(e0.elapsed_time(e1))
            ms.sort()
            med = ms[len(ms) // 2]
            flops = 2.0 * 256 * 256 * k * tiles * wgs
            lds_bytes = 2.0 * 256 * k * 2 * tiles * wgs                # operand bytes brought into LDS
            line = {"probe": name, "k_elems": k, "workgroups": launch_wgs, "tiles_per_workgroup": tiles,
                    "ms_median": med, "ms_min": ms[0], "device": props.name, "compute_units": props.multi_processor_count}
            if name.startswith("data"):
                line["global_to_lds_TBps"] = lds_bytes / (med * 1e-3) / 1e12
                line["mfma_time_equivalent_tflops"] = flops / (med * 1e-3) / 1e12
            else:
                line["tflops"] = flops / (med * 1e-3) / 1e12
                line["frac_of_nominal_peak"] = line["tflops"] / BF16_MFMA_PEAK_TFLOPS
            print(json.dumps(line), flush=True)
        del A, Bm, BT


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama3_8b")
    ap.add_argument("--oracle-rows", type=int, default=None, help="rows of the CPU baseline sample (0 = skip)")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket launches with events")
    ap.add_argument("--copy-calibration", type=int, default=0,
                    help="bytes of one plain device copy issued before the timed region (a yardstick for "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--path", choices=["recompute", "partial_grads"], default="recompute",
                    help="recompute: forward (Alg. 1) + backward (Alg. 2), the benchmarked path; partial_grads: "
                         "forward with partial gradients (Alg. 3) + scaling (Alg. 4)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replays (launch-bound shapes); implies "
                         "--no-profile")
    ap.add_argument("--probe", action="store_true",
                    help="instead of the benchmark line: the rates of the matrix pipe alone, of the bare tuned main "
                         "loop and of its data path alone (flce_probe)")
    ap.add_argument("--sweep", choices=["paper_table2"], default=None,
                    help="instead of the benchmark line: latency and memory over the paper's evaluation grid")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures the one-GPU kernel path only; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.sweep:
        sweep_paper_grid(args.steps, args.warmup)
        return
    if args.probe:
        probe_main_loop(args.steps, args.warmup)
        return

    import numpy as np
    import torch
    from paper_2511_17599_amd import binding as B
    from paper_2511_17599_amd import inputs as I
    from paper_2511_17599_amd.runner import session_for

    wl = I.WORKLOADS[args.workload]
    torch.cuda.set_device(0)
    x = I.make_inputs(wl)
    torch.cuda.reset_peak_memory_stats()
    s = session_for(wl, x)

    def step():
        if args.path == "partial_grads":
            st = s.forward_with_grads()
            assert st == B.FLCE_OK, B.flce_status_string(st)
            st = s.scale()
        else:
            st = s.forward()
            assert st == B.FLCE_OK, B.flce_status_string(st)
            st = s.backward()
        assert st == B.FLCE_OK, B.flce_status_string(st)

    if args.copy_calibration:
        src = torch.empty(args.copy_calibration, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    run_step = step
    if args.graph:
        args.no_profile = True
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        run_step = graph.replay
        run_step()
        torch.cuda.synchronize()
    if not args.no_profile:
        B.flce_profile_enable(1)
    # The timed region: exactly `steps` steps between two synchronisations (ms_per_step is this wall clock).  Each
    # step is also bracketed by events on the stream the kernels run on, with one more after the forward, for
    # the median / minimum and the forward / backward split.
    stream = torch.cuda.current_stream()
    split = not args.graph and args.path == "recompute"
    marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record(stream)
        if split:
            st = s.forward()
            e[1].record(stream)
            st = st or s.backward()
            assert st == B.FLCE_OK, B.flce_status_string(st)
        else:
            run_step()
        e[2].record(stream)
        marks.append(e)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step_ms = sorted(e[0].elapsed_time(e[2]) for e in marks)
    fwd_ms = sorted(e[0].elapsed_time(e[1]) for e in marks) if split else None
    bwd_ms = sorted(e[1].elapsed_time(e[2]) for e in marks) if split else None
    med = lambda v: v[len(v) // 2]
    prof_ms, prof_n = {}, {}
    if not args.no_profile:
        _, prof_ms, prof_n = B.flce_profile_collect()
        B.flce_profile_enable(0)
    st, n_valid = s.device_status()
    assert st == B.FLCE_OK
    loss = float(s.loss.item())

    ms_per_step = dt / args.steps * 1e3
    flops = 8.0 * wl.N * wl.d * wl.V
    # what the kernels execute: the forward runs every row, the three backward contractions run the counted
    # rows only, in whole 256-row tiles
    rows_bwd = -(-n_valid // 256) * 256
    flops_executed = 2.0 * wl.d * wl.V * (-(-wl.N // 256) * 256) + 6.0 * wl.d * wl.V * rows_bwd
    tflops = flops / (ms_per_step * 1e-3) / 1e12
    peak = BF16_MFMA_PEAK_TFLOPS if wl.dtype == "bf16" else F32_MFMA_PEAK_TFLOPS

    # roofline of the dominant kernel class (largest share of the step)
    # nominal flops of each kernel class in units of N*d*V
    class_flops = {"fwd_tiles": 2.0, "recompute": 2.0, "contract_dW": 2.0, "contract_dH": 2.0}
    kernels = {}
    for k, c in class_flops.items():
        if prof_n.get(k):
            ms_step = prof_ms[k] / args.steps
            kernels[k] = {"ms_per_step": ms_step, "launches_per_step": prof_n[k] / args.steps,
                          "tflops": c * wl.N * wl.d * wl.V / (ms_step * 1e-3) / 1e12}
    for k in ("fwd_epilogue", "bwd_prep", "scale"):
        if prof_n.get(k):
            kernels[k] = {"ms_per_step": prof_ms[k] / args.steps, "launches_per_step": prof_n[k] / args.steps}
    plan = B.flce_plan_describe(wl.N, wl.d, wl.V, s.dt)
    traffic, why_not = measured_traffic(wl.name, plan)
    if why_not:
        print(f"bench.py: roofline.traffic is null: {why_not}", file=sys.stderr)
    roofline = None
    if kernels:
        dom = max(class_flops, key=lambda k: kernels.get(k, {}).get("ms_per_step", 0.0))
        a = kernels[dom]["tflops"]
        roofline = {"bound": "mfma", "kernel": dom, "achieved": a, "peak": peak, "unit": "TFLOP/s", "frac": a / peak,
                    "traffic": traffic.get(dom),
                    "flops_per_launch": class_flops[dom] * wl.N * wl.d * wl.V / kernels[dom]["launches_per_step"],
                    "avg_launch_ms": kernels[dom]["ms_per_step"] / kernels[dom]["launches_per_step"]}
    # The other roof of this path: the softmax work runs on the plain vector ALUs while the matrix pipe waits (one
    # wavefront per SIMD), so its time adds to the MFMA time instead of hiding behind it.  Per logit: one exponential
    # in the forward and one in the recompute, and about 10 ordinary vector instructions in each of the two.
    n_logits = float(wl.N) * wl.V
    alu_ms = (2.0 * n_logits / EXP_PER_S + 20.0 * n_logits / VALU_LANE_OPS_PER_S) * 1e3
    mfma_ms = flops / (peak * 1e12) * 1e3
    alu_roof = {"bound": "alu", "exp_per_step": 2.0 * n_logits, "vector_lane_ops_per_step": 20.0 * n_logits,
                "peak_exp_per_s": EXP_PER_S, "peak_vector_lane_ops_per_s": VALU_LANE_OPS_PER_S,
                "ms_at_alu_peak": alu_ms, "ms_at_mfma_peak": mfma_ms,
                "frac_of_step_at_peaks": {"alu": alu_ms / ms_per_step, "mfma": mfma_ms / ms_per_step}}
    props = torch.cuda.get_device_properties(0)
    device = {"name": props.name, "compute_units": props.multi_processor_count, "hbm_bytes": props.total_memory,
              "host_cores": os.cpu_count(), "rocminfo": device_facts()}

    rows = args.oracle_rows
    if rows is None:
        rows = max(16, min(wl.N, int(1.2e13 / (6.0 * wl.d * wl.V))))     # ~10-20 s of fp64 work
    base = None
    if rows > 0:
        base, f = cpu_baseline(wl, x, min(rows, wl.N))
        lse_gpu = s.lse[:len(f["lse"])].float().cpu().numpy()
        base["max_abs_lse_diff_vs_gpu"] = float(np.abs(lse_gpu - f["lse"]).max())

    out = {
        "metric": "fused linear-CE fwd+bwd tokens/sec", "value": wl.N / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": med(step_ms), "ms_per_step_min": step_ms[0],
        "forward_ms_median": med(fwd_ms) if split else None, "forward_ms_min": fwd_ms[0] if split else None,
        "backward_ms_median": med(bwd_ms) if split else None, "backward_ms_min": bwd_ms[0] if split else None,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "N": wl.N, "d": wl.d, "V": wl.V, "reduction": wl.reduction,
                   "targets": wl.targets, "ignore_frac": wl.ignore_frac, "seed": wl.seed, "path": args.path, "launch": "graph replay" if args.graph else "eager"},
        "tflops_8NdV": tflops, "frac_of_mfma_peak": tflops / peak,
        "tflops_executed": flops_executed / (ms_per_step * 1e-3) / 1e12,
        "frac_of_mfma_peak_executed": flops_executed / (ms_per_step * 1e-3) / 1e12 / peak,
        "flops_note": "8NdV counts the ignored rows too; the backward skips them (their rows of G are zero), "
                      "so executed flops are 2NdV + 6*rows_counted*d*V",
        "loss": loss, "n_valid": n_valid,
        "memory": {"peak_allocated_bytes": int(torch.cuda.max_memory_allocated()),
                   "path_tensor_bytes": int(s.tensor_bytes()), "workspace_bytes": int(s.ws.numel()),
                   "naive_fp32_logits_bytes": int(wl.naive_logits_bytes),
                   "peak_over_naive_logits": torch.cuda.max_memory_allocated() / wl.naive_logits_bytes,
                   "workspace_over_naive_logits": s.ws.numel() / wl.naive_logits_bytes},
        "roofline": roofline, "alu_roofline": alu_roof, "kernels": kernels, "cpu_baseline": base,
        "plan": plan, "device": device,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
