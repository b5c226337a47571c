#!/usr/bin/env python3
"""Benchmark of the Adaptive Sampling hot path on one MI355X.

One step = one pass of the whole path (k-means sweep over every k, knee selection, centroid
snap, Sample Synthesis + dedupe) over one batch of synthetic tuning tasks that is already
resident in HBM.  Prints ONE JSON line.

value            distance evaluations the sweep really executed (rows x k x labelling passes run,
                 per (task, k); a unit stops at the pass that changes no label, which leaves its
                 results those of the full iteration) per second of the whole step;
nominal_*        the same with the fixed-length count rows x sum(k) x (Lloyd steps + 1), i.e. the
                 work a kernel without the stop would do for the same results;
roofline         executed evaluations x (2d + 2) flops over the median duration of the sweep call
                 (HIP events on the launch stream, one pair per step) against the peak of the unit
                 the dominant kernel runs on; the kernel's name comes from the library;
cpu_baseline     the CPU oracle timed on a sample of the same workload, and its outputs compared
                 with the GPU outputs of the timed launches (parity_checked_tasks / parity_ok).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# published MI355X peaks used for the roofline fractions
PEAK_FP32_VECTOR_TFLOPS = 157.3
PEAK_F16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0


def executed_evals(wl, passes):
    """rows x k x passes run, summed over (task, k)."""
    import numpy as np
    sizes = np.diff(wl.task_off).astype(np.float64)
    ks = np.asarray(wl.ks, dtype=np.float64)
    return float((sizes[:, None] * ks[None, :] * passes.astype(np.float64)).sum())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--cfg", type=int, default=5, help="workload number 1..5 (default: the full-model sweep)")
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-tasks", type=int, default=48, help="tasks of the workload the oracle is timed on (about 13 s)")
    ap.add_argument("--knee-chunk", type=int, default=8,
                    help="also time the sweep that stops at the knee, in chunks of this many k (0 = skip)")
    ap.add_argument("--no-wide-knobs", dest="wide_knobs", action="store_false",
                    help="skip the timing of the two-byte-knob path")
    ap.add_argument("--no-large-single", dest="large_single", action="store_false",
                    help="skip the timing of the large single clustering (the streaming kernels)")
    ap.add_argument("--sweep-flags", type=int, default=0,
                    help="flags of cham_kmeans_sweep for the timed workload (8 = CHAM_F_NO_MFMA: the vector kernel)")
    ap.add_argument("--wide-flags", type=int, default=0,
                    help="flags of the sweep over the two-byte workload (8 = CHAM_F_NO_MFMA: the vector kernel)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain 1 GiB device copy (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); nothing here uses a second GPU.",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2001_08743_amd import binding, workloads

    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": 1 << 30, "copies": 3}), flush=True)
        return
    wl = workloads.make_config(args.cfg, 0, scale=args.scale)
    dw = binding.DeviceWorkload(wl, "cuda:0")
    dw.build_visited()

    # all outputs and workspaces are allocated once, outside the timed region
    first = dw.run(flags=args.sweep_flags)
    bufs = dict(sweep={k: first["sweep"][k] for k in ("centroids", "counts", "inertia", "status")},
                sweep_ws=first["sweep"]["workspace"], chosen=first["chosen"],
                snap={k: first["snap"][k] for k in ("labels_sel", "pick_row", "pick_cfg")},
                snap_ws=first["snap"]["workspace"],
                synth={k: first["synth"][k] for k in ("out_cfg", "out_flag", "out_count")},
                synth_ws=first["synth"]["workspace"])
    bufs["sweep"]["labels"] = None
    bufs["sweep"]["trace"] = None
    torch.cuda.synchronize()

    def step(ev=None):
        b = bufs
        if ev is not None:
            ev[0].record()
        sw = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, flags=args.sweep_flags,
                                       out=b["sweep"], workspace=b["sweep_ws"])
        if ev is not None:
            ev[1].record()
        chosen = binding.cham_select_k(sw["inertia"], sw["status"], wl.threshold, chosen=b["chosen"])
        sn = binding.cham_snap_centroids(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, chosen, sw["centroids"],
                                         out=b["snap"], workspace=b["snap_ws"])
        binding.cham_synthesize(dw.X, dw.ld, dw.d, wl.task_off, wl.cards, dw.valid, wl.ks, chosen,
                                sn["labels_sel"], sn["pick_row"], sn["pick_cfg"], dw.visited,
                                task_salt=wl.salts, out=b["synth"], workspace=b["synth_ws"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    nominal = wl.nominal_evals()
    passes = binding.cham_sweep_passes(bufs["sweep_ws"], dw.ld, dw.d, wl.task_off, wl.ks,
                                       flags=args.sweep_flags).cpu().numpy()
    executed = executed_evals(wl, passes)
    value = executed / (ms_per_step * 1e-3)
    sweep_times = sorted(a.elapsed_time(b) for a, b in events)
    sweep_ms = float(np.median(sweep_times))
    # Dominant kernel = the sweep kernel the library picks for this shape.  Algorithmic work per distance
    # evaluation: d multiply-adds of the expanded form plus the bias add and the compare = 2d + 2 flops.
    # The matrix-core kernels run the contraction in f16 (hi/lo split), so they are priced against the dense
    # f16 MFMA peak; the vector kernel against the fp32 vector peak.
    path = binding.cham_sweep_path(dw.ld, dw.d, wl.task_off, wl.ks, flags=args.sweep_flags)
    kernel = binding.cham_sweep_path_kernel(path)
    uses_mfma = path in (0, 1)
    flops_per_eval = 2 * wl.d + 2
    achieved_tflops = executed * flops_per_eval / (sweep_ms * 1e-3) / 1e12
    nominal_tflops = nominal * flops_per_eval / (sweep_ms * 1e-3) / 1e12
    peak = PEAK_F16_MFMA_TFLOPS if uses_mfma else PEAK_FP32_VECTOR_TFLOPS
    # HBM traffic of the sweep kernel as the launch shape implies it (every unit reads its task's packed
    # rows once, 2 bytes per padded knob; centroids, counts and working labels are written once); the
    # counter figures of the rocprofv3 --pmc runs are under profiles/ and cannot be read from in here.
    dk = 16 if wl.d <= 15 else 32
    sizes = np.diff(wl.task_off).astype(np.float64)
    traffic_model = float(sizes.sum() * len(wl.ks) * (dk * 2 + 1) + wl.T * sum(wl.ks) * (wl.d * 8 + 4)) \
        if path == 0 else None
    roofline = dict(bound="mfma" if uses_mfma else "alu", achieved=round(achieved_tflops, 3), peak=peak,
                    unit="TFLOP/s", frac=round(achieved_tflops / peak, 4), traffic=None,
                    traffic_model=traffic_model, kernel=kernel,
                    kernel_ms=round(sweep_ms, 3), kernel_ms_min=round(sweep_times[0], 3),
                    flops_per_eval=flops_per_eval,
                    evals_counted="executed (rows x k x passes run)",
                    nominal_achieved=round(nominal_tflops, 3), nominal_frac=round(nominal_tflops / peak, 4),
                    frac_of_fp32_vector_peak=round(achieved_tflops / PEAK_FP32_VECTOR_TFLOPS, 4))

    # Not part of the metric: the same workload through the sweep that stops at the knee (Algorithm 1's
    # loop as printed), in chunks of --knee-chunk values of k.
    knee = None
    if args.knee_chunk > 0:
        kout = binding.cham_kmeans_sweep_knee(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter,
                                              threshold=wl.threshold, chunk=args.knee_chunk)
        torch.cuda.synchronize()
        kbuf = {k: kout[k] for k in ("centroids", "counts", "inertia", "status", "chosen")}
        kbuf["labels"] = None
        kbuf["trace"] = None
        kev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
        for e0, e1 in kev:
            e0.record()
            binding.cham_kmeans_sweep_knee(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, threshold=wl.threshold,
                                           chunk=args.knee_chunk, out=kbuf, workspace=kout["workspace"])
            e1.record()
        torch.cuda.synchronize()
        knee_ms = float(np.median([a.elapsed_time(b) for a, b in kev]))
        kpasses = binding.cham_sweep_passes(kout["workspace"], dw.ld, dw.d, wl.task_off, wl.ks).cpu().numpy()
        kexec = executed_evals(wl, kpasses)
        st = kout["status"].cpu().numpy()
        knee = dict(chunk=args.knee_chunk, sweep_ms=round(knee_ms, 3), executed_evals=kexec,
                    units_run=int((st == 0).sum()), units_total=int(st.size),
                    executed_evals_per_s=round(kexec / (knee_ms * 1e-3), 1))

    # Not part of the metric either: the visited set as a device table (what the outer loop of the search
    # keeps between calls): insert the workload's visited hashes into a table at load <= 1/4.
    vtab = None
    if dw.visited is not None and dw.visited.numel() > 0:
        n_h = int(dw.visited.numel())
        slots = 1 << max(4, int(np.ceil(np.log2(4 * n_h))))
        table = torch.empty(slots, dtype=torch.int64, device="cuda:0")
        tev = []
        for _ in range(3):
            binding.cham_visited_table_clear(table)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            binding.cham_visited_table_insert_hashes(table, dw.visited)
            e1.record()
            tev.append((e0, e1))
        torch.cuda.synchronize()
        ins_ms = min(a.elapsed_time(b) for a, b in tev)
        vtab = dict(slots=slots, inserted=n_h, insert_ms=round(ins_ms, 4),
                    inserts_per_s=round(n_h / (ins_ms * 1e-3), 1))

    # The configuration updater that feeds the path (128 episodes x 500 steps, the paper's values), with the
    # trajectory's distinct configurations collected on the device.
    g = torch.Generator(device="cpu").manual_seed(1)
    B_u, S_u = 128, 500
    cards_u = torch.from_numpy(wl.cards[0].astype(np.int16)).to("cuda:0")
    theta_u = torch.zeros((B_u, wl.d), dtype=torch.uint8, device="cuda:0")
    act_u = torch.randint(-1, 2, (S_u, B_u, wl.d), generator=g, dtype=torch.int8).to("cuda:0")
    seen_u = torch.empty(1 << 18, dtype=torch.int64, device="cuda:0")
    uniq_u = torch.empty((B_u * S_u, wl.d), dtype=torch.uint8, device="cuda:0")
    n_u = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    best_u = None
    for _ in range(3):
        binding.cham_visited_table_clear(seen_u)
        theta_u.zero_()
        n_u.zero_()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        binding.cham_update_configs(theta_u, act_u, cards_u, salt=0, seen_table=seen_u, unique_rows=uniq_u, n_unique=n_u)
        e1.record()
        torch.cuda.synchronize()
        t_u = e0.elapsed_time(e1)
        best_u = t_u if best_u is None else min(best_u, t_u)
    updater = dict(episodes=B_u, steps=S_u, d=wl.d, ms=round(best_u, 4), distinct=int(n_u.item()),
                   config_steps_per_s=round(B_u * S_u / (best_u * 1e-3), 1))

    def side_workload(ww, reps=5, flags=0):
        """Whole path on another workload: median step time and evaluation rates."""
        dww = binding.DeviceWorkload(ww, "cuda:0")
        dww.build_visited()
        wfirst = dww.run(flags=flags)
        wbufs = dict(sweep={k: wfirst["sweep"][k] for k in ("centroids", "counts", "inertia", "status")},
                     sweep_ws=wfirst["sweep"]["workspace"], chosen=wfirst["chosen"],
                     snap={k: wfirst["snap"][k] for k in ("labels_sel", "pick_row", "pick_cfg")},
                     snap_ws=wfirst["snap"]["workspace"],
                     synth={k: wfirst["synth"][k] for k in ("out_cfg", "out_flag", "out_count")},
                     synth_ws=wfirst["synth"]["workspace"])
        wbufs["sweep"]["labels"] = None
        wbufs["sweep"]["trace"] = None
        torch.cuda.synchronize()
        wev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e0, e1 in wev:
            e0.record()
            dww.run(bufs=wbufs, flags=flags)
            e1.record()
        torch.cuda.synchronize()
        w_ms = float(np.median([a.elapsed_time(b) for a, b in wev]))
        wp = binding.cham_sweep_passes(wbufs["sweep_ws"], dww.ld, dww.d, ww.task_off, ww.ks).cpu().numpy()
        return w_ms, executed_evals(ww, wp), ww.nominal_evals()

    # Design spaces with two-byte knobs and more than 32 knobs (the *_u16 entry points): 64 tasks x 2048
    # configurations x 40 knobs with cardinalities up to 600, k = 2..32, 30 Lloyd steps; whole path.
    wide = None
    if args.wide_knobs:
        ww = workloads.wide_space(0)
        w_ms, w_exec, w_nom = side_workload(ww, flags=args.wide_flags)
        wide = dict(workload=f"{ww.name}: T={ww.T} tasks x N={ww.n_total // ww.T} rows x d={ww.d} two-byte knobs "
                             f"(cardinalities up to {int(ww.cards.max())}), k={ww.ks[0]}..{ww.ks[-1]}, "
                             f"{ww.n_iter} Lloyd steps + final pass, visited={ww.n_visited}",
                    ms_per_step=round(w_ms, 3), evals_per_step=w_exec, evals_counted="executed",
                    nominal_evals_per_step=w_nom, evals_per_s=round(w_exec / (w_ms * 1e-3), 1),
                    frac_of_fp32_vector_peak=round(w_exec * (2 * ww.d + 2) / (w_ms * 1e-3) / 1e12
                                                   / PEAK_FP32_VECTOR_TFLOPS, 4))
        # cardinalities of at most 2048: the harness promises values below 2048 and the sweep may run on the
        # matrix cores (the library says which kernel it is)
        w_promise = args.wide_flags | (binding.F_VALUES_BELOW_2048 if int(ww.cards.max()) <= 2048 else 0)
        w_path = binding.cham_sweep_path_u16((ww.n_total + 63) // 64 * 64, ww.d, ww.task_off, ww.ks, flags=w_promise)
        wide["kernel"] = binding.cham_sweep_path_kernel(w_path)
        if w_path == 0:
            wide["frac_of_f16_mfma_peak"] = round(w_exec * (2 * ww.d + 2) / (w_ms * 1e-3) / 1e12
                                                  / PEAK_F16_MFMA_TFLOPS, 4)

    # The large single clustering (1 048 576 configurations x 16 knobs, k in {16..256}, 20 Lloyd steps):
    # tasks beyond one workgroup run the streaming matrix-core kernels.
    large = None
    if args.large_single and args.cfg != 4:
        wl4 = workloads.make_config(4, 0)
        l_ms, l_exec, l_nom = side_workload(wl4, reps=3)
        p4 = binding.cham_sweep_path((wl4.n_total + 63) // 64 * 64, wl4.d, wl4.task_off, wl4.ks)
        large = dict(workload=f"{wl4.name}: N={wl4.n_total} rows x d={wl4.d}, k={list(wl4.ks)}, {wl4.n_iter} Lloyd steps "
                              f"+ final pass", kernel=binding.cham_sweep_path_kernel(p4),
                     ms_per_step=round(l_ms, 3), evals_per_step=l_exec, evals_per_s=round(l_exec / (l_ms * 1e-3), 1),
                     frac_of_f16_mfma_peak=round(l_exec * (2 * wl4.d + 2) / (l_ms * 1e-3) / 1e12
                                                 / PEAK_F16_MFMA_TFLOPS, 4))

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        n_tasks = min(args.cpu_tasks, wl.T)
        sub = wl.subset(range(n_tasks))
        vis = workloads.finalize_visited(oracle.visited_hashes(wl), wl.visited_raw, wl.n_visited)
        c0 = time.perf_counter()
        ref = oracle.pipeline(sub, vis)
        c1 = time.perf_counter()
        # the oracle's outputs for these tasks against what the timed launches left in the output buffers
        ksum, kmax = int(sum(wl.ks)), max(wl.ks)
        n_rows = int(wl.task_off[n_tasks])
        sw, sn, sy = bufs["sweep"], bufs["snap"], bufs["synth"]
        checks = dict(
            status=np.array_equal(sw["status"][:n_tasks].cpu().numpy(), ref["status"]),
            counts=np.array_equal(sw["counts"][:n_tasks].cpu().numpy(), ref["counts"]),
            centroids=np.array_equal(sw["centroids"][:n_tasks].cpu().numpy(), ref["centroids"]),
            inertia=bool(np.allclose(sw["inertia"][:n_tasks].cpu().numpy(), ref["inertia"], rtol=1e-11, atol=0)),
            chosen=np.array_equal(bufs["chosen"][:n_tasks].cpu().numpy(), ref["chosen_idx"]),
            labels_sel=np.array_equal(sn["labels_sel"][:n_rows].cpu().numpy().astype(np.int32), ref["labels_sel"]),
            pick_row=np.array_equal(sn["pick_row"][:n_tasks].cpu().numpy().astype(np.int64), ref["pick_row"]),
            pick_cfg=np.array_equal(binding.knobs_to_host(sn["pick_cfg"][:n_tasks]), ref["pick_cfg"]),
            out_cfg=np.array_equal(binding.knobs_to_host(sy["out_cfg"][:n_tasks]), ref["out_cfg"]),
            out_flag=np.array_equal(sy["out_flag"][:n_tasks].cpu().numpy(), ref["out_flag"]),
            out_count=np.array_equal(sy["out_count"][:n_tasks].cpu().numpy(), ref["out_count"]))
        assert ksum and kmax
        cpu = dict(value=round(sub.nominal_evals() / (c1 - c0), 1), unit="evals/s", cores=oracle.num_threads(),
                   kind="oracle", seconds=round(c1 - c0, 2),
                   sample=f"tasks 0..{n_tasks - 1} of {wl.T} ({sub.nominal_evals():.3e} of {nominal:.3e} evals; the "
                          f"oracle runs every pass), whole path, fp64, OpenMP over (task,k) units",
                   parity_checked_tasks=n_tasks, parity_ok=bool(all(checks.values())),
                   parity_failed=[k for k, v in checks.items() if not v])

    line = {
        "metric": "point-centroid distance evals/sec for full k-sweep",
        "value": round(value, 1), "unit": "evals/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: T={wl.T} tasks x N={wl.n_total // wl.T} rows x d={wl.d}, "
                               f"k={wl.ks[0]}..{wl.ks[-1]} ({len(wl.ks)} values), {wl.n_iter} Lloyd steps + final pass, "
                               f"visited={wl.n_visited}, threshold={wl.threshold}",
                   "evals_per_step": executed, "evals_counted": "executed",
                   "nominal_evals_per_step": nominal, "nominal_evals_per_s": round(nominal / (ms_per_step * 1e-3), 1),
                   "mean_passes_run": round(float(passes.mean()), 2), "passes_nominal": wl.n_iter + 1,
                   "sweep_ms_median": round(sweep_ms, 3)},
        "roofline": roofline, "cpu_baseline": cpu, "knee_sweep": knee,
        "visited_table": vtab, "config_updater": updater, "wide_knobs": wide, "large_single": large,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
