"""Benchmark of the SVD-Attention hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic users:
solar_svd_factorize (Gram, eigen-iteration, projection) followed by
solar_svd_attention in the sequence-softmax mode, inputs already resident in HBM.
Prints one JSON line: user-sequences/s, the roofline figure of the dominant kernel
(measured with HIP events inside the timed region) and the CPU oracle timed on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

WORKLOAD = "C3"
N_BUFFER_SETS = 3   # rotate inputs so that X is not served from the 256 MiB Infinity Cache

# HBM bytes per launch from `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` (see the summaries under
# profiles/ for the commands and the copy-kernel calibration); keyed by (workload, phase).
MEASURED_TRAFFIC = {
    # profiles/hbm_traffic_C3.txt: fetch + write bytes of one launch
    ("C3", "attention"): 99.6e6 + 32.8e6,
    ("C3", "gram"): 164.1e6 + 9.4e6,
    ("C3", "project"): 172.6e6 + 82.5e6,
}

PEAKS = {
    "hbm_GBps": 8000.0,
    "mfma_f32_TFLOPs": 157.3,
    "mfma_bf16_TFLOPs": 2500.0,
}


def cpu_baseline(w, n_users: int):
    """The oracle as it stands, one user per thread, on a bounded sample of the workload."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import oracle

    oracle.build()
    cores = max(1, min(n_users, os.cpu_count() or 1, 16))

    def one(b):
        X = w.X[b:b + 1]
        Q = w.Q[b:b + 1]
        L = w.lengths[b:b + 1]
        f = oracle.svd_factorize(X, w.r, L)
        O = oracle.svd_attention(Q, X, f["S"], f["V"], 1.0, 0, L)
        return O

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as pool:
        outs = list(pool.map(one, range(n_users)))
    dt = time.perf_counter() - t0
    return {
        "value": n_users / dt, "unit": "user-sequences/s", "cores": cores, "kind": "oracle",
        "sample": f"{n_users} users of {w.name} (factorize + mode-0 attention, double precision), "
                  f"one user per thread, {dt:.1f} s wall",
    }, np.concatenate(outs, axis=0)


def latency_sweep(w, steps: int):
    """Forward latency against the history length N at fixed B, M, d, r (Section "Forward-pass
    efficiency of attention"): softmax attention (the correctness-first dense reference kernel, not
    tuned), linear attention Q (X^T X), SVD-attention with the factorization inside and with the
    factors reused.  CPU figures: the oracle on one thread, one user, at the shorter lengths."""
    import numpy as np
    import torch
    from paper_2603_02561_amd import binding, synth
    from oracle import oracle

    def gpu_ms(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    rows = []
    for n in (1000, 2000, 5000, 10000, 20000):
        wl = synth.make_workload(f"sweep{n}", w.B, n, w.d, w.r, w.M, w.dtype, "spectrum", 1.0, 0.01,
                                 seed=4242 + n)
        db = binding.DeviceBatch(wl.X, wl.Q, wl.lengths, wl.r, wl.dtype == synth.BF16)
        row = {"N": n, "B": w.B, "M": w.M, "d": w.d, "r": w.r}

        def svd_full():
            db.factorize()
            db.attention(1.0, binding.SOLAR_ATTN_SEQ_SOFTMAX)
        row["gpu_ms_svd_attention"] = gpu_ms(svd_full, steps)
        row["gpu_ms_svd_attention_factors_reused"] = gpu_ms(
            lambda: db.attention(1.0, binding.SOLAR_ATTN_SEQ_SOFTMAX), steps)
        row["gpu_ms_linear_attention"] = gpu_ms(lambda: db.linear(1.0), steps)
        row["gpu_ms_softmax_attention_reference_kernel"] = gpu_ms(lambda: db.dense(1.0), max(1, steps // 5))
        if n <= 2000:
            X1, Q1 = wl.X[:1], wl.Q[:1]
            t0 = time.perf_counter()
            f = oracle.svd_factorize(X1, wl.r)
            oracle.svd_attention(Q1, X1, f["S"], f["V"], 1.0, 0)
            t1 = time.perf_counter()
            oracle.linear_attention(Q1, X1, 1.0)
            t2 = time.perf_counter()
            oracle.dense_attention(Q1, X1, 1.0)
            t3 = time.perf_counter()
            row["cpu_1thread_ms_per_user"] = {"svd_attention_oracle": (t1 - t0) * 1e3,
                                              "linear_attention_oracle": (t2 - t1) * 1e3,
                                              "softmax_attention_oracle": (t3 - t2) * 1e3}
        rows.append(row)
        del db
    return rows


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default=WORKLOAD)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-users", type=int, default=8)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 256 MiB device copies (reference for PMC byte counters)")
    ap.add_argument("--alg1", action="store_true",
                    help="also time the factorization by Algorithm 1 run as printed (passes over X) "
                         "with 0 and 1 power iterations, next to the Gram route")
    ap.add_argument("--from-x", action="store_true",
                    help="time the variant that never stores P: solar_svd_factorize with P = NULL and "
                         "solar_svd_attention_from_x (the projection inside the attention kernel)")
    ap.add_argument("--backward", action="store_true",
                    help="also time the gradient through the factorization (dL/dX from dL/dS, dL/dV)")
    ap.add_argument("--sweep", action="store_true",
                    help="also sweep the history length N at fixed M, d, r (the protocol of the paper's "
                         "forward-latency figure): softmax, linear and SVD attention on the GPU, and the "
                         "oracle on one CPU thread at the shorter lengths")
    ap.add_argument("--streams", type=int, default=N_BUFFER_SETS,
                    help="independent batches in flight (one HIP stream and one buffer set each)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (users are independent, so more GPUs "
              "would each run the same kernels on their share of the batch); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2603_02561_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    w = synth.make_config(args.workload)
    bf16 = w.dtype == synth.BF16
    n_sets = max(N_BUFFER_SETS, args.streams)   # one buffer set per batch in flight
    sets = [binding.DeviceBatch(w.X, w.Q, w.lengths, w.r, bf16) for _ in range(n_sets)]
    scale = 1.0
    # Steps are independent batches.  Step i runs on stream i % n_streams with buffer set
    # i % n_sets (its own inputs, outputs and workspace), so the latency-bound
    # eigen-iteration of one batch overlaps the bandwidth/ALU-bound phases of its neighbours.
    n_streams = max(1, min(args.streams, n_sets))
    streams = [torch.cuda.Stream() for _ in range(n_streams)]

    if args.from_x:
        def factorize(db): db.factorize_no_p()
        def attend(db): db.attention_from_x(scale)
    else:
        def factorize(db): db.factorize()
        def attend(db): db.attention(scale, binding.SOLAR_ATTN_SEQ_SOFTMAX)

    def step(i):
        db = sets[i % n_sets]
        with torch.cuda.stream(streams[i % n_streams]):
            factorize(db)
            attend(db)

    for i in range(max(args.warmup, 1)):
        step(i)
    torch.cuda.synchronize()

    # Serial pass: the same K steps on one stream, nothing else on the GPU.  Its per-kernel
    # HIP-event durations are what the roofline figures are taken from (a kernel on its own);
    # the pipelined pass below gives the throughput.
    ser_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(args.steps)]
    ser_step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    ser_start = torch.cuda.Event(enable_timing=True)
    ser_stop = torch.cuda.Event(enable_timing=True)
    binding.solar_phase_timing_begin()
    torch.cuda.synchronize()
    with torch.cuda.stream(streams[0]):
        ser_start.record()
        ser_step_ev[0].record()
        for i in range(args.steps):
            db = sets[i % n_sets]
            factorize(db)
            ser_ev[i][0].record()
            attend(db)
            ser_ev[i][1].record()
            ser_step_ev[i + 1].record()
        ser_stop.record()
    torch.cuda.synchronize()
    ser_calls, ser_phase = binding.solar_phase_timing_end()
    solo = {"gram": ser_phase[0] / max(ser_calls, 1), "eig": ser_phase[1] / max(ser_calls, 1),
            "project": ser_phase[2] / max(ser_calls, 1),
            "attention": sum(a.elapsed_time(b) for a, b in ser_ev) / args.steps,
            "step": ser_start.elapsed_time(ser_stop) / args.steps}
    step_times = sorted(ser_step_ev[i].elapsed_time(ser_step_ev[i + 1]) for i in range(args.steps))
    attn_times = sorted(a.elapsed_time(b) for a, b in ser_ev)

    def pct(v, q):
        return v[min(len(v) - 1, int(q * len(v)))]
    solo_spread = {"step_ms": {"p10": pct(step_times, 0.1), "median": pct(step_times, 0.5), "p90": pct(step_times, 0.9)},
                   "attention_ms": {"p10": pct(attn_times, 0.1), "median": pct(attn_times, 0.5),
                                    "p90": pct(attn_times, 0.9)}}

    attn_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(args.steps)]
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    binding.solar_phase_timing_begin()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start.record()
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    for i in range(args.steps):
        db = sets[i % n_sets]
        with torch.cuda.stream(streams[i % n_streams]):
            factorize(db)
            attn_ev[i][0].record()
            attend(db)
            attn_ev[i][1].record()
    for st in streams:
        torch.cuda.current_stream().wait_stream(st)
    stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    total_ms = start.elapsed_time(stop)
    ncalls, phase_ms = binding.solar_phase_timing_end()
    attn_ms = sum(a.elapsed_time(b) for a, b in attn_ev) / args.steps

    # The same throughput pass with the projection A3 formed inside the attention kernel
    # (solar_svd_attention_from_x: P is never stored).  Reported beside `value`, which stays the
    # path that writes P as solar_svd_factorize's output.
    fused = None
    if (not args.from_x and bf16 and w.r % 4 == 0 and w.r <= (32 if w.d == 256 else 64)):
        def fstep(i):
            db = sets[i % n_sets]
            with torch.cuda.stream(streams[i % n_streams]):
                db.factorize_no_p()
                db.attention_from_x(scale)
        for i in range(min(args.warmup, 10)):
            fstep(i)
        torch.cuda.synchronize()
        f0 = torch.cuda.Event(enable_timing=True)
        f1 = torch.cuda.Event(enable_timing=True)
        f0.record()
        for st in streams:
            st.wait_stream(torch.cuda.current_stream())
        for i in range(args.steps):
            fstep(i)
        for st in streams:
            torch.cuda.current_stream().wait_stream(st)
        f1.record()
        torch.cuda.synchronize()
        fms = f0.elapsed_time(f1) / args.steps
        fused = {"value": w.B / (fms * 1e-3), "unit": "user-sequences/s", "ms_per_step": fms,
                 "note": "same pass through solar_svd_factorize(P = NULL) + solar_svd_attention_from_x"}
        # leave the buffer sets as the stored-P path left them for the accuracy check below
        for i in range(n_sets):
            step(i)
        torch.cuda.synchronize()
    gram_ms, eig_ms, proj_ms = [p / max(ncalls, 1) for p in phase_ms]
    ms_per_step = total_ms / args.steps
    info_bad = int((sets[0].info != 0).sum().item())

    # Algorithmic work per launch (whole batch): what the method must move or compute, not
    # what the kernels happen to do.
    lens = w.lengths.astype(np.float64)
    e = 2 if bf16 else 4
    work = {
        # read X once, write G
        "gram": ("hbm", float(np.sum(lens) * w.d * e + w.B * w.d * w.d * 4)),
        # read the valid rows of X once, write P: all N rows of it, because the rows past the valid
        # length are part of the output (zeros)
        "project": ("hbm", float(np.sum(lens) * w.d * e + w.B * w.N * w.r * 4)),
        # Qt = Q V, S = Qt P^T, Z = W P, O = Z V^T
        "attention": ("mfma", float(np.sum(4.0 * w.M * lens * w.r) + w.B * 4.0 * w.M * w.r * w.d)),
    }
    mfma_peak = PEAKS["mfma_bf16_TFLOPs"] if bf16 else PEAKS["mfma_f32_TFLOPs"]
    kernel_names = {"gram": "gram256_shared_kernel" if (bf16 and w.d == 256) else "gram_partial_kernel",
                    "eig": "eig_topr_kernel",
                    "project": "project_bf16_kernel" if bf16 else "project_kernel",
                    "attention": ("attention_seq_x32_kernel" if (w.r <= 64 and w.r % 4 == 0) else "attention_seq_bf16_kernel")
                    if bf16 else "attention_seq_kernel"}
    phases = {"gram": gram_ms, "eig": eig_ms, "project": proj_ms, "attention": attn_ms}
    kernels = {}
    for name, (bound, amount) in work.items():
        for label, ms in (("pipelined", phases[name]), ("alone", solo[name])):
            if bound == "hbm":
                achieved, peak, unit = amount / (ms * 1e-3) / 1e9, PEAKS["hbm_GBps"], "GB/s"
            else:
                achieved, peak, unit = amount / (ms * 1e-3) / 1e12, mfma_peak, "TFLOP/s"
            kernels.setdefault(name, {"kernel": kernel_names[name], "bound": bound, "unit": unit,
                                      "peak": peak, "algorithmic": amount})[label] = {
                "ms": ms, "achieved": achieved, "frac": achieved / peak}
    # second bound of the attention kernel: one exponential per (candidate, key) pair; v_exp_f32
    # issues at half the plain vector rate (8 lanes per clock per SIMD, measured 8.35 cycles per
    # wave instruction): 256 CUs x 4 SIMDs x 8 x 2.4 GHz
    n_exp = float(np.sum(w.M * lens))
    exp_peak = 256 * 4 * 8 * 2.4e9 / 1e12
    kernels["attention"]["exp_bound"] = {
        "exponentials": n_exp, "peak_Texp_per_s": exp_peak,
        "alone": {"achieved": n_exp / (solo["attention"] * 1e-3) / 1e12,
                  "frac": n_exp / (solo["attention"] * 1e-3) / 1e12 / exp_peak}}
    kernels["eig"] = {"kernel": kernel_names["eig"], "bound": "latency (serial Jacobi rounds, one "
                      "workgroup per user; no roofline)", "pipelined": {"ms": eig_ms},
                      "alone": {"ms": solo["eig"]}}
    # dominant kernel = the roofline-bound kernel with the most GPU time
    dominant = max(work, key=lambda k: solo[k])
    traffic = MEASURED_TRAFFIC.get((w.name, dominant))
    roof = {"kernel": kernel_names[dominant], "bound": kernels[dominant]["bound"],
            "achieved": kernels[dominant]["alone"]["achieved"], "peak": kernels[dominant]["peak"],
            "unit": kernels[dominant]["unit"], "frac": kernels[dominant]["alone"]["frac"],
            "traffic": traffic,
            "traffic_source": None if traffic is None else
            "HBM fetch + write bytes of one launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs "
            "summarised in profiles/hbm_traffic_C3.txt (a constant of this script, not measured in this run)",
            "achieved_pipelined": kernels[dominant]["pipelined"]["achieved"],
            "frac_pipelined": kernels[dominant]["pipelined"]["frac"],
            "note": f"achieved = algorithmic work of one launch / its average HIP-event duration over "
                    f"the {args.steps} steps of the serial pass (one stream, the kernel has the GPU; "
                    f"matches `rocprofv3 --kernel-trace --stats -- python bench.py --streams 1`). "
                    f"*_pipelined is the same over the throughput pass, where kernels of {n_streams} "
                    "independent batches share the GPU and each launch lasts longer. "
                    "eig_topr_kernel has the longest single launch but is latency bound (no roofline)."}

    out = {
        "metric": "user-sequences/sec (factorize+attend) at N=10k,d=128,r=32,M=1000; % roofline",
        "value": w.B * args.steps / (total_ms * 1e-3),
        "unit": "user-sequences/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("bf16 inputs; fp16 MFMA operands for P, Q V and the softmax weights in the attention kernel, "
                  "bf16 MFMA operands elsewhere; f32 accumulate") if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} N={w.N} d={w.d} r={w.r} M={w.M} "
                               f"{'bf16' if bf16 else 'f32'} inputs, mode 0, scale {scale}",
                   "recipe": w.recipe, "buffer_sets": n_sets},
        "phase_ms": phases, "dominant_kernel": dominant, "kernels": kernels,
        "host_wall_ms_per_step": wall * 1e3 / args.steps,
        "fused_projection": fused,
        "streams": n_streams, "serial_pass_ms": solo, "serial_pass_spread": solo_spread,
        "value_serial": w.B / (solo["step"] * 1e-3),
        "users_not_converged": info_bad,
        "roofline": roof,
    }
    if args.alg1:
        # Algorithm 1 as printed: Y = X Omega, n_iter x (Omega <- X^T Y, Y = X Omega), Q R = Y,
        # SVD of Q^T X.  Timed one batch at a time; the factors of the Gram route are the reference.
        db = sets[0]
        db.factorize()
        torch.cuda.synchronize()
        V_ref = db.V.clone()
        omega = torch.from_numpy(synth.make_omega(w.B, w.d, w.r)).cuda()
        lens_sum = float(np.sum(lens))
        alg1 = {}
        for q in (0, 1, 2):
            db.factorize_rsvd(omega, q)
            torch.cuda.synchronize()
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            for _ in range(args.steps):
                db.factorize_rsvd(omega, q)
            ev1.record()
            torch.cuda.synchronize()
            ms = ev0.elapsed_time(ev1) / args.steps
            flagged = int((db.info != 0).sum().item())
            pv = torch.bmm(db.V, db.V.transpose(1, 2)) - torch.bmm(V_ref, V_ref.transpose(1, 2))
            # bytes the method must move: X (2q+2 passes, + 1 for P), Y written q+1 and read q+1 times, P
            passes = 2 * q + 2
            nbytes = (passes + 1) * lens_sum * w.d * e + (2 * (q + 1) + 1) * lens_sum * w.r * 4
            alg1[f"n_iter={q}"] = {
                "ms_per_factorize": ms, "passes_over_X": passes + 1, "algorithmic_bytes": nbytes,
                "achieved_GBps": nbytes / (ms * 1e-3) / 1e9, "users_flagged": flagged,
                "max_projector_diff_vs_gram_route": float(pv.abs().amax().item())}
        alg1["gram_route_ms_per_factorize"] = solo["gram"] + solo["eig"] + solo["project"]
        out["alg1_as_printed"] = alg1
    if args.backward:
        # dL/dX = P S^-1 K V^T: reads P (r floats a row), writes dX (d floats a row); the r x r and
        # r x d work per user is negligible next to it, so the pair of kernels is HBM-bound.
        db = sets[0]
        db.factorize()
        s_bar, v_bar = (torch.from_numpy(a).cuda() for a in synth.make_cotangents(w.B, w.d, w.r))
        dX = db.backward(s_bar, v_bar, 0.0)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(args.steps):
            db.backward(s_bar, v_bar, 0.0, dX)
        ev1.record()
        torch.cuda.synchronize()
        ms = ev0.elapsed_time(ev1) / args.steps
        nbytes = w.B * w.N * (w.r + w.d) * 4.0
        out["svd_backward"] = {"ms": ms, "algorithmic_bytes": nbytes,
                               "achieved_GBps": nbytes / (ms * 1e-3) / 1e9, "frac_of_hbm_peak":
                               nbytes / (ms * 1e-3) / 1e9 / PEAKS["hbm_GBps"]}
        del dX
    if args.sweep:
        out["sweep"] = latency_sweep(w, min(args.steps, 20))   # its dense reference kernel takes 50 ms at N = 20000
    if not args.no_cpu_baseline:
        n_cpu = min(args.cpu_users, w.B)
        base, o_cpu = cpu_baseline(w, n_cpu)
        out["cpu_baseline"] = base
        o_gpu = sets[(args.steps - 1) % n_sets].O[:n_cpu].cpu().numpy().astype(np.float64)
        err = max(float(np.abs(o_gpu[b] - o_cpu[b]).max() / np.abs(o_cpu[b]).max()) for b in range(n_cpu))
        out["max_rel_err_vs_oracle"] = err
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
