#!/usr/bin/env python3
"""Benchmark of the signature hot path on one MI355X.

A step = sig_forward + sig_backward over one batch of the headline workload (c2: B=256, L=256, d=4,
depth 6, 5460 coefficients; synthetic random-walk paths with a time channel).  All buffers live in HBM
before the timed region; nothing is allocated inside it.

Prints ONE JSON line:
  value        coefficient-steps/s for forward + backward = B * L * |W| / (time of one step)
  roofline     the dominant kernel (backward main kernel) against the FP32 vector peak: algorithmic
               flops per launch / average kernel duration measured with HIP events in the timed region
  cpu_baseline the fp64 oracle timed on the host cores on a bounded sample of the same workload
  per_workload forward / backward GPU times (whole call) and roofline fractions of all six workloads
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_VECTOR_TFLOPS = 157.3     # 256 CU x 4 SIMD x 16 lanes x 2 (packed) x 2 flop x 2.4 GHz
HEADLINE = "c2"


def flops_forward(ws, B, L):
    """2 flops per multiply-add, one multiply-add per (word, longer-or-equal target length) pair."""
    return 2.0 * ws.min_fma_per_step * B * L


def flops_backward(ws, B, L):
    """Adjoint scheme: 3 multiply-adds per pair with target length = word length (reconstruct, adjoint push,
    gradient bucket), 4 multiply-adds + 1 add per pair with a longer target (those plus the recomputed
    accumulator and the adjoint sum)."""
    fmin, nw = ws.min_fma_per_step, ws.size
    return 2.0 * (3.0 * nw + 4.5 * (fmin - nw)) * B * L


def WORKLOADS_REF_get():
    from sig_workloads import WORKLOADS
    return WORKLOADS


def setup(name, S, torch):
    from sig_workloads import WORKLOADS, make_grad_coeffs, workload_path, workload_word_list
    wl = WORKLOADS[name]
    words = workload_word_list(wl) if wl.kind == "words" else None
    t0 = time.perf_counter()
    if wl.kind == "truncated":
        ws = S.sig_wordset_build_truncated(wl.d, wl.depth)
    elif wl.kind == "anisotropic":
        ws = S.sig_wordset_build_anisotropic(wl.d, wl.weights, wl.cutoff)
    else:
        ws = S.sig_wordset_build(wl.d, words)
    build_ms = (time.perf_counter() - t0) * 1e3        # host: tables + launch plans, once per word set
    ws.upload("cuda:0")
    X = workload_path(wl)
    G = make_grad_coeffs(wl.seed, wl.B, ws.size)
    lib = S.load_library()
    st = {
        "wl": wl, "ws": ws, "X": X, "G": G, "build_ms": build_ms,
        "path": torch.from_numpy(X).cuda(),
        "grad": torch.from_numpy(G).cuda(),
        "coeffs": torch.empty((wl.B, ws.size), dtype=torch.float32, device="cuda"),
        "gpath": torch.empty((wl.B, wl.L + 1, wl.d), dtype=torch.float32, device="cuda"),
    }
    nf = int(lib.sig_forward_workspace_bytes(ws._h, wl.B, wl.L + 1))
    nb = int(lib.sig_backward_workspace_bytes(ws._h, wl.B, wl.L + 1))
    st["wf"] = torch.empty(max(nf, 256), dtype=torch.uint8, device="cuda")
    st["wb"] = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
    assert st["wf"].data_ptr() % 256 == 0 and st["wb"].data_ptr() % 256 == 0
    return st


def step(S, st):
    S.sig_forward(st["ws"], st["path"], out=st["coeffs"], workspace=st["wf"])
    S.sig_backward(st["ws"], st["path"], st["coeffs"], st["grad"], out=st["gpath"], workspace=st["wb"])


def time_steps(S, torch, st, steps, warmup):
    """Returns (seconds per step by the host clock, forward main-kernel ms, backward main-kernel ms, GPU ms of the
    whole forward call, of the whole backward call), averaged over `steps` steps.  Every recorded event costs a few
    microseconds on the stream, so the timed region records one pair per step only, around the dominant kernel (found
    in the warm-up, which records everything); the other durations come from untimed passes of the same steps
    afterwards."""
    S.sig_profile_enable(True)
    for _ in range(max(warmup, 1)):
        step(S, st)
    torch.cuda.synchronize()
    nf, msf = S.sig_profile_read(False)
    nb, msb = S.sig_profile_read(True)
    dominant = 1 if msb / max(nb, 1) >= msf / max(nf, 1) else 0
    S.sig_profile_enable(True, channels=[dominant])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(S, st)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    nd, msd = S.sig_profile_read(bool(dominant))
    assert nd == steps
    # two untimed passes: event pairs around the main kernels, then around whole calls (nested pairs would add their
    # own recording time to the outer one)
    S.sig_profile_enable(True, channels=[0, 1])
    for _ in range(steps):
        step(S, st)
    torch.cuda.synchronize()
    nf, msf = S.sig_profile_read(False)
    nb, msb = S.sig_profile_read(True)
    S.sig_profile_enable(True, channels=[2, 3])
    for _ in range(steps):
        step(S, st)
    torch.cuda.synchronize()
    ncf, cf = S.sig_profile_read(False, whole_call=True)
    ncb, cb = S.sig_profile_read(True, whole_call=True)
    S.sig_profile_enable(False)
    assert nf == steps and nb == steps and ncf == steps and ncb == steps
    kf, kb = msf / nf, msb / nb
    if dominant:
        kb = msd / nd                 # the dominant kernel's duration is the one measured inside the timed region
    else:
        kf = msd / nd
    return (t1 - t0) / steps, kf, kb, cf / nf, cb / nb


def roofline_entry(flops, ms, kernel=""):
    """Algorithmic flops per launch over the measured kernel duration.  The cascade kernels for full truncations issue
    most of their multiply-adds as fp32 matrix-core instructions (dense fp32 MFMA peak = FP32 vector peak = 157.3
    TFLOP/s); the d = 4 and d = 8 backward kernels, the run-time specialised and the table-driven kernels use the vector
    ALU only."""
    ach = flops / (ms * 1e-3) / 1e12
    on_matrix_cores = kernel.startswith("trunc_") and not kernel.startswith(("trunc_tails_bwd", "trunc_node_bwd"))
    return {"bound": "mfma" if on_matrix_cores else "alu", "achieved": round(ach, 3),
            "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_FP32_VECTOR_TFLOPS, 4),
            "traffic": None}


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` on `workload` from the committed rocprofv3 counter runs (FETCH_SIZE and
    WRITE_SIZE, scaled by a copy kernel of known size); None when that pair has not been measured."""
    path = os.path.join(ROOT, "paper_2602_24066_amd", "measured_traffic.json")
    try:
        with open(path) as f:
            table = json.load(f)
    except OSError:
        return None
    for row in table.get("kernels", []):
        if row["workload"] == workload and kernel.startswith(row["kernel_prefix"]):
            return row["hbm_bytes_per_launch"]
    return None


def cpu_baseline(st, sample_paths, budget_s=12.0):
    """The oracle as it stands (fp64 dense tensor algebra, one path per OpenMP thread) on the first `sample_paths`
    paths, repeated until about `budget_s` seconds of wall-clock have been spent (at least once)."""
    import numpy as np
    from oracle import sig_oracle as O
    wl, ws = st["wl"], st["ws"]
    X = np.ascontiguousarray(st["X"][:sample_paths])
    G = st["G"][:sample_paths].astype(np.float64)
    O.forward_dense(X[:1], wl.depth)                       # load + warm
    tf = tb = 0.0
    reps = 0
    while reps == 0 or (tf + tb < budget_s and reps < 200):
        t0 = time.perf_counter()
        O.forward_dense(X, wl.depth)
        t1 = time.perf_counter()
        O.backward_dense(X, wl.depth, G)
        t2 = time.perf_counter()
        tf, tb, reps = tf + (t1 - t0), tb + (t2 - t1), reps + 1
    work = reps * sample_paths * wl.L * ws.size
    return {"value": round(work / (tf + tb), 1), "unit": "coefficient-steps/s (forward + backward)", "cores": O.threads(),
            "kind": "oracle",
            "sample": f"{sample_paths} of {wl.B} paths of {wl.name}, full length L={wl.L}, {reps} repetitions; fp64 dense "
                      f"tensor-algebra forward {tf:.2f} s + reverse-mode backward {tb:.2f} s in total",
            "forward_value": round(work / tf, 1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the clock of an idle MI355X takes some tens of milliseconds of load to settle (c2: 0.105 ms per step over 50 steps,
    # 0.094 ms from about 1,000 steps on), so the defaults time a tenth of a second after a fifth of that as warm-up
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--no-others", action="store_true", help="skip the per-workload table")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--cpu-sample", type=int, default=0, help="paths given to the oracle (0 = the whole batch)")
    ap.add_argument("--calibrate", action="store_true",
                    help="after the timed region launch a plain 256 MiB copy kernel three times (reference for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (paths are independent; sharding over the batch needs no "
              "exchange). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    if args.steps > 4096:
        print("bench.py: --steps is limited to 4096 (kernel timer capacity)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2602_24066_amd as S
    S.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    st = setup(args.workload, S, torch)
    wl, ws = st["wl"], st["ws"]
    sec, ms_f, ms_b, call_f, call_b = time_steps(S, torch, st, args.steps, args.warmup)
    work = wl.B * wl.L * ws.size
    ff, fb = flops_forward(ws, wl.B, wl.L), flops_backward(ws, wl.B, wl.L)
    kn_f, kn_b = ws.kernel_name(False, wl.B, wl.L + 1), ws.kernel_name(True, wl.B, wl.L + 1)
    rf, rb = roofline_entry(ff, ms_f, kn_f), roofline_entry(fb, ms_b, kn_b)
    dominant = rb if ms_b >= ms_f else rf
    dominant = dict(dominant)
    dominant["kernel"] = kn_b if ms_b >= ms_f else kn_f
    dominant["kernel_ms"] = round(max(ms_b, ms_f), 4)
    dominant["algorithmic_flops_per_launch"] = fb if ms_b >= ms_f else ff
    dominant["traffic"] = measured_traffic(dominant["kernel"], wl.name)

    # plain v_fma_f32 rate of this chip, measured in the same run (register-only kernel, 32 wavefronts per compute unit):
    # the roof for vector code that does not use packed FP32
    dominant["measured_unpacked_fma_tflops"] = round(S.sig_probe_fma_tflops(), 1)

    out = {
        "metric": "signature coeff-steps/sec (fwd, fwd+bwd) + % of FP32 vector roofline, 1 GPU",
        "value": round(work / sec, 1),
        "unit": "coefficient-steps/s (forward + backward)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.B} L={wl.L} d={wl.d} {wl.kind}"
                               + (f" depth={wl.depth}" if wl.depth else "") + f" |W|={ws.size}",
                   "min_fma_per_path_step": ws.min_fma_per_step},
        # call_ms: GPU time of everything sig_forward / sig_backward enqueue (main kernel + transposes, chunk products,
        # chain rule); roofline_frac prices the algorithmic flops against that whole time
        "forward": {"kernel": kn_f, "kernel_ms": round(ms_f, 4), "call_ms": round(call_f, 4),
                    "coeff_steps_per_s": round(work / (call_f * 1e-3), 1),
                    "roofline_frac": roofline_entry(ff, call_f)["frac"], "main_kernel_roofline_frac": rf["frac"]},
        "backward": {"kernel": kn_b, "kernel_ms": round(ms_b, 4), "call_ms": round(call_b, 4),
                     "coeff_steps_per_s": round(work / (call_b * 1e-3), 1),
                     "roofline_frac": roofline_entry(fb, call_b)["frac"], "main_kernel_roofline_frac": rb["frac"]},
        "roofline": dominant,
    }

    if not args.no_others:
        per = {}
        for name in ("c1", "c2", "c3", "c4a", "c4b", "c5"):
            torch.cuda.reset_peak_memory_stats()
            base = torch.cuda.memory_allocated()
            s2 = st if name == args.workload else setup(name, S, torch)
            # about 0.15 s of work per measuring pass (the clock settles first): 20 to --steps steps
            step(S, s2)                                  # first call: run-time compilation, kernel attributes
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(3):
                step(S, s2)
            torch.cuda.synchronize()
            n = int(min(max(args.steps, 20), max(20, 0.15 / max((time.perf_counter() - t0) / 3, 1e-6))))
            sec2, kf2, kb2, f2, b2 = time_steps(S, torch, s2, n, max(n // 5, 2))
            per_steps = n
            w2, wl2 = s2["ws"], s2["wl"]
            wk = wl2.B * wl2.L * w2.size
            per[name] = {
                "coeffs": w2.size, "fwd_ms": round(f2, 4), "bwd_ms": round(b2, 4),
                "fwd_main_kernel_ms": round(kf2, 4), "bwd_main_kernel_ms": round(kb2, 4),
                "fwd_coeff_steps_per_s": round(wk / (f2 * 1e-3), 1),
                "fwd_bwd_coeff_steps_per_s": round(wk / ((f2 + b2) * 1e-3), 1),
                "fwd_roofline_frac": roofline_entry(flops_forward(w2, wl2.B, wl2.L), f2)["frac"],
                "bwd_roofline_frac": roofline_entry(flops_backward(w2, wl2.B, wl2.L), b2)["frac"],
                "kernels": [w2.kernel_name(False, wl2.B, wl2.L + 1), w2.kernel_name(True, wl2.B, wl2.L + 1)],
                "wordset_build_ms": round(s2["build_ms"], 3), "steps": per_steps,
            }
            if name == "c5":
                per[name]["peak_device_bytes"] = int(torch.cuda.max_memory_allocated() - base)
                per[name]["mem_out_bytes"] = 4 * wl2.B * w2.size
            if s2 is not st:
                del s2
                torch.cuda.empty_cache()
        out["per_workload"] = per

        # signatures over windows (Section 5 of the paper): 32 paths of 1,024 segments, 64 sliding windows of 128
        # segments each, the headline word set; all 2,048 (path, window) pairs advance in one launch
        try:
            from sig_workloads import make_path
            wsw = st["ws"] if args.workload == HEADLINE else setup(HEADLINE, S, torch)["ws"]
            Bw, Lw, Kw, lenw = 32, 1024, 64, 128
            Xw = torch.from_numpy(make_path("time0", 77, Bw, Lw, wsw.dim)).cuda()
            wins = [(k * (Lw - lenw) // (Kw - 1), k * (Lw - lenw) // (Kw - 1) + lenw) for k in range(Kw)]
            cw = S.sig_forward_windows(wsw, Xw, wins)
            gw = torch.randn_like(cw)
            S.sig_backward_windows(wsw, Xw, wins, cw, gw)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(200):
                cw = S.sig_forward_windows(wsw, Xw, wins)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(200):
                S.sig_backward_windows(wsw, Xw, wins, cw, gw)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            wk = Bw * Kw * lenw * wsw.size
            out["windows"] = {"workload": f"B={Bw} L={Lw} d={wsw.dim} |W|={wsw.size}, {Kw} sliding windows of {lenw} segments",
                              "fwd_ms": round((t1 - t0) * 5, 4), "bwd_ms": round((t2 - t1) * 5, 4),
                              "fwd_bwd_coeff_steps_per_s": round(wk / ((t2 - t0) / 200), 1),
                              "note": "host clock, includes the per-call workspace allocation of the Python wrapper"}
        except Exception as e:                       # an optional extra must not take the benchmark line down
            out["windows"] = {"error": str(e)[:200]}

        # log-signature (Section 3.3) on the headline shape: signature on the reduced word set (every word shorter than
        # the depth + the Lyndon words of full length), tensor logarithm word by word, and back
        try:
            from sig_workloads import workload_path as workload_path_ref
            wlh = WORKLOADS_REF_get()[HEADLINE]
            wsl = S.sig_wordset_build_logsig(wlh.d, wlh.depth)
            wsl.upload("cuda:0")
            Xl = torch.from_numpy(workload_path_ref(wlh)).cuda()
            cl = S.sig_forward(wsl, Xl)
            lg = S.sig_logsig_forward(wsl, cl)
            gl = torch.randn_like(lg)
            S.sig_backward(wsl, Xl, cl, S.sig_logsig_backward(wsl, cl, gl))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(200):
                cl = S.sig_forward(wsl, Xl)
                lg = S.sig_logsig_forward(wsl, cl)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(200):
                S.sig_backward(wsl, Xl, cl, S.sig_logsig_backward(wsl, cl, gl))
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            out["log_signature"] = {"workload": f"{wlh.name} shape, depth {wlh.depth}: {wsl.size} signature words for {lg.shape[1]} "
                                                f"log-signature coordinates",
                                    "kernels": [wsl.kernel_name(False, wlh.B, wlh.L + 1), wsl.kernel_name(True, wlh.B, wlh.L + 1)],
                                    "fwd_ms": round((t1 - t0) * 5, 4), "bwd_ms": round((t2 - t1) * 5, 4),
                                    "note": "host clock, signature + tensor logarithm (forward) and their adjoints (backward)"}
        except Exception as e:
            out["log_signature"] = {"error": str(e)[:200]}

        # shapes of the paper's own timing table (Section 5, Table 1: training step = forward + backward, float32,
        # one H200): synthetic random walks of the same shape; the paper's figure is context, another machine's
        try:
            from sig_workloads import make_path as make_path_ref
            table = {}
            for (Bp, Mp, dp, Np, paper_us) in [(32, 100, 6, 4, 207.52), (32, 100, 6, 5, 555.63), (32, 100, 6, 6, 3360.0),
                                               (64, 1000, 4, 6, 6450.0), (1, 200, 10, 4, 320.35),
                                               (256, 200, 10, 4, 9830.0)]:
                wsp = S.sig_wordset_build_truncated(dp, Np)
                wsp.upload("cuda:0")
                Xp = torch.from_numpy(make_path_ref("iid", 7, Bp, Mp - 1, dp)).cuda()
                cp = S.sig_forward(wsp, Xp)
                gp = torch.randn_like(cp)
                S.sig_backward(wsp, Xp, cp, gp)
                torch.cuda.synchronize()
                S.sig_profile_enable(True, channels=[2, 3])       # whole calls only
                for _ in range(300):
                    S.sig_forward(wsp, Xp, out=cp)
                    S.sig_backward(wsp, Xp, cp, gp)
                torch.cuda.synchronize()
                nf, mf = S.sig_profile_read(False, True)
                nb, mb = S.sig_profile_read(True, True)
                S.sig_profile_enable(False)
                us = (mf / max(nf, 1) + mb / max(nb, 1)) * 1e3
                table[f"B={Bp} points={Mp} d={dp} N={Np}"] = {
                    "coeffs": wsp.size, "step_us": round(us, 1), "paper_h200_step_us": paper_us,
                    "fwd_bwd_coeff_steps_per_s": round(Bp * (Mp - 1) * wsp.size / (us * 1e-6), 1),
                    "kernels": [wsp.kernel_name(False, Bp, Mp), wsp.kernel_name(True, Bp, Mp)]}
            out["paper_table_shapes"] = table
        except Exception as e:
            out["paper_table_shapes"] = {"error": str(e)[:200]}

        # the other word-set builders (host only): graph-induced set and the sparse lead-lag set of a 5-dimensional path
        t0 = time.perf_counter()
        g = S.sig_wordset_build_graph(10, [(a, b) for a in range(10) for b in range(10) if 0 < b - a <= 3], 6)
        t1 = time.perf_counter()
        ll = S.sig_wordset_build_leadlag_sparse(5, 4)
        t2 = time.perf_counter()
        out["other_word_sets"] = {"graph(d=10, edges i->i+1..i+3, depth 6)": {"words": g.size, "build_ms": round((t1 - t0) * 1e3, 3)},
                                  "leadlag_sparse(d=5, depth 4)": {"words": ll.size, "build_ms": round((t2 - t1) * 1e3, 3)}}

    if not args.no_cpu and wl.kind == "truncated":
        out["cpu_baseline"] = cpu_baseline(st, min(args.cpu_sample, wl.B) if args.cpu_sample > 0 else wl.B)

    if args.calibrate:
        n = 64 * 1024 * 1024
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)                   # elementwise kernel: reads 4n bytes, writes 4n bytes
        torch.cuda.synchronize()

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
