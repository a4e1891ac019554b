#!/usr/bin/env python3
"""Benchmark of the signature hot path on one MI355X.

A step = sig_forward + sig_backward over one batch of the headline workload, the largest configuration: c5
(B=64, L=4096, d=16, depth 4, 69,904 coefficients; synthetic AR(1) paths).  All buffers live in HBM before the
timed region; nothing is allocated inside it.

Prints ONE JSON line:
  value        coefficient-steps/s for forward + backward = B * L * |W| / (time of one step)
  roofline     the dominant kernel (backward main kernel) against the FP32 peak: algorithmic flops per launch /
               average kernel duration measured with HIP events in the timed region
  cpu_baseline the fp64 oracle timed on the host cores on a bounded sample of the same workload
  errors       forward error per word length and gradient error of this run's GPU results against the oracle on
               the same sample (the measures the parity tests use)
  per_workload the same for all six workloads: GPU times (whole call and main kernel), roofline fractions,
               errors against the oracle, oracle timing
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_TFLOPS = 157.3            # 256 CU x 4 SIMD x 16 lanes x 2 (packed) x 2 flop x 2.4 GHz = dense fp32 MFMA peak
HBM_PEAK_GBS = 8000.0
HEADLINE = "c5"
ALL = ("c1", "c2", "c3", "c4a", "c4b", "c5")
# paths handed to the oracle per workload (the first n of the batch): about 15 s of host work for c5, 1-3 s for the others
CPU_SAMPLE = {"c1": 32, "c2": 256, "c3": 16, "c4a": 16, "c4b": 16, "c5": 16}


def flops_forward(ws, B, L):
    """2 flops per multiply-add, one multiply-add per (word, longer-or-equal target length) pair."""
    return 2.0 * ws.min_fma_per_step * B * L


def flops_backward(ws, B, L):
    """Adjoint scheme: 3 multiply-adds per pair with target length = word length (reconstruct, adjoint push,
    gradient bucket), 4 multiply-adds + 1 add per pair with a longer target (those plus the recomputed
    accumulator and the adjoint sum)."""
    fmin, nw = ws.min_fma_per_step, ws.size
    return 2.0 * (3.0 * nw + 4.5 * (fmin - nw)) * B * L


def bytes_backward(ws, B, L, d):
    """Algorithmic HBM bytes of one backward call: path and both coefficient arrays read, the gradient written."""
    return 4.0 * B * (L + 1) * d + 8.0 * B * ws.size + 4.0 * B * (L + 1) * d


def bytes_forward(ws, B, L, d):
    return 4.0 * B * (L + 1) * d + 4.0 * B * ws.size


def setup(name, S, torch, plain=False):
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
        "wl": wl, "ws": ws, "X": X, "G": G, "build_ms": build_ms, "words": words,
        "path": torch.from_numpy(X).cuda(),
        "grad": torch.from_numpy(G).cuda(),
        "coeffs": torch.empty((wl.B, ws.size), dtype=torch.float32, device="cuda"),
        "gpath": torch.empty((wl.B, wl.L + 1, wl.d), dtype=torch.float32, device="cuda"),
    }
    # where the library offers it for the shape, a step keeps the time-chunk signatures of the forward pass for the
    # backward pass (sig_forward_checkpointed / sig_backward_checkpointed); plain=True times sig_forward / sig_backward
    nck = 0 if plain else int(lib.sig_checkpoint_bytes(ws._h, wl.B, wl.L + 1))
    st["ck"] = torch.empty(nck, dtype=torch.uint8, device="cuda") if nck else None
    if nck:
        nf = int(lib.sig_forward_checkpointed_workspace_bytes(ws._h, wl.B, wl.L + 1))
        nb = int(lib.sig_backward_checkpointed_workspace_bytes(ws._h, wl.B, wl.L + 1))
    else:
        nf = int(lib.sig_forward_workspace_bytes(ws._h, wl.B, wl.L + 1))
        nb = int(lib.sig_backward_workspace_bytes(ws._h, wl.B, wl.L + 1))
    st["workspace_bytes"] = [nf, nb]
    st["checkpoint_bytes"] = nck
    st["wf"] = torch.empty(max(nf, 256), dtype=torch.uint8, device="cuda")
    st["wb"] = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
    assert st["wf"].data_ptr() % 256 == 0 and st["wb"].data_ptr() % 256 == 0
    return st


def step(S, st):
    if st["ck"] is not None:
        S.sig_forward_checkpointed(st["ws"], st["path"], out=st["coeffs"], checkpoint=st["ck"], workspace=st["wf"])
        S.sig_backward_checkpointed(st["ws"], st["path"], st["coeffs"], st["grad"], st["ck"], out=st["gpath"], workspace=st["wb"])
        return
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
    """Algorithmic flops per launch over the measured kernel duration.  The kernels for full truncations issue their
    leaf-level multiply-adds as fp32 matrix-core instructions (dense fp32 MFMA peak = FP32 vector peak = 157.3
    TFLOP/s); the run-time specialised and the table-driven kernels use the vector ALU only."""
    ach = flops / (ms * 1e-3) / 1e12
    on_matrix_cores = kernel.startswith("trunc_")
    return {"bound": "mfma" if on_matrix_cores else "alu", "achieved": round(ach, 3),
            "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_FP32_TFLOPS, 4),
            "traffic": None}


def device_report(torch):
    """What the device says of itself, and the FP32 vector rate that follows from its compute-unit count at the
    published 2.4 GHz (x 4 SIMDs x 16 lanes x 2 flops x 2 for the packed / dual-issue forms): the roofline's peak."""
    p = torch.cuda.get_device_properties(0)
    cus = int(p.multi_processor_count)
    return {"name": p.name, "arch": getattr(p, "gcnArchName", ""), "compute_units": cus,
            "fp32_vector_tflops_at_2400_mhz": round(cus * 4 * 16 * 2 * 2 * 2.4e9 / 1e12, 1), "memory_bytes": int(p.total_memory)}


def counter_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` on `workload` from the rocprofv3 counter runs summarised under profiles/
    (FETCH_SIZE and WRITE_SIZE of a run of this program, scaled by a copy kernel of known size); None when that
    pair has no entry.  Counters cannot be collected from inside the timed run."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        table = json.load(f)
    for row in table.get("kernels", []):
        if row["workload"] == workload and kernel.startswith(row["kernel_prefix"]):
            return row["hbm_bytes_per_launch"]
    return None


def oracle_words(st):
    from oracle import sig_oracle as O
    wl = st["wl"]
    if wl.kind == "truncated":
        return O.truncated_words(wl.d, wl.depth)
    if wl.kind == "anisotropic":
        return O.anisotropic_words(wl.d, wl.weights, wl.cutoff)
    return O.prefix_closure(st["words"])


def oracle_check(st, n_paths):
    """The oracle as it stands (fp64; dense tensor algebra for truncations, word by word for the other sets; one path
    per OpenMP thread) on the first `n_paths` paths of the batch, timed once after a one-path warm-up; and the errors
    of the GPU results in st["coeffs"] / st["gpath"] against it.  Returns (cpu_baseline dict, errors dict)."""
    import numpy as np
    from oracle import sig_oracle as O
    wl, ws = st["wl"], st["ws"]
    n = min(n_paths, wl.B)
    X = np.ascontiguousarray(st["X"][:n])
    G = st["G"][:n].astype(np.float64)
    W = oracle_words(st)
    dense = wl.kind == "truncated"
    fwd = (lambda x: O.forward_dense(x, wl.depth)) if dense else (lambda x: O.forward_words(x, W))
    bwd = (lambda x, g: O.backward_dense(x, wl.depth, g)) if dense else (lambda x, g: O.backward_words(x, W, g))
    fwd(X[:1, :min(wl.L, 16) + 1])                       # load the library, start the thread pool
    t0 = time.perf_counter()
    ref = fwd(X)
    t1 = time.perf_counter()
    gref = bwd(X, G)
    t2 = time.perf_counter()
    work = n * wl.L * ws.size
    cpu = {"value": round(work / (t2 - t0), 1), "unit": "coefficient-steps/s (forward + backward)",
           "cores": min(O.threads(), n), "kind": "oracle",
           "sample": f"first {n} of {wl.B} paths of {wl.name}, full length L={wl.L}, one run; fp64 "
                     + ("dense tensor algebra" if dense else "word-by-word evaluation")
                     + f": forward {t1 - t0:.2f} s + reverse-mode backward {t2 - t1:.2f} s",
           "forward_value": round(work / (t1 - t0), 1)}
    lengths = np.array([len(w) for w in W])
    c = st["coeffs"][:n].cpu().numpy()
    g = st["gpath"][:n].cpu().numpy()
    ferr = O.level_errors(c, ref, lengths)
    gerr = O.grad_errors(g, gref)
    errors = {"paths_checked": n,
              "forward_error_per_level": {str(k): float(f"{v:.3e}") for k, v in ferr.items()},
              "forward_tolerance": 1e-4,
              "gradient_error_max": float(f"{float(gerr.max()):.3e}"), "gradient_tolerance": 1e-3,
              "within_tolerance": bool(max(ferr.values()) <= 1e-4 and gerr.max() <= 1e-3)}
    return cpu, errors


def workload_row(S, torch, st, sec, kf, kb, cf, cb, steps):
    wl, ws = st["wl"], st["ws"]
    wk = wl.B * wl.L * ws.size
    kn_f, kn_b = ws.kernel_name(False, wl.B, wl.L + 1), ws.kernel_name(True, wl.B, wl.L + 1)
    ff, fb = flops_forward(ws, wl.B, wl.L), flops_backward(ws, wl.B, wl.L)
    bb = bytes_backward(ws, wl.B, wl.L, wl.d)
    return {
        "coeffs": ws.size, "fwd_ms": round(cf, 4), "bwd_ms": round(cb, 4),
        "fwd_main_kernel_ms": round(kf, 4), "bwd_main_kernel_ms": round(kb, 4),
        "fwd_coeff_steps_per_s": round(wk / (cf * 1e-3), 1),
        "fwd_bwd_coeff_steps_per_s": round(wk / ((cf + cb) * 1e-3), 1),
        "fwd_roofline_frac": roofline_entry(ff, cf)["frac"],
        "bwd_roofline_frac": roofline_entry(fb, cb)["frac"],
        "fwd_main_kernel_roofline_frac": roofline_entry(ff, kf)["frac"],
        "bwd_main_kernel_roofline_frac": roofline_entry(fb, kb)["frac"],
        # algorithmic bytes of the backward call over its GPU time, against the 8 TB/s of HBM3E
        "bwd_algorithmic_bytes": int(bb), "bwd_hbm_gbs_algorithmic": round(bb / (cb * 1e-3) / 1e9, 1),
        "bwd_hbm_bytes_counters": counter_traffic(kn_b, wl.name),
        "kernels": [kn_f, kn_b], "workspace_bytes": st["workspace_bytes"], "checkpoint_bytes": st["checkpoint_bytes"],
        "calls": "sig_forward_checkpointed + sig_backward_checkpointed" if st["ck"] is not None else "sig_forward + sig_backward",
        "wordset_build_ms": round(st["build_ms"], 3), "steps": steps,
    }


def plain_row(S, torch, name, n):
    """The workload through sig_forward / sig_backward, which keep the terminal signature alone between the calls."""
    s3 = setup(name, S, torch, plain=True)
    step(S, s3)
    torch.cuda.synchronize()
    _, kf3, kb3, f3, b3 = time_steps(S, torch, s3, n, max(n // 5, 2))
    w3, wl3 = s3["ws"], s3["wl"]
    return {"fwd_ms": round(f3, 4), "bwd_ms": round(b3, 4),
            "fwd_roofline_frac": roofline_entry(flops_forward(w3, wl3.B, wl3.L), f3)["frac"],
            "bwd_roofline_frac": roofline_entry(flops_backward(w3, wl3.B, wl3.L), b3)["frac"],
            "kernels": [w3.kernel_name(False, wl3.B, wl3.L + 1), w3.kernel_name(True, wl3.B, wl3.L + 1)],
            "workspace_bytes": s3["workspace_bytes"]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the clock of an idle MI355X takes some tens of milliseconds of load to settle; a c5 step takes 2-3 ms, so the
    # default times about a second of work after a fifth of that as warm-up
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=80)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--only", default="", help="comma-separated workloads for the per-workload table (default: all six)")
    ap.add_argument("--no-others", action="store_true", help="skip the per-workload table and the extras")
    ap.add_argument("--no-extras", action="store_true", help="skip windows, log-signature and the paper's table shapes")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle (timing and errors)")
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

    torch.cuda.reset_peak_memory_stats()
    base_mem = torch.cuda.memory_allocated()
    st = setup(args.workload, S, torch)
    wl, ws = st["wl"], st["ws"]
    sec, ms_f, ms_b, call_f, call_b = time_steps(S, torch, st, args.steps, args.warmup)
    peak_mem = int(torch.cuda.max_memory_allocated() - base_mem)
    work = wl.B * wl.L * ws.size
    ff, fb = flops_forward(ws, wl.B, wl.L), flops_backward(ws, wl.B, wl.L)
    kn_f, kn_b = ws.kernel_name(False, wl.B, wl.L + 1), ws.kernel_name(True, wl.B, wl.L + 1)
    rf, rb = roofline_entry(ff, ms_f, kn_f), roofline_entry(fb, ms_b, kn_b)
    dominant = dict(rb if ms_b >= ms_f else rf)
    dominant["kernel"] = kn_b if ms_b >= ms_f else kn_f
    dominant["kernel_ms"] = round(max(ms_b, ms_f), 4)
    dominant["algorithmic_flops_per_launch"] = fb if ms_b >= ms_f else ff
    dominant["traffic"] = counter_traffic(dominant["kernel"], wl.name)
    dominant["traffic_source"] = ("profiles/hbm_traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this program"
                                  if dominant["traffic"] is not None else None)
    # plain v_fma_f32 rate of this chip, measured in the same run with a register-only kernel: 8 wavefronts per SIMD (the
    # roof for vector code that does not use packed FP32) and a single wavefront per SIMD (which issues at about half
    # the rate of its SIMD: why the kernels want two wavefronts per SIMD)
    dominant["measured_unpacked_fma_tflops"] = round(S.sig_probe_fma_tflops(), 1)
    dominant["measured_unpacked_fma_tflops_one_wavefront_per_simd"] = round(S.sig_probe_fma_tflops(blocks=256, iters=16384), 1)
    # what a SIMD issues per nanosecond, by instruction kind and wavefronts per SIMD (register-only probes): ns per
    # wavefront-iteration of 64 multiply-adds (vector or scalar multiplier), of 8 16x16x4 matrix instructions, and of both
    dominant["issue_probe_ns"] = {
        f"{w}_per_simd": {"fma64_vector_operands": round(S.sig_probe_issue_ns(0, w), 1),
                          "fma64_scalar_multiplier": round(S.sig_probe_issue_ns(1, w), 1),
                          "mfma8_16x16x4": round(S.sig_probe_issue_ns(2, w), 1),
                          "fma64_and_mfma8_interleaved": round(S.sig_probe_issue_ns(3, w), 1),
                          "fma64_sources_in_one_register_bank": round(S.sig_probe_issue_ns(4, w), 1),
                          "fma64_sources_in_three_register_banks": round(S.sig_probe_issue_ns(5, w), 1),
                          "fma64_accumulator_and_multiplier_in_one_bank": round(S.sig_probe_issue_ns(6, w), 1),
                          "fma64_multiplier_and_addend_in_one_bank": round(S.sig_probe_issue_ns(7, w), 1)} for w in (1, 2, 4)}

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
                     "roofline_frac": roofline_entry(fb, call_b)["frac"], "main_kernel_roofline_frac": rb["frac"],
                     "algorithmic_bytes": int(bytes_backward(ws, wl.B, wl.L, wl.d)),
                     "hbm_gbs_algorithmic": round(bytes_backward(ws, wl.B, wl.L, wl.d) / (call_b * 1e-3) / 1e9, 1),
                     "hbm_peak_gbs": HBM_PEAK_GBS},
        "roofline": dominant,
        "memory": {"peak_device_bytes": peak_mem, "mem_out_bytes": 4 * wl.B * ws.size,
                   "note": "inputs, outputs and workspaces of forward + backward held at once"},
        "device": device_report(torch),
    }
    if wl.kind == "truncated" and ws.kernel_name(True).startswith("trunc_"):
        # reconstruction drift: the terminal signature stepped back through all L segments should end at zero
        _, resid = S.sig_backward_residual(ws, st["path"], st["coeffs"], st["grad"])
        out["reconstruction"] = {"segments": wl.L, "residual_max_abs": float(f"{float(resid.max()):.3e}"),
                                 "largest_coefficient": float(f"{float(st['coeffs'].abs().max()):.3e}"),
                                 "note": "largest |S(w)| left after multiplying by exp(-dX_j) for j = L..1, over all paths"}
    head_row = workload_row(S, torch, st, sec, ms_f, ms_b, call_f, call_b, args.steps)
    out["calls"] = head_row["calls"]
    if st["ck"] is not None and not args.no_others:
        head_row["without_checkpoint"] = plain_row(S, torch, wl.name, min(args.steps, 100))
    if not args.no_cpu:
        cpu, errs = oracle_check(st, CPU_SAMPLE[wl.name])
        out["cpu_baseline"] = cpu
        out["errors"] = errs
        head_row["cpu_baseline"], head_row["errors"] = cpu, errs

    if not args.no_others:
        per = {}
        names = [n for n in (args.only.split(",") if args.only else ALL) if n]
        for name in names:
            if name == wl.name:
                per[name] = head_row
                continue
            torch.cuda.reset_peak_memory_stats()
            base = torch.cuda.memory_allocated()
            s2 = setup(name, S, torch)
            # about 0.15 s of work per measuring pass (the clock settles first): 20 to --steps steps
            step(S, s2)                                  # first call: run-time compilation, kernel attributes
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(3):
                step(S, s2)
            torch.cuda.synchronize()
            n = int(min(max(args.steps, 20), max(20, 0.15 / max((time.perf_counter() - t0) / 3, 1e-6))))
            sec2, kf2, kb2, f2, b2 = time_steps(S, torch, s2, n, max(n // 5, 2))
            per[name] = workload_row(S, torch, s2, sec2, kf2, kb2, f2, b2, n)
            per[name]["peak_device_bytes"] = int(torch.cuda.max_memory_allocated() - base)
            per[name]["mem_out_bytes"] = 4 * s2["wl"].B * s2["ws"].size
            if not args.no_cpu:
                per[name]["cpu_baseline"], per[name]["errors"] = oracle_check(s2, CPU_SAMPLE[name])
            if s2["ck"] is not None:
                per[name]["without_checkpoint"] = plain_row(S, torch, name, n)
            del s2
            torch.cuda.empty_cache()
        out["per_workload"] = per

    if not args.no_others and not args.no_extras:
        from sig_workloads import WORKLOADS, make_path, workload_path
        lib = S.load_library()
        c2 = WORKLOADS["c2"]

        def gpu_ms(fn, reps=200):
            """Average GPU time of fn() over `reps` back-to-back calls, by events on the current stream."""
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            e1.synchronize()
            return e0.elapsed_time(e1) / reps

        # signatures over windows (Section 5 of the paper): 32 paths of 1,024 segments, the c2 word set; 64 sliding
        # windows of 128 segments, and 64 expanding windows (0, 16 k); all (path, window) pairs advance in one launch
        wsw = S.sig_wordset_build_truncated(c2.d, c2.depth)
        wsw.upload("cuda:0")
        Bw, Lw, Kw, lenw = 32, 1024, 64, 128
        Xw = torch.from_numpy(make_path("iid", 77, Bw, Lw, wsw.dim)).cuda()
        shapes = {"sliding": [(k * (Lw - lenw) // (Kw - 1), k * (Lw - lenw) // (Kw - 1) + lenw) for k in range(Kw)],
                  "expanding": [(0, (k + 1) * (Lw // Kw)) for k in range(Kw)]}
        out["windows"] = {"workload": f"B={Bw} L={Lw} d={wsw.dim} |W|={wsw.size}, {Kw} windows"}
        for kind, wins in shapes.items():
            plan = S.WindowPlan(wsw, Xw, wins)
            gw = torch.randn((Bw, Kw, wsw.size), device="cuda")
            tf = gpu_ms(lambda: plan.forward())
            tb = gpu_ms(lambda: plan.backward(gw))
            seg = sum(r - l for l, r in wins)
            out["windows"][kind] = {"fwd_ms": round(tf, 4), "bwd_ms": round(tb, 4),
                                    "fwd_bwd_coeff_steps_per_s": round(Bw * seg * wsw.size / ((tf + tb) * 1e-3), 1)}

        # log-signature (Section 3.3) on the c2 shape: signature on the word set of the Lyndon words' factors, tensor
        # logarithm word by word, and back
        wsl = S.sig_wordset_build_logsig(c2.d, c2.depth)
        wsl.upload("cuda:0")
        Xl = torch.from_numpy(workload_path(c2)).cuda()
        cl = S.sig_forward(wsl, Xl)
        lg = S.sig_logsig_forward(wsl, cl)
        gl = torch.randn_like(lg)
        wfl = torch.empty(max(int(lib.sig_forward_workspace_bytes(wsl._h, c2.B, c2.L + 1)), 256), dtype=torch.uint8, device="cuda")
        wbl = torch.empty(max(int(lib.sig_backward_workspace_bytes(wsl._h, c2.B, c2.L + 1)), 256), dtype=torch.uint8, device="cuda")
        gpl = torch.empty_like(Xl)

        def logsig_fwd():
            S.sig_forward(wsl, Xl, out=cl, workspace=wfl)
            return S.sig_logsig_forward(wsl, cl)

        def logsig_bwd():
            S.sig_backward(wsl, Xl, cl, S.sig_logsig_backward(wsl, cl, gl), out=gpl, workspace=wbl)

        out["log_signature"] = {"workload": f"c2 shape, depth {c2.depth}: {wsl.size} signature words for {lg.shape[1]} "
                                            f"log-signature coordinates",
                                "kernels": [wsl.kernel_name(False, c2.B, c2.L + 1), wsl.kernel_name(True, c2.B, c2.L + 1)],
                                "fwd_ms": round(gpu_ms(logsig_fwd), 4), "bwd_ms": round(gpu_ms(logsig_bwd), 4),
                                "note": "GPU time, signature + tensor logarithm (forward) and their adjoints (backward)"}

        # shapes of the paper's own timing table (Section 5, Table 1: training step = forward + backward, float32,
        # one H200): synthetic random walks of the same shape; the paper's figure is context, another machine's
        table = {}
        for (Bp, Mp, dp, Np, paper_us) in [(32, 100, 6, 4, 207.52), (32, 100, 6, 5, 555.63), (32, 100, 6, 6, 3360.0),
                                           (64, 1000, 4, 6, 6450.0), (1, 200, 10, 4, 320.35),
                                           (256, 200, 10, 4, 9830.0)]:
            wsp = S.sig_wordset_build_truncated(dp, Np)
            wsp.upload("cuda:0")
            Xp = torch.from_numpy(make_path("iid", 7, Bp, Mp - 1, dp)).cuda()
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

        # few long paths: sig_backward cuts every path into time chunks by itself (Chen's relation, eq. 2; the chunk
        # signatures are recomputed); beside it the same backward pass over whole paths (sig_backward_static never chunks)
        c5w = WORKLOADS["c5"]
        wsf = S.sig_wordset_build_truncated(c5w.d, c5w.depth)
        wsf.upload("cuda:0")
        Bf, Lf = 8, 8192
        Xf = torch.from_numpy(make_path("iid", 91, Bf, Lf, wsf.dim)).cuda()
        cf = S.sig_forward(wsf, Xf)
        gf = torch.randn_like(cf)
        gpf = torch.empty_like(Xf)
        out["few_long_paths"] = {
            "workload": f"c5 word set, B={Bf} L={Lf}", "coeffs": wsf.size,
            "fwd_ms": round(gpu_ms(lambda: S.sig_forward(wsf, Xf, out=cf), 50), 4),
            "bwd_ms": round(gpu_ms(lambda: S.sig_backward(wsf, Xf, cf, gf, out=gpf), 50), 4),
            "bwd_ms_whole_paths": round(gpu_ms(lambda: S.sig_backward_static(wsf, Xf, cf, gf, gpf), 20), 4)}

        # the other word-set builders (host only): graph-induced set and the sparse lead-lag set of a 5-dimensional path
        t0 = time.perf_counter()
        g = S.sig_wordset_build_graph(10, [(a, b) for a in range(10) for b in range(10) if 0 < b - a <= 3], 6)
        t1 = time.perf_counter()
        ll = S.sig_wordset_build_leadlag_sparse(5, 4)
        t2 = time.perf_counter()
        out["other_word_sets"] = {"graph(d=10, edges i->i+1..i+3, depth 6)": {"words": g.size, "build_ms": round((t1 - t0) * 1e3, 3)},
                                  "leadlag_sparse(d=5, depth 4)": {"words": ll.size, "build_ms": round((t2 - t1) * 1e3, 3)}}

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
