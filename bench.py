"""Benchmark of cos_verify on one MI355X.

A step is one cos_verify call (all of softmax statistics, combine, acceptance
test, first rejection and the residual/bonus draw) on one batch of synthetic
logits that is already resident in HBM.  Prints ONE JSON line.
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

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak


def _traffic_from_profiles(workload: str):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary of this
    workload's shape (measured through the plain C++ driver, not in this run), or None."""
    path = os.path.join(ROOT, "profiles", f"cos_verify_{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":")[1])
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c5", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--batch", type=int, default=0, help="override B (debugging only; changes the workload name)")
    ap.add_argument("--cpu-rows", type=int, default=-1, help="batch rows the CPU oracle is timed on (-1 = auto, 0 = skip)")
    ap.add_argument("--chunk-vectors", type=int, default=0, help="tuning knob (0 = library heuristic)")
    ap.add_argument("--sample-blocks", type=int, default=0, help="tuning knob (0 = library heuristic)")
    ap.add_argument("--tail-sequences", type=int, default=0,
                    help="tuning knob: sequences at the end of the grid with shorter chunks (0 = library heuristic, < 0 = none)")
    ap.add_argument("--tail-factor", type=int, default=0, help="tuning knob: how many times shorter (0 = 4)")
    ap.add_argument("--stop-window", type=int, default=0,
                    help="verify this many positions per launch and never read past a sequence's first "
                         "rejection (0 = the headline step: every position read, one launch)")
    ap.add_argument("--extras", action="store_true",
                    help="also time the same step with stop_window = 1 (reported beside the headline as stop_window_1)")
    ap.add_argument("--skip-extras", action="store_true", help="accepted for older command lines; the default now")
    ap.add_argument("--with-alpha", action="store_true",
                    help="also compute the acceptance rates of Eq. (7) (an optional output, not the headline step)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (rows of the batch are independent, so several GPUs "
              "would each take a slice of the batch without any exchange). Re-run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2502_01662_amd import cos_verify as C
    from paper_2502_01662_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: needs a GPU; there is no CPU path", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = W.WORKLOADS[args.workload]
    if args.batch:
        w = w.scaled(B=args.batch, name=f"{w.name}_B{args.batch}")
    C.load_library()
    shape = C.LaunchShape(chunk_vectors=args.chunk_vectors, sample_blocks=args.sample_blocks,
                          tail_sequences=args.tail_sequences, tail_factor=args.tail_factor)

    t0 = time.time()
    # small workloads: rotate over distinct input sets so that the timed calls stream from HBM,
    # not from the 256 MB memory-side cache
    nsets = max(1, min(64, int(np.ceil(600e6 / w.logit_bytes)))) if w.logit_bytes < 600e6 else 1
    sets = [W.generate(w, device=dev, step=s) for s in range(nsets)]
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    dt = C.COS_DTYPE_F32 if w.dtype == "f32" else C.COS_DTYPE_BF16
    ws = C.allocate_workspace(w.n, w.B, w.gamma, w.V, dt, w.mode, dev, shape)
    alen = torch.empty(w.B, dtype=torch.int32, device=dev)
    toks = torch.empty((w.B, w.gamma + 1), dtype=torch.int32, device=dev)

    alpha = torch.empty((w.B, w.gamma), dtype=torch.float64, device=dev) if args.with_alpha else None

    # the serving loop's form of the call: one shape step after step on one workspace, so from the second
    # call on the workspace is promised ready (every call leaves its arrival counters at zero) and the
    # kernel that clears them is skipped
    from dataclasses import replace
    steady = replace(shape, workspace_ready=1)

    def step(i, events=None, first=False):
        s = sets[i % nsets]
        C.cos_verify(s["logits"], s["draft_tokens"], s["proposer_idx"], w.mode, w.weights,
                     s["u_accept"], s["u_resample"], accepted_len=alen, out_tokens=toks, workspace=ws,
                     alpha=alpha, stop_window=args.stop_window, shape=shape if first else steady, events=events)

    step(0, first=True)
    for i in range(args.warmup):
        step(i)
    # HIP events of this program, recorded by each call on its own stream around the kernel(s) that
    # read every logit: the dominant kernel's duration, measured live over the timed region
    timed_events = [C.make_events(dev) for _ in range(min(args.steps, 1024))]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(args.steps):
        step(i, timed_events[i % len(timed_events)])
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    kernel_ms = [a.elapsed_time(b) for a, b in timed_events]
    ms_per_step = (t2 - t1) * 1e3 / args.steps
    kavg = float(np.mean(kernel_ms))
    value = w.positions / (ms_per_step * 1e-3)

    achieved = w.logit_bytes / (kavg * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "contrastive_stats_kernel" if w.mode == W.CONTRASTIVE else "ensemble_stats_kernel",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": _traffic_from_profiles(args.workload),
                "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE through the plain C++ driver on this workload's "
                                  "shape; committed summary under profiles/, not measured in this run",
                "algorithmic_bytes_per_launch": w.logit_bytes, "kernel_avg_ms": round(kavg, 5),
                "kernel_min_ms": round(float(np.min(kernel_ms)), 5)}

    # ---- small workloads only: the same step on ONE input set, i.e. served from the memory-side cache;
    # labelled as such, never the headline ----
    cache_resident = None
    if nsets > 1:
        for i in range(args.warmup):
            step(0)
        torch.cuda.synchronize()
        r1 = time.perf_counter()
        for i in range(args.steps):
            step(0)
        torch.cuda.synchronize()
        cache_resident = round((time.perf_counter() - r1) * 1e3 / args.steps, 5)

    # ---- the same step with stop_window = 1 (opt-in: rows after a sequence's first rejection are
    # never read, one launch per position): reported beside the headline, never as `value` ----
    lazy = None
    if args.extras and args.stop_window == 0 and not args.with_alpha:
        def lazy_step(i):
            s = sets[i % nsets]
            C.cos_verify(s["logits"], s["draft_tokens"], s["proposer_idx"], w.mode, w.weights,
                         s["u_accept"], s["u_resample"], accepted_len=alen, out_tokens=toks, workspace=ws,
                         stop_window=1, shape=steady if i > 0 else shape)
        for i in range(args.warmup):
            lazy_step(i)
        torch.cuda.synchronize()
        l1 = time.perf_counter()
        for i in range(args.steps):
            lazy_step(i)
        torch.cuda.synchronize()
        l2 = time.perf_counter()
        lazy_ms = (l2 - l1) * 1e3 / args.steps
        lazy = {"ms_per_step": round(lazy_ms, 5), "value": round(w.positions / (lazy_ms * 1e-3), 1),
                "unit": "positions/s",
                "note": "identical outputs; logits after a sequence's first rejection are not read, so fewer "
                        "bytes than the algorithmic count move: not comparable with the HBM roofline"}

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same batch ----
    cpu = None
    parity = None
    cpu_rows = args.cpu_rows
    if cpu_rows < 0:
        # ~20-30 core-seconds for the two oracle passes: about 6 ns per logit element read
        per_row = w.n * (w.gamma + 1) * w.V * 3e-9
        cpu_rows = int(max(1, min(w.B, round(20.0 / per_row))))
    failed = False
    if cpu_rows > 0:
        from oracle import cos_oracle as O
        from tests import parity as P
        s = sets[0]
        rows = np.unique(np.linspace(0, w.B - 1, cpu_rows).round().astype(int))
        sel = torch.as_tensor(rows, device=dev)
        lg = W.host_logits(s["logits"][:, sel].contiguous())
        odt = O.DTYPE_F32 if w.dtype == "f32" else O.DTYPE_BF16
        hd, hp = s["draft_tokens"][sel].cpu().numpy(), s["proposer_idx"][sel].cpu().numpy()
        hua, hur = s["u_accept"][sel].cpu().numpy(), s["u_resample"][sel].cpu().numpy()
        threads = O.max_threads()
        # the same work as the GPU does: every position of every row (all_positions)
        c0 = time.perf_counter()
        res = O.verify(lg, odt, hd, hp, w.mode, list(w.weights), hua, hur, all_positions=True, num_threads=threads)
        c1 = time.perf_counter()
        assert res.status == 0
        # the sequential procedure as the paper states it: stops at each row's first rejection
        e0 = time.perf_counter()
        early = O.verify(lg, odt, hd, hp, w.mode, list(w.weights), hua, hur, all_positions=False, num_threads=threads)
        e1 = time.perf_counter()
        assert early.status == 0
        # per-core rate: the same oracle on one thread, on a few of those rows
        few = max(1, min(len(rows), 8))
        s0 = time.perf_counter()
        one = O.verify(lg[:, :few], odt, hd[:few], hp[:few], w.mode, list(w.weights), hua[:few], hur[:few],
                       all_positions=True, num_threads=1)
        s1 = time.perf_counter()
        assert one.status == 0
        read_frac = float(np.mean(np.minimum(early.accepted_len + 1, w.gamma + 1)) / (w.gamma + 1))
        cpu = {"value": round(len(rows) * w.gamma / (c1 - c0), 2), "unit": "positions/s",
               "early_stop_value": round(len(rows) * w.gamma / (e1 - e0), 2),
               "one_core_value": round(few * w.gamma / (s1 - s0), 2),
               "cores": int(min(threads, len(rows))), "kind": "oracle",
               "sample": f"{len(rows)} of {w.B} batch rows of {w.name}: float64 C oracle, OpenMP over rows; `value` reads "
                         f"every position of every row as the GPU does ({c1 - c0:.2f} s wall), `early_stop_value` stops at "
                         f"each row's first rejection and so reads {read_frac:.0%} of the logits ({e1 - e0:.2f} s wall)",
               "host_cpus": os.cpu_count()}
        # parity of the timed configuration on those rows: lengths, tokens, r(d), q(d), flags
        diag = C.Diagnostics.allocate(w.B, w.gamma, dev)
        C.cos_verify(s["logits"], s["draft_tokens"], s["proposer_idx"], w.mode, w.weights, s["u_accept"],
                     s["u_resample"], accepted_len=alen, out_tokens=toks, workspace=ws, diag=diag,
                     stop_window=args.stop_window, shape=steady)
        torch.cuda.synchronize()
        rep = P.compare(s, w.mode, w.weights, alen.cpu().numpy(), toks.cpu().numpy(), diag, rows=rows)
        parity = {"rows": rep.rows, "bit_exact_rows": rep.exact_rows,
                  "excused_accept_ties": rep.excused_accept_ties, "excused_cdf_ties": rep.excused_cdf_ties,
                  "unexcused_rows": len(rep.failures), "flag_mismatches": rep.flag_mismatches,
                  "max_rel_err_r": rep.max_rel_err_r, "max_rel_err_q": rep.max_rel_err_q,
                  "accepted_len_histogram": np.bincount(alen.cpu().numpy(), minlength=w.gamma + 1).tolist()}
        failed = (not rep.ok) or rep.exact_rows + rep.excused_accept_ties + rep.excused_cdf_ties != rep.rows
        for msg in rep.failures[:5]:
            print("bench.py: GPU/oracle mismatch:", msg, file=sys.stderr)

    out = {
        "metric": "verified positions/sec + achieved HBM GB/s of cos_verify (bf16 logits, 1 GPU)",
        "value": round(value, 1), "unit": "positions/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",
        "logit_storage": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "B": w.B, "gamma": w.gamma, "V": w.V,
                   "combine": "contrastive" if w.mode == W.CONTRASTIVE else "ensemble", "weights": list(w.weights),
                   "input_sets_rotated": nsets, "chunk_vectors": args.chunk_vectors,
                   "sample_blocks": args.sample_blocks, "tail_sequences": args.tail_sequences, "tail_factor": args.tail_factor, "acceptance_rate_output": bool(args.with_alpha), "workspace_ready": True,
                   "stop_window": args.stop_window},
        "achieved_hbm_gbs_per_step": round(w.logit_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roofline, "cpu_baseline": cpu, "parity_sample": parity, "stop_window_1": lazy,
        "cache_resident_ms_per_step": cache_resident,
        "input_generation_s": round(gen_s, 1),
    }
    print(json.dumps(out), flush=True)
    if failed:
        print("bench.py: the timed configuration does not match the oracle on the sampled rows", file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
