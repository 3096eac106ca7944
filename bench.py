#!/usr/bin/env python3
"""Benchmark of the linear-chain CRF hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4] [--no-cpu-baseline]

One "step" is one `lccrf_marginals` call over the whole synthetic batch: both log-semiring
chains, logZ, and the fused write of every edge marginal.  Inputs are resident in HBM before
the timed region starts.  The headline number is potentials per second, B*N*T*T / time per
step.  Prints exactly one JSON line on stdout; everything else goes to stderr.

Extra objects in the line:
  roofline      for the dominant kernel (the second pass, which re-reads phi and writes the
                marginals), timed with HIP events the library records on the launch stream
                between its passes: algorithmic bytes = (sizeof(phi element) + 4) per potential.
  cpu_baseline  the CPU oracle (as it stands, OpenMP over the batch) timed on this host on a
                bounded sample of the same workload.
  other_queries log-partition alone, Viterbi decode, entropy, the log-probability of a path, one sample, and the
                cross-entropy and KL divergence against a second chain, the semi-Markov log-partition over the same bytes,
                timed the same way (context).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X datasheet HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def stored_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (profiles/marginals_<workload>_traffic.txt, line `traffic_bytes_per_launch: N`), else None."""
    path = os.path.join(ROOT, "profiles", f"marginals_{workload}_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1].strip())
    except OSError:
        pass
    return None


def cpu_baseline(w, budget_s: float = 20.0):
    """Time the oracle's marginals on a bounded sample of the workload (whole sequences)."""
    import numpy as np
    import oracle
    from paper_2308_03291_amd import workloads
    threads = oracle.threads()
    lens = workloads.lengths(w)
    trans = workloads.shared_transitions(w)
    # calibrate on one sequence (or a prefix of it when sequences are very long)
    probe_pos = min(w.N, max(8, (1 << 22) // (w.T * w.T)))
    phi0 = workloads.phi_sequence(w, 0, trans)[:probe_pos].unsqueeze(0).contiguous()
    t0 = time.perf_counter()
    oracle.marginals(phi0, None)
    per_pot = (time.perf_counter() - t0) / (probe_pos * w.T * w.T)
    per_seq = per_pot * w.N * w.T * w.T
    nseq = int(max(1, min(w.B, budget_s * threads / max(per_seq, 1e-9) / 2)))
    import torch
    phi = torch.stack([workloads.phi_sequence(w, b, trans) for b in range(nseq)]).contiguous()
    sample_lens = lens[:nseq].numpy()
    cores = int(min(threads, nseq))
    # the same pass again until about 10 s of CPU work have been timed (a workload smaller than that is repeated)
    dt, reps = 0.0, 0
    while reps == 0 or (dt * cores < 10.0 and reps < 64):
        t0 = time.perf_counter()
        oracle.marginals(phi, sample_lens)
        dt += time.perf_counter() - t0
        reps += 1
    pots = nseq * w.N * w.T * w.T
    return {"value": reps * pots / dt, "unit": "potentials/s", "cores": cores, "kind": "oracle",
            "sample": f"fp64 oracle marginals on the first {nseq} of {w.B} sequences of {w.key} "
                      f"({pots} potentials a pass, {reps} passes, {dt:.2f} s wall, OpenMP over sequences)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-queries", action="store_true")
    ap.add_argument("--cold", action="store_true",
                    help="write a 512 MB scratch buffer before every timed call, so that nothing of the "
                         "workload is left in L2 or the 256 MB memory-side cache (matters for workloads "
                         "smaller than that; times then come from the per-call events, not the wall clock)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain elementwise kernel of known size (reads and writes exactly "
                         "4 bytes per potential) so that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                         "readings can be scaled to bytes")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (sequences are independent; sharding the batch over "
                 "GPUs needs no exchange and is not part of this run). Use --gpus 1.")

    import torch
    from paper_2308_03291_amd import binding as crf, workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    crf.load_library()
    dev = torch.device("cuda:0")
    w = workloads.WORKLOADS[args.workload]
    esz = 2 if w.dtype == "bf16" else 4
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    pots = w.B * w.N * w.T * w.T

    log(f"[bench] building {w.key}: B={w.B} N={w.N} T={w.T} {w.dtype} ({pots * esz / 1e6:.1f} MB of potentials)")
    t0 = time.perf_counter()
    phi = torch.empty(w.B, w.N, w.T, w.T, dtype=dt, device=dev)
    workloads.phi_batch(w, out=phi)
    lens_cpu = workloads.lengths(w)
    lens = lens_cpu.to(dev)
    eff_pots = int(lens_cpu.clamp(0, w.N).sum().item()) * w.T * w.T
    mu = torch.empty(w.B, w.N, w.T, w.T, dtype=torch.float32, device=dev)
    lz = torch.empty(w.B, dtype=torch.float32, device=dev)
    tags = torch.empty(w.B, w.N, dtype=torch.int32, device=dev)
    score = torch.empty(w.B, dtype=torch.float32, device=dev)
    ws = torch.empty(max(crf.workspace_bytes(op, w.B, w.N, w.T, 0 if esz == 4 else 1) for op in (0, 1, 2, 3, 4, 5, 6)),
                     dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    log(f"[bench] inputs resident after {time.perf_counter() - t0:.1f} s")

    def new_events(n):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        for e in evs:
            e.record()   # materialise the HIP handles
        torch.cuda.synchronize()
        return evs

    scratch = torch.empty(512 << 20, dtype=torch.uint8, device=dev) if args.cold else None

    def evict():
        if scratch is not None:
            scratch.add_(1)

    def run_step(evs=None):
        evict()
        if evs is None:
            crf.lccrf_marginals(phi, lens, out=mu, logZ=lz, workspace=ws)
        else:
            crf.lccrf_marginals_timed(phi, lens, mu, lz, ws, evs)

    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()

    # ---- the timed region: exactly K steps, bracketed by synchronisation
    per_step_events = [new_events(3) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for evs in per_step_events:
        run_step(evs)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    pass1 = [e[0].elapsed_time(e[1]) for e in per_step_events]
    pass2 = [e[1].elapsed_time(e[2]) for e in per_step_events]
    whole = [e[0].elapsed_time(e[2]) for e in per_step_events]
    # cold runs: the wall clock also holds the scratch writes, the events only the calls
    ms_per_step = sum(whole) / len(whole) if args.cold else wall * 1e3 / args.steps
    pass2_avg = sum(pass2) / len(pass2)
    log(f"[bench] {args.steps} steps: wall {ms_per_step:.4f} ms/step; events: call avg {sum(whole) / len(whole):.4f} ms "
        f"(pass 1 {sum(pass1) / len(pass1):.4f}, pass 2 {pass2_avg:.4f}), median call {median(whole):.4f} ms")

    value = pots / (ms_per_step * 1e-3)
    call_bytes = eff_pots * (2 * esz + 4)
    if crf.auto_algo(crf.OP_MARGINALS, w.B, w.N, w.T) == crf.ALGO_SCAN or (w.T <= 32 and 2 <= w.N <= 65):
        # Chunked scan: the interval after the boundary phases is one kernel that makes both passes over
        # every chunk (two reads of phi, the second from cache at best, and one write of mu).  Sequences of
        # at most 65 positions over at most 32 tags take the same kernel whole.
        kernel, alg_bytes = "wave_chunk_kernel", call_bytes
    else:
        # dominant kernel: second pass = one read of phi + one write of mu over the positions in the chains.
        # With few sequences and T = 128 that pass is the two-workgroups-per-chain kernel (plus two
        # few-microsecond helpers the event interval also covers: mailbox reset, exact fix-up launch).
        alg_bytes = eff_pots * (esz + 4)
        paired = w.T == 128 and 4 * w.B <= torch.cuda.get_device_properties(dev).multi_processor_count
        kernel = "pair_marginal_kernel" if paired else ("wave_marginal_kernel" if w.T <= 32 else "chain_marginal_kernel")
    achieved = alg_bytes / (pass2_avg * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": kernel,
                "achieved": achieved, "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": stored_traffic(w.key),
                "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_ms": pass2_avg,
                "whole_call": {"algorithmic_bytes": call_bytes, "avg_ms": sum(whole) / len(whole),
                               "achieved": call_bytes / (sum(whole) / len(whole) * 1e-3) / 1e9,
                               "frac": call_bytes / (sum(whole) / len(whole) * 1e-3) / 1e9 / HBM_PEAK_GBPS}}

    if args.pmc_calibration:
        cal_src = phi if esz == 4 else mu
        torch.add(cal_src, 1.0, out=mu)   # one float read + one float write per potential
        torch.cuda.synchronize()
        log(f"[bench] calibration kernel: elementwise add over {pots} floats "
            f"({pots * 4} bytes read, {pots * 4} bytes written)")

    other = None
    if not args.no_other_queries:
        other = {}
        crf.lccrf_argmax(phi, lens, out=tags, score=score, workspace=ws)   # a path to score: the best one
        path = tags.clamp(min=0)
        uniforms = torch.rand(w.B, w.N, device=dev, generator=torch.Generator(device=dev).manual_seed(1))
        # a second chain for the two-chain queries: half-scale potentials, in the marginals' buffer when the types agree
        if esz == 4:
            phi_q = torch.mul(phi, 0.5, out=mu)
        else:
            phi_q = (phi.float() * 0.5).to(phi.dtype)
        for name, fn, bpp in (
                ("log_partition", lambda: crf.lccrf_log_partition(phi, lens, out=lz, workspace=ws), esz),
                ("argmax", lambda: crf.lccrf_argmax(phi, lens, out=tags, score=score, workspace=ws), esz),
                ("entropy", lambda: crf.lccrf_entropy(phi, lens, out=score, workspace=ws), esz),
                ("log_prob", lambda: crf.lccrf_log_prob(phi, path, lens, out=score, workspace=ws), esz),
                ("sample", lambda: crf.lccrf_sample(phi, uniforms, lens, out=tags, workspace=ws), esz),
                ("cross_entropy", lambda: crf.lccrf_cross_entropy(phi, phi_q, lens, out=score, workspace=ws), 3 * esz),
                ("kl_divergence", lambda: crf.lccrf_kl_divergence(phi, phi_q, lens, out=score, workspace=ws), 3 * esz),
                # the same bytes read as a semi-Markov CRF: N / 8 positions, segments of up to 8 positions
                ("semi_markov_log_partition_k8",
                 (lambda: crf.lccrf_semi_markov_log_partition(phi.view(w.B, w.N // 8, 8, w.T, w.T), out=score))
                 if w.N % 8 == 0 else None, esz)):
            if fn is None:
                continue
            for _ in range(2):
                fn()
            evs = new_events(2 * max(5, args.steps // 2))
            for k in range(0, len(evs), 2):
                evict()
                evs[k].record()
                fn()
                evs[k + 1].record()
            torch.cuda.synchronize()
            ts = [evs[k].elapsed_time(evs[k + 1]) for k in range(0, len(evs), 2)]
            ms = median(ts)
            other[name] = {"ms": ms, "potentials_per_s": pots / (ms * 1e-3),
                           "hbm_frac": eff_pots * bpp / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
            log(f"[bench] {name}: {ms:.4f} ms")

    base = None
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a sample ...")
        base = cpu_baseline(w)
        log(f"[bench] oracle: {base['value'] / 1e6:.1f} Mpot/s on {base['cores']} threads")

    out = {
        "metric": "linear-chain CRF marginals: potentials/sec (B*N*T^2/s)", "value": value, "unit": "potentials/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if esz == 4 else "bf16-in/f32",
        "data": "synthetic",
        "config": {"workload": f"{w.key}: B={w.B} N={w.N} T={w.T} {w.dtype} phi, lengths U[{w.len_lo},{w.len_hi}], "
                               f"seeded {w.kind} potentials (scale {w.scale})",
                   "query": "lccrf_marginals (logZ + all edge marginals)", "caches": "cold" if args.cold else "warm",
                   "potentials": pots,
                   "effective_potentials": eff_pots},
        "roofline": roofline, "cpu_baseline": base,
    }
    if other is not None:
        out["other_queries"] = other
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
