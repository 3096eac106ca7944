#!/usr/bin/env python3
"""Benchmark of the linear-chain CRF hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4] [--no-cpu-baseline]
                    [--no-per-config] [--no-other-queries] [--cold] [--ceilings]

One "step" is one `lccrf_marginals` call over the whole synthetic batch: both log-semiring
chains, logZ, and the fused write of every edge marginal.  Inputs are resident in HBM before
the timed region starts.  The headline number is potentials per second, B*N*T*T / time per
step, on the headline workload (cfg4).  Prints exactly one JSON line on stdout; everything else
goes to stderr.

Extra objects in the line:
  roofline      for the dominant kernel (the second pass, which re-reads phi and writes the
                marginals), timed with HIP events the library records on the launch stream
                between its passes: algorithmic bytes = (sizeof(phi element) + 4) per potential.
  cpu_baseline  the CPU oracle (as it stands, OpenMP over the batch) timed on this host on a
                bounded sample of the same workload.
  per_config    every other synthetic workload (cfg1, cfg2, cfg3, cfg5 and the paper's own benchmark
                shape) and the headline one: marginals, log-partition and argmax timed call by call
                with HIP events (median and minimum), with warm caches and, for working sets below the
                256 MB memory-side cache, cold (a 512 MB scratch buffer is rewritten before every
                call); algorithmic bytes over the positions inside the chains, the fraction of the HBM
                peak they amount to, the bound that applies, and the parity of the same buffers
                against the oracle (max |mu - oracle|, relative logZ error, Viterbi paths).
  stream_ceilings  what 128 / 256 / 1024 workgroups of this chip read, and read + write, streaming
                contiguous regions (the library's instrumentation probe): the practical ceilings
                beside the datasheet peak.
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
CACHE_BYTES = 256 << 20  # memory-side cache: smaller working sets are also timed cold
PER_CONFIG = ("cfg1", "cfg2", "cfg3", "cfg5", "paper_lccrf")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def committed_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (profiles/marginals_<workload>_traffic.txt, line `traffic_bytes_per_launch: N`), else None.
    Counters cannot be read from inside the run; the summary names the command that made it."""
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
    import oracle
    import torch
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
            "single_thread_value": 1.0 / per_pot,  # the calibration pass: one sequence (a prefix of it), one thread
            "sample": f"fp64 oracle marginals on the first {nseq} of {w.B} sequences of {w.key} "
                      f"({pots} potentials a pass, {reps} passes, {dt:.2f} s wall, OpenMP over sequences)"}


class Timer:
    """Times single calls with a pair of HIP events on the current stream."""

    def __init__(self, torch, scratch):
        self.torch, self.scratch = torch, scratch

    def events(self, n):
        evs = [self.torch.cuda.Event(enable_timing=True) for _ in range(n)]
        for e in evs:
            e.record()   # materialise the HIP handles
        self.torch.cuda.synchronize()
        return evs

    def evict(self):
        self.scratch.add_(1)   # rewrites 512 MB: nothing of the workload stays in L2 or the memory-side cache

    def run(self, fn, calls, cold):
        for _ in range(2):
            fn()
        evs = self.events(2 * calls)
        for k in range(0, len(evs), 2):
            if cold:
                self.evict()
            evs[k].record()
            fn()
            evs[k + 1].record()
        self.torch.cuda.synchronize()
        ts = [evs[k].elapsed_time(evs[k + 1]) * 1e3 for k in range(0, len(evs), 2)]
        return {"median_us": median(ts), "min_us": min(ts), "calls": calls}


def parity(crf, oracle, phi_cpu, lens_cpu, lz, mu, score, tags, pick):
    """The GPU results of sequences `pick` against the oracle on the same inputs."""
    import numpy as np
    sub = phi_cpu[pick].contiguous()
    ln = lens_cpu[pick].numpy()
    want_lz, want_mu = oracle.marginals(sub, ln)
    want_score, want_tags, gap = oracle.viterbi(sub, ln)
    got_lz = lz[pick].cpu().numpy().astype(np.float64)
    mu_err = float(np.abs(mu[pick].cpu().numpy() - want_mu).max())
    lz_err = float((np.abs(got_lz - want_lz) / np.maximum(1.0, np.abs(want_lz))).max())
    sc_err = float((np.abs(score[pick].cpu().numpy() - want_score) / np.maximum(1.0, np.abs(want_score))).max())
    got_tags = tags[pick].cpu().numpy()
    clear = gap > 1e-3
    same = [bool(np.array_equal(got_tags[k], want_tags[k])) for k in range(len(pick))]
    return {"sequences_checked": len(pick), "max_abs_marginal_error": mu_err, "max_rel_logz_error": lz_err,
            "max_rel_score_error": sc_err, "paths_with_clear_gap": int(clear.sum()),
            "paths_identical_where_gap_clear": int(sum(s for s, c in zip(same, clear) if c))}


def bound_of(w, algo_scan, longest):
    """The ceiling that applies to a workload, as its measurements show (profiles/ holds the counters)."""
    bytes_marg = w.B * w.N * w.T * w.T * ((2 if w.dtype == "bf16" else 4) * 2 + 4)
    if w.key == "cfg4":
        return "hbm"
    if bytes_marg < (32 << 20):
        return "latency: launches plus the serial depth of the chains; the batch is far too small to load the chip"
    return ("latency: serial depth of " + ("the scan's three phases" if algo_scan else f"{longest // 2} dependent steps per half chain")
            + " at about one wave per SIMD; HBM fraction reported for scale")


def bench_config(crf, workloads, oracle, torch, timer, key, calls, dev, with_parity=True):
    w = workloads.WORKLOADS[key]
    esz = 2 if w.dtype == "bf16" else 4
    phi_cpu = workloads.phi_batch(w)
    lens_cpu = workloads.lengths(w)
    phi, lens = phi_cpu.to(dev), lens_cpu.to(dev)
    dtc = crf.LCCRF_BF16 if esz == 2 else crf.LCCRF_F32
    mu = torch.empty(w.B, w.N, w.T, w.T, dtype=torch.float32, device=dev)
    lz = torch.empty(w.B, dtype=torch.float32, device=dev)
    lz1 = torch.empty(w.B, dtype=torch.float32, device=dev)
    tags = torch.empty(w.B, w.N, dtype=torch.int32, device=dev)
    score = torch.empty(w.B, dtype=torch.float32, device=dev)
    ws = torch.empty(max(crf.workspace_bytes(op, w.B, w.N, w.T, dtc) for op in (0, 1, 2)), dtype=torch.uint8, device=dev)
    pots = w.B * w.N * w.T * w.T
    eff_pos = int(lens_cpu.clamp(0, w.N).sum().item())
    eff_pots = eff_pos * w.T * w.T
    working_set = pots * (esz + 4)
    queries = {
        "marginals": (lambda: crf.lccrf_marginals(phi, lens, out=mu, logZ=lz, workspace=ws), 2 * esz + 4, crf.OP_MARGINALS),
        "log_partition": (lambda: crf.lccrf_log_partition(phi, lens, out=lz1, workspace=ws), esz, crf.OP_LOGZ),
        "argmax": (lambda: crf.lccrf_argmax(phi, lens, out=tags, score=score, workspace=ws), esz, crf.OP_ARGMAX),
    }
    out = {"shape": {"B": w.B, "N": w.N, "T": w.T, "dtype": w.dtype}, "potentials": pots,
           "effective_potentials": eff_pots, "working_set_bytes": working_set, "queries": {}}
    scan_any = False
    for name, (fn, bpp, op) in queries.items():
        taken = crf.auto_algo(op, w.B, w.N, w.T)
        scan = taken == crf.ALGO_SCAN
        scan_any = scan_any or (scan and name == "marginals")
        lanes_label = "sequential (chain wave + helper waves)" if name == "argmax" else "sequential (chain wave + producer waves)"
        q = {"schedule": "scan" if scan else lanes_label if taken == crf.ALGO_SEQUENTIAL_LANES
             else "sequential", "algorithmic_bytes": eff_pots * bpp,
             "warm": timer.run(fn, calls, cold=False)}
        states = ["warm"]
        if working_set < CACHE_BYTES:
            q["cold"] = timer.run(fn, calls, cold=True)
            states.append("cold")
        for st in states:
            t = q[st]["median_us"] * 1e-6
            q[st]["potentials_per_s"] = pots / t
            q[st]["effective_potentials_per_s"] = eff_pots / t
            q[st]["hbm_frac"] = eff_pots * bpp / t / 1e9 / HBM_PEAK_GBPS
        out["queries"][name] = q
    out["bound"] = bound_of(w, scan_any, int(lens_cpu.max().item()))
    m = out["queries"]["marginals"]
    log(f"[bench] {key}: marginals {m['warm']['median_us']:.1f} us warm"
        + (f" / {m['cold']['median_us']:.1f} us cold ({100 * m['cold']['hbm_frac']:.1f} % of HBM peak)" if "cold" in m else "")
        + f", logZ {out['queries']['log_partition']['warm']['median_us']:.1f}, argmax {out['queries']['argmax']['warm']['median_us']:.1f}")
    if with_parity:
        torch.cuda.synchronize()
        out["parity"] = parity(crf, oracle, phi_cpu, lens_cpu, lz, mu, score, tags, list(range(w.B)))
    return out


def stream_ceilings(crf, torch, src, dst, timer_events):
    """What G workgroups stream (read only; read + write), GB/s, best of 5."""
    sink = torch.zeros(1, dtype=torch.float32, device=src.device)
    out = {}
    for G in (64, 128, 256, 512, 1024, 4096):
        for mode, d in (("read", None), ("read_write", dst)):
            best = None
            for _ in range(6):
                a, b = timer_events(2)
                a.record()
                nbytes = crf.lccrf_stream_probe(src, d, G, sink)
                b.record()
                torch.cuda.synchronize()
                ms = a.elapsed_time(b)
                best = ms if best is None else min(best, ms)
            moved = nbytes * (2 if d is not None else 1)
            out[f"{mode}_{G}wg"] = {"GB_per_s": moved / (best * 1e-3) / 1e9, "ms": best, "bytes": moved}
            log(f"[bench] stream probe {mode:10s} {G:5d} workgroups: {moved / (best * 1e-3) / 1e9:7.1f} GB/s")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--algo", default="auto", choices=("auto", "sequential", "scan", "lanes"),
                    help="schedule of the timed marginals call (profiles of a schedule AUTO would not take)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-queries", action="store_true")
    ap.add_argument("--no-per-config", action="store_true")
    ap.add_argument("--calls", type=int, default=30, help="timed calls per query and cache state in per_config")
    ap.add_argument("--cold", action="store_true",
                    help="write a 512 MB scratch buffer before every timed call, so that nothing of the "
                         "workload is left in L2 or the 256 MB memory-side cache (matters for workloads "
                         "smaller than that; times then come from the per-call events, not the wall clock)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain elementwise kernel of known size (reads and writes exactly "
                         "4 bytes per potential) so that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                         "readings can be scaled to bytes")
    ap.add_argument("--ceilings", action="store_true",
                    help="only run the streaming probe (what G workgroups read and write) and print its table")
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

    def new_events(n):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        for e in evs:
            e.record()   # materialise the HIP handles
        torch.cuda.synchronize()
        return evs

    if args.ceilings:
        src = torch.zeros(1 << 29, dtype=torch.float32, device=dev)   # 2 GiB each
        dst = torch.empty_like(src)
        print(json.dumps({"stream_ceilings": stream_ceilings(crf, torch, src, dst, new_events),
                          "hbm_peak_GB_per_s": HBM_PEAK_GBPS}), flush=True)
        return

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

    scratch = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
    timer = Timer(torch, scratch)

    def evict():
        if args.cold:
            scratch.add_(1)

    algo = {"auto": crf.ALGO_AUTO, "sequential": crf.ALGO_SEQUENTIAL, "scan": crf.ALGO_SCAN,
            "lanes": crf.ALGO_SEQUENTIAL_LANES}[args.algo]

    def run_step(evs=None):
        evict()
        if evs is None:
            crf.lccrf_marginals(phi, lens, out=mu, logZ=lz, workspace=ws, algo=algo)
        else:
            crf.lccrf_marginals_timed(phi, lens, mu, lz, ws, evs, algo)

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
    auto_taken = crf.auto_algo(crf.OP_MARGINALS, w.B, w.N, w.T)
    scan_taken = algo == crf.ALGO_SCAN or (algo == crf.ALGO_AUTO and auto_taken == crf.ALGO_SCAN)
    lanes_taken = algo == crf.ALGO_SEQUENTIAL_LANES or (algo == crf.ALGO_AUTO and auto_taken == crf.ALGO_SEQUENTIAL_LANES)
    if lanes_taken:
        # second pass of the chain-wave / producer-wave kernels: one read of phi + one write of mu
        kernel, alg_bytes = "lane_chain_kernel (second pass)", eff_pots * (esz + 4)
    elif w.T <= 32 and (scan_taken or 2 <= w.N <= 65):
        # Chunked scan: the interval after the boundary phases is one kernel that makes both passes over
        # every chunk (two reads of phi, the second from cache at best, and one write of mu).  Sequences of
        # at most 65 positions over at most 32 tags take the same kernel whole.
        kernel, alg_bytes = "wave_chunk_kernel", call_bytes
    elif scan_taken:
        # 33 .. 64 tags under the scan: after the boundary phases the chunks run the two passes of the chain kernels
        kernel, alg_bytes = "chain_marginal_kernel (chunks; the interval also holds the chunks' first pass)", call_bytes
    else:
        # dominant kernel: second pass = one read of phi + one write of mu over the positions in the chains.
        # With few sequences and T = 128 that pass is the two-workgroups-per-chain kernel (plus two
        # few-microsecond helpers the event interval also covers: mailbox reset, exact fix-up launch).
        alg_bytes = eff_pots * (esz + 4)
        paired = w.T == 128 and 4 * w.B <= torch.cuda.get_device_properties(dev).multi_processor_count
        kernel = "pair_marginal_kernel" if paired else ("wave_marginal_kernel" if w.T <= 32 else
                                                        "stream_chain_kernel" if w.T > 128 else "chain_marginal_kernel")
    achieved = alg_bytes / (pass2_avg * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": kernel,
                "achieved": achieved, "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                # counters cannot be read inside the run: this figure comes from the committed rocprofv3 --pmc summary
                "traffic": committed_traffic(w.key), "traffic_source": f"profiles/marginals_{w.key}_traffic.txt (committed)",
                "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_ms": pass2_avg,
                "first_pass": {"kernel": "lane_chain_kernel (first pass)" if lanes_taken else "chain_half_kernel",
                               "algorithmic_bytes": eff_pots * esz,
                               "avg_ms": sum(pass1) / len(pass1),
                               "frac": eff_pots * esz / (sum(pass1) / len(pass1) * 1e-3) / 1e9 / HBM_PEAK_GBPS},
                "whole_call": {"algorithmic_bytes": call_bytes, "avg_ms": sum(whole) / len(whole),
                               "achieved": call_bytes / (sum(whole) / len(whole) * 1e-3) / 1e9,
                               "frac": call_bytes / (sum(whole) / len(whole) * 1e-3) / 1e9 / HBM_PEAK_GBPS}}

    if args.pmc_calibration:
        cal_src = phi if esz == 4 else mu
        torch.add(cal_src, 1.0, out=mu)   # one float read + one float write per potential
        torch.cuda.synchronize()
        log(f"[bench] calibration kernel: elementwise add over {pots} floats "
            f"({pots * 4} bytes read, {pots * 4} bytes written)")

    per_config = None
    ceilings = None
    if not args.no_per_config:
        import oracle
        # the headline workload: the three main queries call by call, and parity of these very buffers on 8 sequences
        crf.lccrf_marginals(phi, lens, out=mu, logZ=lz, workspace=ws)
        crf.lccrf_argmax(phi, lens, out=tags, score=score, workspace=ws)
        torch.cuda.synchronize()
        head = {"shape": {"B": w.B, "N": w.N, "T": w.T, "dtype": w.dtype}, "potentials": pots,
                "effective_potentials": eff_pots, "working_set_bytes": pots * (esz + 4), "queries": {}, "bound": "hbm"}
        pick = list(range(0, w.B, max(1, w.B // 8)))[:8]
        sub = torch.stack([workloads.phi_sequence(w, b, workloads.shared_transitions(w)) for b in pick])
        head["parity"] = parity(crf, oracle, sub, lens_cpu[pick], lz[pick], mu[pick], score[pick], tags[pick],
                                list(range(len(pick))))
        del sub
        lz1 = torch.empty_like(lz)
        for name, fn, bpp in (
                ("marginals", lambda: crf.lccrf_marginals(phi, lens, out=mu, logZ=lz, workspace=ws), 2 * esz + 4),
                ("log_partition", lambda: crf.lccrf_log_partition(phi, lens, out=lz1, workspace=ws), esz),
                ("argmax", lambda: crf.lccrf_argmax(phi, lens, out=tags, score=score, workspace=ws), esz)):
            state = "warm" if pots * (esz + 4) < CACHE_BYTES else "cold"   # larger than the cache: every call is cold
            q = {"schedule": "sequential", "algorithmic_bytes": eff_pots * bpp, state: timer.run(fn, args.calls, cold=False)}
            t = q[state]["median_us"] * 1e-6
            q[state].update(potentials_per_s=pots / t, effective_potentials_per_s=eff_pots / t,
                            hbm_frac=eff_pots * bpp / t / 1e9 / HBM_PEAK_GBPS)
            head["queries"][name] = q
        per_config = {w.key: head}
        log(f"[bench] {w.key}: parity on {len(pick)} sequences: max |mu - oracle| = {head['parity']['max_abs_marginal_error']:.2e}")
        # the stream probe on the headline buffers (2 GiB read, 2 GiB written)
        if esz == 4 and pots * 4 >= (1 << 30):
            ceilings = stream_ceilings(crf, torch, phi, mu, new_events)
        for key in PER_CONFIG:
            if key != w.key:
                per_config[key] = bench_config(crf, workloads, oracle, torch, timer, key, args.calls, dev)

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
                   "query": "lccrf_marginals (logZ + all edge marginals)", "schedule": args.algo,
                   "caches": "cold" if args.cold else "warm",
                   "potentials": pots,
                   "effective_potentials": eff_pots},
        "roofline": roofline, "cpu_baseline": base,
    }
    if per_config is not None:
        out["per_config"] = per_config
    if ceilings is not None:
        out["stream_ceilings"] = ceilings
    if other is not None:
        out["other_queries"] = other
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
