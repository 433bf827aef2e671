#!/usr/bin/env python3
"""Benchmark of the DBA step on one MI355X.

python bench.py [--gpus 1] [--steps K] [--warmup W]

A "step" is one dba_step call: the whole hot path (score add, top-k, row best, constraint
gather, state update, banks, allocation, new beam) for one [B,k,V] log-prob tensor that is
already resident in HBM.  Workload: config 4 (B=64, k=20, V=32000, 32 constraint tokens per
sentence, decodes of 100 steps).  Steps beyond the 100th start the next decode (contexts are
initialised before the timed region).  Inputs rotate over several distinct resident tensors so
that the 164 MB per step cannot be served from the 256 MB Infinity Cache.

Prints ONE JSON line.  `value` = steps/s (wall clock, synchronised on both sides);
`roofline.achieved` = algorithmic bytes per step / average duration of one step's launches
(dba_stream_kernel, which reads the log-probs, followed by dba_merge_kernel), measured with HIP
events on the launch stream over the timed region - the two kernels run back to back with no
gap, so this is the sum of their durations; profiles/ holds the rocprofv3 split of the two.
`reference_read` = a kernel of the library that only reads the same tensors once (row maxima),
timed the same way: what the device delivers for this access pattern with no selection work.
`cpu_baseline` = the CPU oracle timed on the host's cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
# HBM bytes per step (fetched + written by its two launches) on the config-4 workload, from the
# rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in profiles/ (scaled against a plain copy), and
# the digest of the kernel sources those counters were taken with: the line carries the figure only
# while the sources are still those, null otherwise.
TRAFFIC_BYTES_PER_LAUNCH = 168729167
TRAFFIC_KERNEL_SHA16 = "fcace5d29b7358dc"


def kernel_sources_sha16() -> str:
    import hashlib
    m = hashlib.sha256()
    for name in ("dba.hip", "dba_kernels.hpp", "wave_topk.hpp"):
        with open(os.path.join(ROOT, "paper_1804_06609_amd", "csrc", name), "rb") as fh:
            text = fh.read()
        if name == "dba.hip":                    # the kernels come first in that file; the host side is not hashed
            text = text.split(b"// host side")[0]
        m.update(text)
    return m.hexdigest()[:16]


def build_workload(cfg: int, cons_tokens):
    import synth_inputs as si
    wl = si.make_config(cfg)
    if cons_tokens is not None:
        wl.constraints = si.fixed_total_constraints(wl.seed, wl.B, wl.V, cons_tokens)
    wl.eos_switch = 1 << 30      # every timed row stays live: EOS keeps its low logit
    return wl


def timed_steps(wl, dev, K, W, dlen, repeats, options=None):
    """Median wall seconds and event milliseconds of K steps (fresh contexts every repeat)."""
    import torch
    from paper_1804_06609_amd.session import Session
    toks, poff, soff = wl.csr()
    R = len(dev)
    stream = torch.cuda.current_stream()
    wall, evms = [], []
    for _ in range(repeats):
        n_dec = (W + K + dlen - 1) // dlen
        sessions = [Session(wl.B, wl.k, wl.V, dlen, wl.eos_id, wl.pad_id, toks, poff, soff, options=options)
                    for _ in range(n_dec)]
        g = 0
        for _ in range(W):
            sessions[g // dlen].step(dev[g % R])
            g += 1
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(K):
            sessions[g // dlen].step(dev[g % R])
            g += 1
        e1.record(stream)
        torch.cuda.synchronize()
        wall.append(time.perf_counter() - t0)
        evms.append(e0.elapsed_time(e1))
        for s in sessions:
            s.close()
    return float(np.median(wall)), float(np.median(evms))


_DECODE_STREAMS = []


def concurrent_decodes(wl, dev, K, W, dlen, repeats, n_decodes, options=None):
    """Several independent decodes of the same workload in flight at once, each context on a stream of
    its own (default priority): what a server with more than one batch to translate does.  A step still
    depends on the step before it of the same decode, but one decode's per-sentence merge and launch
    latencies are filled with another decode's streaming.  So that the host's launch rate (Python) does
    not limit three decodes, the K steps of every decode are recorded beforehand into a HIP graph of
    its own (kernel nodes only) and the timed region launches the graphs side by side; if recording
    fails the steps are enqueued in turn instead.  options: dba_set_option settings of every context.
    Returns (median wall-clock microseconds per step, all decodes together; how the steps were submitted)."""
    import torch
    from paper_1804_06609_amd.session import Session
    toks, poff, soff = wl.csr()
    R = len(dev)
    while len(_DECODE_STREAMS) < n_decodes:      # made once and used again: streams share four hardware queues,
        _DECODE_STREAMS.append(torch.cuda.Stream())   # and streams made one after the other get different ones
    streams = _DECODE_STREAMS[:n_decodes]
    per_step = []
    how = "one HIP graph per decode"
    for _ in range(repeats):
        n_dec = (W + K + dlen - 1) // dlen
        ses = [[Session(wl.B, wl.k, wl.V, dlen, wl.eos_id, wl.pad_id, toks, poff, soff, stream=st, options=options)
                for _ in range(n_dec)] for st in streams]
        torch.cuda.synchronize()

        def enqueue(i, first, n):                # the decodes read different tensors at any one time
            for g in range(first, first + n):
                ses[i][g // dlen].step(dev[(g + 3 * i) % R])

        for i in range(n_decodes):
            enqueue(i, 0, W)
        torch.cuda.synchronize()
        graphs = []
        if how.startswith("one HIP graph"):
            try:
                for i, st in enumerate(streams):
                    gr = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(gr, stream=st):
                        enqueue(i, W, K)
                    graphs.append(gr)
                torch.cuda.synchronize()
            except Exception as exc:
                print(f"bench.py: HIP graph capture failed ({exc}); concurrent decodes are enqueued step by step",
                      file=sys.stderr)
                how, graphs = "steps enqueued in turn", []
                break
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if graphs:
            for st, gr in zip(streams, graphs):
                with torch.cuda.stream(st):
                    gr.replay()
        else:
            for g in range(W, W + K):
                for i in range(n_decodes):
                    ses[i][g // dlen].step(dev[(g + 3 * i) % R])
        torch.cuda.synchronize()
        per_step.append((time.perf_counter() - t0) / (K * n_decodes) * 1e6)
        del graphs
        for row in ses:
            for x in row:
                x.close()
    if not per_step:                             # recording failed in the first repeat: eager throughout
        for _ in range(repeats):
            n_dec = (W + K + dlen - 1) // dlen
            ses = [[Session(wl.B, wl.k, wl.V, dlen, wl.eos_id, wl.pad_id, toks, poff, soff, stream=st,
                            options=options)
                    for _ in range(n_dec)] for st in streams]
            for g in range(W):
                for i in range(n_decodes):
                    ses[i][g // dlen].step(dev[(g + 3 * i) % R])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for g in range(W, W + K):
                for i in range(n_decodes):
                    ses[i][g // dlen].step(dev[(g + 3 * i) % R])
            torch.cuda.synchronize()
            per_step.append((time.perf_counter() - t0) / (K * n_decodes) * 1e6)
            for row in ses:
                for x in row:
                    x.close()
    return float(np.median(per_step)), how


def flatness_pair(base_wl, dev, K, W, dlen, repeats):
    """Sec. 1 / Table 1, inside the headline line: the same resident tensors decoded with exactly 1
    and exactly 32 constraint tokens per sentence, the two legs taking turns; median event time per
    step of each."""
    import synth_inputs as si
    ms = {"1": [], "32": []}
    wls = {}
    for c in (1, 32):
        wl = si.make_config(4)
        wl.constraints = si.fixed_total_constraints(base_wl.seed, base_wl.B, base_wl.V, c)
        wl.eos_switch = 1 << 30
        wls[str(c)] = wl
    for _ in range(repeats):
        for c in ("1", "32"):
            _, ev_ms = timed_steps(wls[c], dev, K, W, dlen, 1)
            ms[c].append(ev_ms / K)
    med = {c: float(np.median(v)) for c, v in ms.items()}
    return {"1": med["1"], "32": med["32"], "max_over_min": max(med.values()) / min(med.values()),
            "unit": "ms/step (HIP events)", "steps": K, "repeats": repeats,
            "what": "config-4 shapes and tensors, exactly 1 vs exactly 32 constraint tokens per sentence"}


def gbs_simulation(args):
    """Sec. 5 / Fig. 4 on synthetic inputs: the paper simulates grid beam search inside DBA with a
    beam of b(C+1) and the adjustment off, and reports its time growing with the number of
    constraints C while DBA at a fixed beam stays flat.  Here: B = 64, V = 32000, C single-token
    constraints per sentence, base beam b = 4 -> k = b(C+1), adjustment off, against DBA at k = 20
    with the adjustment on, same C; step time from HIP events, median of the repeats."""
    import torch
    import synth_inputs as si
    from paper_1804_06609_amd import DBA_OPT_ADJUSTMENT
    torch.cuda.set_device(0)
    B, V, b = 64, 32000, 4
    cache = {}

    def tensors(k):
        if k not in cache:
            cache.clear()                      # one beam width resident at a time
            gen = si.Workload(B=B, k=k, V=V, T=100, seed=si.BASE_SEED + 40 + k, constraints=[[] for _ in range(B)])
            gen.eos_switch = 1 << 30
            need = max(2, -(-600_000_000 // (4 * B * k * V)))      # more than the 256 MB Infinity Cache in rotation
            cache[k] = [torch.from_numpy(gen.logp(t)).cuda() for t in range(min(need, 8))]
        return cache[k]

    Cs = (0, 1, 3, 7, 15)
    rows = [{"C": C} for C in Cs]
    # all legs of one beam width together, so that its tensors are generated once
    legs = [("gbs_sim", i, b * (C + 1), 0) for i, C in enumerate(Cs)] + [("dba", i, 20, 1) for i in range(len(Cs))]
    for name, i, k, adjust in legs:
        cons = si.fixed_total_constraints(si.BASE_SEED + 50, B, V, Cs[i], max_len=1)
        wl = si.Workload(B=B, k=k, V=V, T=100, seed=si.BASE_SEED + 60, constraints=cons)
        wl.eos_switch = 1 << 30
        _, ev_ms = timed_steps(wl, tensors(k), args.steps, args.warmup, 100, max(3, args.repeats),
                               {DBA_OPT_ADJUSTMENT: adjust})
        rows[i][name] = {"k": k, "us_per_step": ev_ms * 1e3 / args.steps}
    print(json.dumps({"metric": "step time vs number of constraints: simulated grid beam search (beam b(C+1), no "
                                "adjustment) against DBA at a fixed beam", "unit": "us/step",
                      "config": {"workload": f"B={B} V={V}, C single-token constraints per sentence, base beam b={b}; "
                                             "DBA at k=20"},
                      "rows": rows, "steps": args.steps, "warmup": args.warmup, "n_gpus": 1, "data": "synthetic",
                      "gbs_over_dba_at_C15": rows[-1]["gbs_sim"]["us_per_step"] / rows[-1]["dba"]["us_per_step"],
                      "dba_max_over_min": max(r["dba"]["us_per_step"] for r in rows) /
                      min(r["dba"]["us_per_step"] for r in rows)}))


def flatness(args):
    """Sec. 1 / Table 1: the cost of a DBA step does not grow with the number of constraints."""
    import torch
    torch.cuda.set_device(0)
    res = {}
    dev = None
    for c in (1, 2, 4, 8, 16, 32):
        wl = build_workload(args.config, c)
        if dev is None:           # the log-probs do not depend on the constraints
            dev = [torch.from_numpy(wl.logp(t)).cuda() for t in range(max(1, args.tensors))]
        wall_s, _ = timed_steps(wl, dev, args.steps, args.warmup, args.decode_len or wl.T, max(3, args.repeats))
        res[str(c)] = wall_s * 1e3 / args.steps
    vals = list(res.values())
    print(json.dumps({"metric": "DBA ms/step vs constraint tokens per sentence", "unit": "ms",
                      "config": {"workload": f"config{args.config} shapes, exactly C constraint tokens per sentence"},
                      "ms_per_step": res, "max_over_min": max(vals) / min(vals), "steps": args.steps,
                      "warmup": args.warmup, "n_gpus": 1, "data": "synthetic"}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload (default: the headline config 4)")
    ap.add_argument("--cons-tokens", type=int, default=None,
                    help="override: exactly this many constraint tokens per sentence (flatness sweep)")
    ap.add_argument("--tensors", type=int, default=8, help="distinct resident input tensors to rotate over")
    ap.add_argument("--decode-len", type=int, default=None, help="steps per decode (default: the config's)")
    ap.add_argument("--repeats", type=int, default=5, help="timed repetitions; the median is reported")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--flatness", action="store_true",
                    help="instead of the headline line: step time for 1,2,4,8,16,32 constraint tokens per "
                         "sentence (the paper's O(1)-in-C claim), one JSON line")
    ap.add_argument("--gbs-sim", action="store_true",
                    help="instead of the headline line: Sec. 5 / Fig. 4 on synthetic inputs - step time of the "
                         "simulated grid beam search (beam 4(C+1), no adjustment) and of DBA at k=20 for "
                         "C = 0,1,3,7,15 constraints, one JSON line")
    ap.add_argument("--no-flatness", action="store_true", help="leave the 1-vs-32-token legs out of the headline line")
    ap.add_argument("--no-concurrent", action="store_true",
                    help="leave the legs with 2 and 3 decodes in flight out of the headline line")
    ap.add_argument("--logp-format", choices=["f32", "f16", "bf16"], default="f32",
                    help="element type of the resident log-prob tensors (default f32, the headline workload); "
                         "16-bit tensors halve the algorithmic bytes, the sums stay fp32")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain device copy of one input tensor (known size) a few times, so "
                         "that a counter run can scale FETCH_SIZE / WRITE_SIZE against it")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library runs on ONE GPU; sentences shard across GPUs without any "
              "exchange, so a multi-GPU figure would be N independent copies of this run. "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth_inputs as si
    from paper_1804_06609_amd.session import Session

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    if args.flatness:
        return flatness(args)
    if args.gbs_sim:
        return gbs_simulation(args)

    wl = build_workload(args.config, args.cons_tokens)
    B, k, V = wl.B, wl.k, wl.V
    K, W, R = args.steps, args.warmup, max(1, args.tensors)
    dlen = args.decode_len or wl.T
    toks, poff, soff = wl.csr()

    # resident inputs
    host = [wl.logp(t) for t in range(R)]
    esize = 4
    if args.logp_format == "f32":
        dev = [torch.from_numpy(h).cuda() for h in host]
    else:
        tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[args.logp_format]
        bits = [si.narrow16(h, args.logp_format) for h in host]
        dev = [torch.from_numpy(x.view(np.int16)).cuda().view(tdt) for x in bits]
        esize = 2
    torch.cuda.synchronize()

    wall_s, ev_ms = timed_steps(wl, dev, K, W, dlen, args.repeats)

    # algorithmic bytes: every live row's V log-probs once.  The first step of a decode has one
    # live row, all later steps k (EOS never fires in this workload).
    live_rows = 0
    for g in range(W, W + K):
        live_rows += B * (1 if g % dlen == 0 else k)
    bytes_total = float(esize) * live_rows * V
    launches = K
    achieved = bytes_total / launches / (ev_ms * 1e-3 / launches) / 1e9

    ntok = sorted({wl.n_tokens(b) for b in range(B)})
    ctok_desc = str(ntok[0]) if len(ntok) == 1 else f"{ntok[0]}..{ntok[-1]}"
    out = {
        "metric": "DBA steps/sec",
        "value": K / wall_s,
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": wall_s * 1e3 / K,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if esize == 4 else f"f32 sums, {args.logp_format} log-probs",
        "data": "synthetic",
        "config": {
            "workload": f"config{args.config}: B={B} k={k} V={V}, {ctok_desc} constraint tokens/sentence, "
                        f"decodes of {dlen} steps, {R} rotating resident {args.logp_format} tensors",
            "batch": B, "beam": k, "vocab": V, "decode_len": dlen,
        },
        "selection_GBps": bytes_total / wall_s / 1e9,
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": TRAFFIC_BYTES_PER_LAUNCH
            if (args.config == 4 and args.cons_tokens is None and esize == 4 and
                kernel_sources_sha16() == TRAFFIC_KERNEL_SHA16) else None,
            "kernel": "dba_stream_kernel + dba_merge_kernel (the two launches of one step, back to back)",
            "us_per_launch": ev_ms * 1e3 / launches,
            "algorithmic_bytes_per_launch": bytes_total / launches,
        },
    }

    # the reference read: the same tensors, the same loads, no selection work (f32 tensors only)
    if esize == 4:
        from paper_1804_06609_amd import dba_debug_row_max
        sink = torch.empty(B * k, dtype=torch.float32, device="cuda")
        stream = torch.cuda.current_stream()
        reps = 200
        for i in range(20):
            dba_debug_row_max(dev[i % R].data_ptr(), B * k, V, sink.data_ptr(), stream.cuda_stream)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(reps):
            dba_debug_row_max(dev[i % R].data_ptr(), B * k, V, sink.data_ptr(), stream.cuda_stream)
        e1.record(stream)
        torch.cuda.synchronize()
        read_us = e0.elapsed_time(e1) * 1e3 / reps
        full_step_us = ev_ms * 1e3 / launches * (4.0 * B * k * V) / (bytes_total / launches)
        out["reference_read"] = {
            "kernel": "dba_row_max_kernel (reads each [B,k,V] tensor once with the stream phase's loads)",
            "us_per_launch": read_us,
            "GBps": 4.0 * B * k * V / read_us / 1e3,
            "step_over_read": full_step_us / read_us,
        }

    # Sec. 1 / Table 1: the step's cost does not depend on the number of constraints
    if args.config == 4 and esize == 4 and not args.no_flatness and args.cons_tokens is None:
        out["flatness"] = flatness_pair(wl, dev, max(K, 200), W, dlen, max(3, args.repeats))

    # more than one decode in flight: the same kernels, the serial chain of one decode hidden by another
    if args.config == 4 and esize == 4 and not args.no_concurrent and args.cons_tokens is None:
        from paper_1804_06609_amd import DBA_OPT_MERGE_WAVES

        def leg(n, options):
            us, how = concurrent_decodes(wl, dev, max(K, 200), W, dlen, max(3, args.repeats), n, options)
            return {"us_per_step": us, "steps_per_s": 1e6 / us, "GBps": 4.0 * B * k * V / us / 1e3,
                    "frac_of_hbm_peak": 4.0 * B * k * V / us / 1e3 / HBM_PEAK_GBS, "submission": how}

        cd = {str(n): leg(n, None) for n in (2, 3)}
        cd["four_wave_merge"] = {str(n): leg(n, {DBA_OPT_MERGE_WAVES: 4}) for n in (2, 3)}
        cd["what"] = ("aggregate over 2 / 3 independent config-4 decodes, each context on a stream of its own (wall "
                      "clock); `value` and `roofline` above are ONE decode, whose every step waits for the one before. "
                      "four_wave_merge: the same with DBA_OPT_MERGE_WAVES = 4 (smaller workgroups in the second "
                      "launch, placed more easily on a busy GPU; the default is chosen for one decode)")
        out["concurrent_decodes"] = cd

    if args.copy_probe:
        dst = torch.empty_like(dev[0])
        for i in range(4):
            dst.copy_(dev[i % R])        # reads 4*B*k*V bytes, writes as many
        torch.cuda.synchronize()
        out["copy_probe_bytes_each_way"] = esize * B * k * V

    if not args.no_cpu_baseline:
        import oracle
        threads = min(16, os.cpu_count() or 1)
        S = 40 if args.config == 4 else 4      # about 16 core-seconds of oracle work at config 4
        ob = oracle.BatchBeam(k, V, wl.constraints, wl.eos_id, wl.pad_id)
        ses = Session(B, k, V, S, wl.eos_id, wl.pad_id, toks, poff, soff)
        if esize == 2:
            host = [oracle.widen16(x, args.logp_format) for x in bits]
        want = []                              # the oracle's beam after every step of the sample
        cpu_s = 0.0
        for t in range(S):
            t0 = time.perf_counter()
            ob.step(host[t % R], threads=threads)
            cpu_s += time.perf_counter() - t0
            want.append(tuple(ob.stacked(n).tobytes() for n in ("token", "backptr", "score", "flags", "met")))
        same = True
        for t in range(S):                     # every step of the sample is compared, not only the last
            ses.step(dev[t % R])
            g_tok, g_bp, g_sc, g_fl = ses.outputs()
            got = (g_tok.tobytes(), g_bp.tobytes(), g_sc.tobytes(), g_fl.tobytes(), ses.state()["met_mask"].tobytes())
            same = same and got == want[t]
        ses.close()
        # the same oracle on one core, on a shorter sample (a step there takes about 0.4 s at config 4)
        S1 = 4 if args.config == 4 else 1
        ob1 = oracle.BatchBeam(k, V, wl.constraints, wl.eos_id, wl.pad_id)
        t0 = time.perf_counter()
        for t in range(S1):
            ob1.step(host[t % R], threads=1)
        cpu1_s = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": S / cpu_s, "unit": "steps/s", "cores": threads, "kind": "oracle",
            "sample": f"first {S} steps of the same workload, all {B} sentences, one sentence per thread",
            "gpu_matches_oracle_on_sample": bool(same),
            "one_core": {"value": S1 / cpu1_s, "unit": "steps/s", "cores": 1,
                         "sample": f"first {S1} steps of the same workload, all {B} sentences"},
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
