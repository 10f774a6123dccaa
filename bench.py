#!/usr/bin/env python3
"""Benchmark: per-sentence token-ID BLEU sentences/s on one MI355X, with roofline and CPU baseline.

A "step" is one pass of the whole hot path (n-gram extraction .. geometric mean) over one
synthetic batch already resident in HBM.  The default workload is the headline configuration
(B=512 candidates of 1024 tokens, 4 references each, vocabulary 50257).  One JSON line is
printed: `value` = sentences/s of the whole call, `roofline` = the dominant kernel's algorithmic
bytes per launch over its HIP-event duration against the 8 TB/s HBM peak (plus its measured HBM
traffic and instruction counts, parsed from the committed rocprofv3 summaries under profiles/),
`passes` = every
kernel of the path that ran, `global_path` = the staged pipeline's passes timed one by one,
`achievable_hbm_GBps` = plain fill / read / copy kernels in the same run, `cpu_baseline` = the CPU
oracle on a bounded sample of the same workload.
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

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak


def algorithmic_bytes(w, lay, N, token_bytes=4):
    """Bytes each pass must move by the method itself (tokens, keys, ids, statistics)."""
    T = w.tokens * token_bytes // 4      # tokens counted in 4-byte units
    G = [w.ngrams(n) for n in range(1, N + 1)]
    kb = [lay.key_bytes[n] for n in range(N)]
    stats = 8 * w.B * N
    return {
        "pack": 4 * T + sum(k * g for k, g in zip(kb, G)),
        "dictionary": sum((k + 4) * g for k, g in zip(kb, G)),
        "count_clip": 4 * sum(G) + stats,
        "finalize": stats + 4 * w.B * (1 + w.R) + 4 * w.B,
        "fused": 4 * T + 4 * w.B + stats,
    }


_SLEEP_CYCLES_PER_MS = None


def _block_stream(ms, torch):
    """Keep the GPU busy for about `ms` milliseconds (torch's spin kernel on the current stream),
    so that the host can enqueue the timed launches ahead of the GPU."""
    global _SLEEP_CYCLES_PER_MS
    if _SLEEP_CYCLES_PER_MS is None:
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        torch.cuda._sleep(2_000_000)
        b.record()
        torch.cuda.synchronize()
        _SLEEP_CYCLES_PER_MS = 2_000_000 / max(a.elapsed_time(b), 1e-3)
    torch.cuda._sleep(int(ms * _SLEEP_CYCLES_PER_MS))


def time_region(fn, iters, torch):
    """Average milliseconds of GPU time of `fn` over `iters` back-to-back launches, timed with HIP
    events recorded on the stream the kernels are launched on (torch's current stream).  A call
    through Python costs 8-12 us of host time, more than some of the kernels take; so a spin
    kernel first holds the stream while the host enqueues start event, launches and stop event:
    the events then bracket GPU execution, not the host's enqueue rate."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(8):
        fn()
    host_ms = (time.perf_counter() - t0) / 8
    torch.cuda.synchronize()
    _block_stream(host_ms * iters * 2.0 + 0.5, torch)
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / iters


def achievable_hbm(torch, dev):
    """What plain device kernels reach on this machine, in the same run: a fill (write only), a sum
    (read only) and a copy, at a size like the GLOBAL path's arrays (128 MiB: partly served by
    the 256 MB last-level cache) and at 1 GiB (beyond it).  GB/s of bytes read + written."""
    out = {}
    for mib in (128, 1024):
        n = mib * 1024 * 1024 // 8
        x = torch.empty(n, dtype=torch.int64, device=dev)
        y = torch.empty_like(x)
        x.fill_(1)
        y.fill_(1)
        b = mib * 1024 * 1024
        for name, fn, nbytes in (("fill", lambda: y.fill_(7), b), ("read", lambda: x.sum(), b),
                                 ("copy", lambda: y.copy_(x), 2 * b)):
            for _ in range(3):
                fn()
            ms = time_region(fn, 20, torch)
            out[f"{name}_{mib}MiB"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
        del x, y
    return out


def cpu_baseline(w, run, gpu=None, budget_s=10.0):
    """The oracle, as it stands, on the host cores: sentences/s on a bounded sample, with all
    threads and with one; `gpu` (scores, clipped, total, closest length of the timed call, as
    numpy arrays) is compared with the oracle's results on the same sample."""
    import numpy as np
    import oracle
    cores = len(os.sched_getaffinity(0))
    threads = min(cores, 16)
    args = dict(max_n=w.max_n, weights=w.weights, smoothing=run.smoothing,
                smooth_param=run.smooth_param)

    def timed(sample, nthreads):
        t0 = time.time()
        res = oracle.bleu(sample.cand, sample.cand_len, sample.refs, sample.ref_len,
                          threads=nthreads, **args)
        return time.time() - t0, res

    # a small probe fixes the sample: as much of the workload as about budget_s of CPU work
    # (three repetitions with all threads) allows
    probe = w.subset(min(w.B, 4 * threads))
    dt, _ = timed(probe, threads)
    rate = probe.B / max(dt, 1e-6)
    sample = w.subset(int(min(w.B, max(probe.B, rate * budget_s / 3))))
    best, res = None, None
    for _ in range(3):
        dt, res = timed(sample, threads)
        best = dt if best is None else min(best, dt)
    single = w.subset(min(sample.B, max(8, int(rate / threads))))      # about a second
    dt1, _ = timed(single, 1)
    what = "the whole workload" if sample.B == w.B else f"first {sample.B} sentence groups"
    out = {"value": sample.B / best, "unit": "sentences/s", "cores": threads,
           "cores_available": cores, "kind": "oracle",
           "sample": f"{what}, best of 3, {threads} std::threads over sentences",
           "value_1_thread": single.B / dt1,
           "sample_1_thread": f"first {single.B} sentence groups, one run"}
    if gpu is not None:
        k = sample.B
        out["parity_on_sample"] = {
            "max_abs_dbleu": float(np.abs(gpu["bleu"][:k].astype(np.float64) - res.bleu).max()),
            "clipped_exact": bool(np.array_equal(gpu["clipped"][:k], res.clipped)),
            "total_exact": bool(np.array_equal(gpu["total"][:k], res.total)),
            "closest_ref_len_exact": bool(np.array_equal(gpu["closest"][:k],
                                                         res.closest_ref_len))}
    return out


def other_configs(skip, steps, torch, tb, syn, np, dev):
    """The remaining benchmark configurations and the long-generation workload (128 candidates of
    8192 tokens, one reference each) in short form: sentences/s of the default path and
    the three main GLOBAL passes as fractions of the HBM peak.  A failure is recorded, not
    raised: it must not take the headline line with it."""
    rows = []
    for k in (1, 2, 3, 4, 5, "long"):   # "long": the long-generation workload of --long-form 8192
        if k == skip:
            continue
        try:
            w = syn.long_form() if k == "long" else syn.make(k)
            run = [r for r in w.runs if not r.corpus][-1]
            to = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
            cand, cl, refs, rl = to(w.cand), to(w.cand_len), to(w.refs), to(w.ref_len)
            cs, rs = int(w.cand.shape[1]), int(w.refs.shape[2])
            mk = lambda path: tb.make_config(max_n=w.max_n, weights=w.weights,
                                             smoothing=run.smoothing,
                                             smooth_param=run.smooth_param, vocab_size=w.vocab,
                                             path=path)
            cfg = mk("auto")
            lay = tb.tensorbleu_workspace_layout(w.B, w.R, cs, rs, cfg)
            ws = tb.allocate_workspace(w.B, w.R, cs, rs, cfg, dev)
            out = torch.empty(w.B, dtype=torch.float32, device=dev)
            fn = lambda: tb.tensorbleu_sentence(cand, cl, refs, rl, cfg, out=out, workspace=ws)
            for _ in range(5):
                fn()
            ms = time_region(fn, steps, torch)
            row = {"workload": w.name, "path": {1: "fused", 2: "global"}[lay.path],
                   "us": round(ms * 1e3, 2), "sentences_per_s": round(w.B / (ms * 1e-3), 1)}
            if lay.global_ok:
                gcfg = mk("global")
                glay = tb.tensorbleu_workspace_layout(w.B, w.R, cs, rs, gcfg)
                gws = tb.allocate_workspace(w.B, w.R, cs, rs, gcfg, dev)
                alg = algorithmic_bytes(w, glay, w.max_n)
                tb.tensorbleu_sentence(cand, cl, refs, rl, gcfg, out=out, workspace=gws)
                stages = {
                    "pack": lambda: tb.tensorbleu_pack(cand, cl, refs, rl, gcfg, gws),
                    "dictionary": lambda: tb.tensorbleu_dictionary(cl, rl, cs, rs, gcfg, gws),
                    "count_clip": lambda: tb.tensorbleu_count_clip(cl, rl, cs, rs, gcfg, gws)}
                for name, st in stages.items():
                    for _ in range(3):
                        st()
                    t_ms = time_region(st, steps, torch)
                    row[name + "_us"] = round(t_ms * 1e3, 2)
                    row[name + "_frac_hbm"] = round(alg[name] / (t_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                                    4)
            rows.append(row)
            del cand, refs, ws
        except Exception as err:       # noqa: BLE001 - reported in the output line
            rows.append({"config": k, "error": repr(err)})
    return rows


# Which kernels implement which pass (names as they appear in the rocprofv3 summaries).
PASS_KERNELS = {
    "fused": ("fused_kernel",),
    "pack": ("pack_kernel",),
    "dictionary": ("hier_dictionary_kernel", "dictionary_narrow_kernel", "dictionary_wide_kernel",
                   "part_dictionary_kernel", "big_dictionary_kernel"),
    "count_clip": ("hier_count_kernel", "count_fields_kernel", "count_clip_kernel",
                   "part_count_kernel", "big_count_kernel"),
    "finalize": ("sentence_score_kernel",),
}
NUM_CUS, CLOCK_GHZ = 256, 2.4
# Issue rates measured with micro-benchmarks on this GPU (wavefront instructions per CU-cycle at
# full occupancy): vector ALU alone, scalar ALU alone (one scalar unit per CU), both kinds mixed.
ISSUE_PEAK = {"valu": 1.5, "salu": 1.0, "mixed": 1.7}


def paper_grid(steps, torch, tb, syn, np, dev):
    """The sizes the paper tabulates (its Section 5.1): sequence lengths 256 and 1024, batch
    sizes 16..512, one reference each (the paper states none; workloads as configuration 1 at
    these sizes).  Per size: device time per call with the host queued ahead, and the paper's
    protocol, the mean wall-clock time of 5 calls each synchronised on its own (Section 4.2)."""
    rows = []
    for L in (256, 1024):
        for B in (16, 32, 64, 128, 256, 512):
            w = syn.config1(B=B, L=L)
            run = [r for r in w.runs if not r.corpus][-1]
            to = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
            cand, cl, refs, rl = to(w.cand), to(w.cand_len), to(w.refs), to(w.ref_len)
            cs, rs = int(w.cand.shape[1]), int(w.refs.shape[2])
            cfg = tb.make_config(max_n=w.max_n, weights=w.weights, smoothing=run.smoothing,
                                 smooth_param=run.smooth_param, vocab_size=w.vocab, path="auto")
            ws = tb.allocate_workspace(w.B, w.R, cs, rs, cfg, dev)
            out = torch.empty(w.B, dtype=torch.float32, device=dev)
            fn = lambda: tb.tensorbleu_sentence(cand, cl, refs, rl, cfg, out=out, workspace=ws)
            for _ in range(5):
                fn()
            ms = time_region(fn, steps, torch)
            runs = []
            for _ in range(5):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                fn()
                torch.cuda.synchronize()
                runs.append((time.perf_counter() - t0) * 1e3)
            rows.append({"L": L, "B": B, "R": w.R, "vocab": w.vocab, "device_us": round(ms * 1e3, 2),
                         "sentences_per_s": round(B / (ms * 1e-3), 1),
                         "ms_mean_of_5_synchronised_calls": round(sum(runs) / 5, 4)})
    return rows


def profile_counters(workload, pass_name):
    """Counters of the kernel that implements `pass_name`, read from the committed rocprofv3
    summary profiles/pmc_<workload>.md (sections '## `kernel`' with '* COUNTER: value' lines;
    values are means per launch).  Returns (kernel name, {counter: value}) or (None, {}) when no
    summary exists for the workload or the kernel."""
    path = os.path.join(ROOT, "profiles", f"pmc_{workload}.md")
    if not os.path.exists(path):
        return None, {}
    best = (None, {})
    kernel, counters = None, {}
    for line in open(path).read().splitlines() + ["## `end`"]:
        if line.startswith("## `"):
            if kernel and any(k in kernel for k in PASS_KERNELS[pass_name]) and \
                    counters.get("SQ_WAVES", 0) >= best[1].get("SQ_WAVES", -1):
                best = (kernel, counters)          # several instantiations: the largest launch
            kernel, counters = line[4:].rstrip("`"), {}
        elif line.startswith("* ") and ":" in line and kernel:
            name, value = line[2:].split(":", 1)
            if "traffic" in name:                  # "... = 10.89 MB"
                try:
                    counters["hbm_traffic_bytes"] = float(value.split("=")[-1].split()[0]) * 1e6
                except ValueError:
                    pass
            else:
                try:
                    counters[name.strip()] = float(value.replace(",", ""))
                except ValueError:
                    pass
    return best


def issue_model(counters, kernel_us):
    """Time the kernel's instruction stream needs at the measured issue peaks, against its
    measured duration."""
    valu, salu = counters.get("SQ_INSTS_VALU"), counters.get("SQ_INSTS_SALU")
    if valu is None or salu is None:
        return None
    cycles = max(valu / ISSUE_PEAK["valu"], salu / ISSUE_PEAK["salu"],
                 (valu + salu) / ISSUE_PEAK["mixed"]) / NUM_CUS
    issue_us = cycles / (CLOCK_GHZ * 1e3)
    return {"valu_wave_instr": valu, "salu_wave_instr": salu,
            "issue_peaks_per_cu_cycle": ISSUE_PEAK, "issue_us_at_peak": round(issue_us, 2),
            "frac_of_kernel_time": round(issue_us / kernel_us, 3)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (3 = headline)")
    ap.add_argument("--path", default="auto", choices=["auto", "fused", "global"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-hbm-ceiling", action="store_true",
                    help="skip the fill / read / copy bandwidth check of plain device kernels")
    ap.add_argument("--rouge", type=int, default=0, metavar="N",
                    help="also time ROUGE-N (tensorrouge_n, order N) on the same batch")
    ap.add_argument("--int64", action="store_true",
                    help="feed int64 token ids (the usual tokenizer dtype) instead of int32")
    ap.add_argument("--long-form", type=int, default=0, metavar="L",
                    help="instead of a benchmark configuration: 128 candidates of about L tokens "
                         "with one reference each (groups beyond one LDS table for L > 6144)")
    ap.add_argument("--long-batch", type=int, default=128, metavar="B",
                    help="with --long-form: the number of candidates")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short measurements of the other benchmark configurations")
    ap.add_argument("--paper-grid", action="store_true",
                    help="also time the sizes the paper tabulates (L = 256 and 1024, B = 16..512)")
    ap.add_argument("--no-global-passes", action="store_true",
                    help="skip the per-pass timing of the GLOBAL path")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="launch one plain device copy of this many MiB first (a known-size "
                         "reference for the FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch of the dominant kernel from rocprofv3 --pmc")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); sentence groups are "
              "independent, so N GPUs would each score B/N groups with no exchange",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2510_05485_amd as tb
    import synth_inputs as syn

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    tb.load_library()
    dev = "cuda:0"
    if a.calib_copy_mib:
        src = torch.ones(a.calib_copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    w = syn.long_form(B=a.long_batch, L=a.long_form) if a.long_form else syn.make(a.config)
    run = [r for r in w.runs if not r.corpus][-1]
    N = w.max_n
    to = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    cand, cl, refs, rl = to(w.cand), to(w.cand_len), to(w.refs), to(w.ref_len)
    if a.int64:
        cand, refs = cand.long(), refs.long()
    cs, rs = int(w.cand.shape[1]), int(w.refs.shape[2])

    def config(path):
        return tb.make_config(max_n=N, weights=w.weights, smoothing=run.smoothing,
                              smooth_param=run.smooth_param, vocab_size=w.vocab, path=path)

    cfg = config(a.path)
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, cs, rs, cfg)
    path = {1: "fused", 2: "global"}[lay.path]
    ws = tb.allocate_workspace(w.B, w.R, cs, rs, cfg, dev)
    out = torch.empty(w.B, dtype=torch.float32, device=dev)
    stats = tb.Stats.allocate(w.B, N, dev, corpus_stats=False)

    def step():
        tb.tensorbleu_sentence(cand, cl, refs, rl, cfg, out=out, stats=stats, workspace=ws)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / a.steps
    ev_ms = time_region(step, a.steps, torch)
    ms = max(wall_ms, ev_ms)    # enqueue-bound runs show up in wall time, GPU-bound in events

    def time_stages(stages, alg):
        rows = []
        for name, fn in stages:
            for _ in range(3):
                fn()
            t_ms = time_region(fn, a.steps, torch)
            gbps = alg[name] / (t_ms * 1e-3) / 1e9
            rows.append({"kernel": name, "us": round(t_ms * 1e3, 2),
                         "alg_bytes": int(alg[name]), "GBps": round(gbps, 1),
                         "frac_hbm": round(gbps / HBM_PEAK_GBPS, 4)})
        return rows

    # per-kernel durations, each kernel on its own between HIP events
    glay = tb.tensorbleu_workspace_layout(w.B, w.R, cs, rs, config("global")) \
        if lay.global_ok else None
    alg = algorithmic_bytes(w, glay or lay, N, 8 if a.int64 else 4)
    global_section = None
    if glay is not None and not (a.no_global_passes and path != "global"):
        gcfg = config("global")
        gws = ws if path == "global" else tb.allocate_workspace(w.B, w.R, cs, rs, gcfg, dev)
        gstages = [
            ("pack", lambda: tb.tensorbleu_pack(cand, cl, refs, rl, gcfg, gws, stats)),
            ("dictionary", lambda: tb.tensorbleu_dictionary(cl, rl, cs, rs, gcfg, gws, stats)),
            ("count_clip", lambda: tb.tensorbleu_count_clip(cl, rl, cs, rs, gcfg, gws, stats)),
            ("finalize", lambda: tb.tensorbleu_finalize(cl, rl, cs, rs, gcfg, False, out, gws,
                                                        stats)),
        ]
        grows = time_stages(gstages, alg)

        def gstep():
            tb.tensorbleu_sentence(cand, cl, refs, rl, gcfg, out=out, stats=stats, workspace=gws)
        gstep()
        g_ms = time_region(gstep, a.steps, torch)
        global_section = {"ms_per_step": round(g_ms, 5),
                          "sentences_per_s": round(w.B / (g_ms * 1e-3), 1), "passes": grows}
    if path == "global":
        passes = global_section["passes"]
    else:
        passes = time_stages([("fused", step)], alg)
    dom = max(passes, key=lambda p: p["us"])
    prof_kernel, counters = profile_counters(w.name, dom["kernel"])
    traffic = a.traffic_bytes if a.traffic_bytes is not None else counters.get("hbm_traffic_bytes")
    roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["GBps"],
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": dom["frac_hbm"],
                "traffic": traffic,
                "traffic_source": (f"profiles/pmc_{w.name}.md ({prof_kernel})" if traffic and
                                   a.traffic_bytes is None else
                                   "command line" if traffic else
                                   "no rocprofv3 summary committed for this workload")}
    model = issue_model(counters, dom["us"])
    if model is not None:
        roofline["instruction_issue"] = model

    # the paper's protocol beside it (its Section 4.2): mean wall-clock time of 5 single calls,
    # each synchronised on its own (launch and synchronisation latency included)
    runs = []
    for _ in range(5):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        runs.append((time.perf_counter() - t0) * 1e3)
    paper_protocol = {"ms_mean_of_5_synchronised_calls": round(sum(runs) / 5, 5),
                      "sentences_per_s": round(w.B / (sum(runs) / 5 * 1e-3), 1)}

    result = {
        "metric": "per-sentence BLEU sentences/sec at B=512, L=1024; % HBM roofline",
        "value": round(w.B / (ms * 1e-3), 1), "unit": "sentences/s", "n_gpus": 1,
        "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("u32 keys / u16 counts / f32 scores" if path == "fused"
                  else "u64 keys / u16 counts / f32 scores") + (" (int64 ids)" if a.int64 else ""),
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "R": w.R, "cand_stride": cs, "ref_stride": rs,
                   "vocab": w.vocab, "max_n": N, "smoothing": run.smoothing, "path": path,
                   "tokens": w.tokens},
        "ms_per_step_events": round(ev_ms, 5), "ms_per_step_wall": round(wall_ms, 5),
        "roofline": roofline, "passes": passes, "paper_protocol": paper_protocol,
    }
    if global_section is not None and path != "global":
        result["global_path"] = global_section
    if a.paper_grid:
        result["paper_grid"] = paper_grid(a.steps, torch, tb, syn, np, dev)
    if a.rouge:
        # the ROUGE-N extension on the same batch (same kernel family, order a.rouge)
        rws = tb.allocate_workspace(w.B, w.R, cs, rs, tb.make_config(
            max_n=a.rouge, vocab_size=w.vocab, path="auto"), dev)
        rfn = lambda: tb.tensorrouge_n(cand, cl, refs, rl, n=a.rouge, vocab_size=w.vocab,
                                       workspace=rws)
        for _ in range(a.warmup):
            rfn()
        r_ms = time_region(rfn, a.steps, torch)
        result["rouge"] = {"n": a.rouge, "us": round(r_ms * 1e3, 2),
                           "sentences_per_s": round(w.B / (r_ms * 1e-3), 1),
                           "frac_hbm": round(alg["fused"] / (r_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
    if not a.no_other_configs:
        result["other_configs"] = other_configs("long" if (a.long_form, a.long_batch) == (8192, 128) else
                                                0 if a.long_form else a.config, min(a.steps, 100),
                                                torch, tb, syn, np, dev)
    if not a.no_hbm_ceiling:
        result["achievable_hbm_GBps"] = achievable_hbm(torch, dev)
    if not a.no_cpu_baseline:
        step()
        torch.cuda.synchronize()
        gpu = {"bleu": out.cpu().numpy(), "clipped": stats.clipped.cpu().numpy(),
               "total": stats.total.cpu().numpy(), "closest": stats.closest_ref_len.cpu().numpy()}
        result["cpu_baseline"] = cpu_baseline(w, run, gpu)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
