#!/usr/bin/env python3
"""Benchmark of the verification step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config hybrid]

A step is one pass of the whole hot path over one synthetic batch, inputs resident in HBM:
spec_verify_attn -> spec_lm_head -> spec_accept -> spec_kv_commit.  Prints ONE JSON line: verified
tokens/s (sum of accepted drafts + bonus tokens per wall-clock second) on the named workload (default: the
hybrid ordinary-parallel mix, the largest one), the roofline figures of the dominant kernel measured with HIP
events on the launch stream, per-call timings, the ceilings two probes measure on this chip (linear read, MFMA-only
loop), short runs of the other workloads (`per_config`), and the CPU oracle timed on a bounded sample of the same
workload on this machine's host cores.

Other modes (no step is timed):
    python bench.py --peaks                      only the two probes, one JSON line
    python bench.py --summarize-counters FETCH.csv WRITE.csv --config NAME
    python bench.py --summarize-trace KERNEL_STATS.csv --config NAME
        turn rocprofv3 CSVs of a run of this script into profiles/step_NAME_*.md and profiles/traffic.json
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")
NAMES = ("verify_attn", "lm_head", "accept", "kv_commit")
# GPU kernel that carries a call's bytes or flops, by call and weight layout (first name found in a profile wins)
KERNEL_OF_CALL = {
    ("verify_attn", True): ("verify_attn_rows_kernel", "verify_attn_kernel"),
    ("verify_attn", False): ("verify_attn_rows_kernel", "verify_attn_kernel"),
    ("lm_head", True): ("lm_head_mfma_kernel", "lm_head_packed_kernel"),
    ("lm_head", False): ("lm_head_big2_kernel", "lm_head_big_kernel", "lm_head_skinny_kernel", "lm_head_tiled_kernel"),
    ("accept", True): ("accept_row_stats_kernel",), ("accept", False): ("accept_row_stats_kernel",),
    ("kv_commit", True): ("kv_commit_kernel",), ("kv_commit", False): ("kv_commit_kernel",),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="hybrid", help="workload name in paper_2605_08151_amd.workloads.CONFIGS")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--no-peaks", action="store_true", help="skip the linear-read and MFMA-only probes")
    ap.add_argument("--peaks", action="store_true", help="run only the two probes and print their JSON line")
    ap.add_argument("--peaks-md", default="", metavar="PATH", help="with --peaks: also write the probes' summary (markdown) to PATH")
    ap.add_argument("--summarize-sq", metavar="COUNTER_CSV",
                    help="rocprofv3 --pmc counter_collection CSV of `bench.py --config NAME` with the SQ counters named in the "
                         "summary: writes profiles/step_NAME_sq_counters.md")
    ap.add_argument("--attn-chunk", type=int, default=0, help="override keys per kv split (0 = library heuristic)")
    ap.add_argument("--fused-stats", action="store_true",
                    help="the LM head also leaves per-block maxima (spec_lm_head_stats or spec_lm_head_packed_stats) and "
                         "greedy acceptance reads those instead of the logits (spec_accept_stats); same outputs")
    ap.add_argument("--summaries", choices=("auto", "on", "off"), default="auto",
                    help="block summaries from the large-tile LM head (spec_lm_head_packed_summary + spec_accept_summary) when the "
                         "batch has more than 160 rows: on, off, or auto = with --fused-stats")
    ap.add_argument("--lm-weights", choices=("auto", "packed", "rowmajor"), default="auto",
                    help="layout of the vocabulary matrix: packed (spec_lm_head_packed; re-laid once before the timed "
                         "region, as at model load) or rowmajor (spec_lm_head); auto = packed whenever the kernel takes "
                         "the shape (H a multiple of 256)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy 3 times (untimed): under rocprofv3 --pmc its FETCH_SIZE / "
                         "WRITE_SIZE readings calibrate the counters against a known byte count")
    ap.add_argument("--summarize-counters", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE counter_collection CSVs of `bench.py --config NAME "
                         "--copy-probe`: writes profiles/step_NAME_hbm_traffic.md and NAME's keys of profiles/traffic.json")
    ap.add_argument("--summarize-trace", metavar="KERNEL_STATS_CSV",
                    help="rocprofv3 --kernel-trace --stats kernel_stats CSV of `bench.py --config NAME`: writes "
                         "profiles/step_NAME_kernel_trace.md")
    ap.add_argument("--profile-cmd", default="", help="the command line the CSVs came from (quoted in the summary)")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------------------------
# algorithmic work per launch of each call
# ------------------------------------------------------------------------------------------------------------
def algorithmic(cfg, b):
    M, V, H = b["M"], cfg.V, cfg.H
    kv_tokens = int((b["ctx"] + b["gammas"] + 1).sum())
    n_stoch = int((b["temperature"] > 0).sum())
    return dict(
        kv_tokens=kv_tokens,
        attn_bytes=kv_tokens * cfg.Hkv * cfg.D * 2 * 2 + 2 * M * cfg.Hq * cfg.D * 2,   # 512 B per key per kv head + q, out
        lm_bytes=V * H * 2 + M * H * 2 + M * V * 4,                                      # W once + hidden + fp32 logits
        lm_flops=2.0 * M * H * V,
        accept_bytes=M * V * 4 + n_stoch * 2 * V * 4,                                    # every logits row once + 2 rows per sampled request
    )


def short_kernel_name(full: str) -> str:
    """'void specv::lm_head_packed_kernel<10, 1, ...>(...)' -> 'lm_head_packed_kernel'"""
    s = full.replace("void ", "").split("(")[0].split("<")[0]
    return s.split("::")[-1].strip()


def load_traffic(cfg_name, call, packed):
    """(HBM bytes per launch of the call's dominant kernel, that kernel's name) from profiles/traffic.json, or (None, None)."""
    if not os.path.exists(TRAFFIC_JSON):
        return None, None
    table = json.load(open(TRAFFIC_JSON))
    for k in KERNEL_OF_CALL[(call, packed)]:
        v = table.get(f"{cfg_name}:{k}")
        if v is not None:
            return float(v), k
    return None, None


# ------------------------------------------------------------------------------------------------------------
# the two probes
# ------------------------------------------------------------------------------------------------------------
def measure_peaks(torch, sv):
    """Linear device read (2 GiB, beyond the memory-side cache) and MFMA-only loop, HIP events on the launch stream."""
    new_event = lambda: torch.cuda.Event(enable_timing=True)
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    src = torch.empty(1 << 31, dtype=torch.uint8, device="cuda")
    src.view(torch.int32).random_(0, 1 << 30)
    reads = []
    for it in range(7):
        e0, e1 = new_event(), new_event()
        e0.record()
        sv.spec_probe_read(src, sink)
        e1.record()
        torch.cuda.synchronize()
        if it >= 2:
            reads.append(src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    out = {"hbm_linear_read_GBs": float(sorted(reads)[len(reads) // 2]), "hbm_linear_read_GBs_best": float(max(reads)),
           "hbm_probe": "spec_probe_read over 2 GiB, median of 5 launches"}
    # the attention reads 4 KB pages (16 keys x 128 x bf16) scattered over the pool: the same 2 GiB as pages
    n_pages = src.numel() // 4096
    orders = {"in_order": torch.arange(n_pages, dtype=torch.int32, device="cuda"),
              "random_order": torch.randperm(n_pages, generator=torch.Generator(device="cuda").manual_seed(1), device="cuda").to(torch.int32)}
    for label, pages in orders.items():
        rates = []
        for it in range(5):
            e0, e1 = new_event(), new_event()
            e0.record()
            sv.spec_probe_read_pages(src, pages, sink)
            e1.record()
            torch.cuda.synchronize()
            if it >= 2:
                rates.append(src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        out[f"hbm_4k_pages_{label}_GBs"] = float(sorted(rates)[len(rates) // 2])
    out["hbm_pages_probe"] = "spec_probe_read_pages over the same 2 GiB as 524288 pages of 4 KB, median of 3 launches"
    del src, orders
    for label, const in (("random", 0), ("constant", 1)):
        rates = []
        for it in range(5):
            e0, e1 = new_event(), new_event()
            e0.record()
            flops = sv.spec_probe_mfma(20000, const, sink)
            e1.record()
            torch.cuda.synchronize()
            if it >= 1:
                rates.append(flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        out[f"mfma_bf16_TFLOPs_{label}_operands"] = float(sorted(rates)[len(rates) // 2])
    out["mfma_probe"] = ("spec_probe_mfma: 8 waves per CU, 20000 x 16 independent v_mfma_f32_16x16x32_bf16 per wave, "
                         "median of 4 launches of ~5 ms")
    return out


# ------------------------------------------------------------------------------------------------------------
# one workload
# ------------------------------------------------------------------------------------------------------------
def measure(args, cfg_name, steps, warmup, extras):
    """Builds the workload, times `steps` steps after `warmup` instrumented ones.  `extras`: also the back-to-back
    timings and everything the CPU baseline needs (the headline workload); otherwise a short record."""
    import numpy as np
    import torch

    from paper_2605_08151_amd import binding as sv
    from paper_2605_08151_amd import workloads as wl
    from paper_2605_08151_amd.step import VerifyStep

    cfg = wl.CONFIGS[cfg_name]
    # ---- inputs (untimed) ------------------------------------------------------------------
    # K/V pools rotate so that no step finds its keys in the 256 MB memory-side cache: enough copies for more than
    # 1 GiB in total, or, for the small workloads, one fresh pool per step of the run
    n_warm = max(warmup, 2)                               # the breakdown below needs a few instrumented steps
    total = steps + n_warm
    gammas, ctx = wl.draw_lengths(cfg, wl._gen(cfg.seed, "cpu"))
    pages = int(((ctx + gammas + 1 + cfg.P - 1) // cfg.P).sum())
    pool_bytes = max(1, int(math.ceil(pages * cfg.pool_slack)) * cfg.Hkv * cfg.P * cfg.D * 2 * 2)
    kv_copies = max(2, min(-(-(1 << 30) // pool_bytes), total + 24))
    b = wl.make_batch(cfg, device="cuda", kv_copies=kv_copies)
    B, M, V, H = b["B"], b["M"], cfg.V, cfg.H
    step = VerifyStep(B, M, cfg.Hq, cfg.Hkv, cfg.D, H, V, b["gamma_max"], b["max_kv_len"])
    qo = b["qo_indptr"]
    packed = args.lm_weights == "packed" or (args.lm_weights == "auto" and H % 256 == 0)
    Wp = step.pack_weights(b["W"]) if packed else None      # load-time work, not part of a step
    logits = step.lm_head_packed(b["hidden"], Wp) if packed else step.lm_head(b["hidden"], b["W"])
    torch.cuda.synchronize()
    stochastic = bool((b["temperature"] > 0).any())
    tokens_g, _ = wl.draft_tokens_greedy(cfg, qo, logits.argmax(1).cpu())
    draft_probs, tokens = None, tokens_g
    if stochastic:
        draft_probs, tokens_s = wl.draft_probs_noisy(cfg, qo, logits)
        per_row_T = torch.repeat_interleave(b["temperature"].cpu(), (qo[1:] - qo[:-1]).cpu().long())
        tokens = torch.where(per_row_T > 0, tokens_s, tokens_g)
    tokens = tokens.cuda()
    seeds = b["seeds"] if stochastic else None

    # commit mutates the page table / lengths / free list: give every step its own pristine copy
    states = [(b["page_table"].clone(), b["seq_lens"].clone(), b["free_list"].clone(), b["free_count"].clone())
              for _ in range(total)]
    fused = args.fused_stats            # same outputs; greedy acceptance reads the LM head's block maxima instead of the logits
    # more than 160 rows on packed weights: the large-tile LM head can leave block summaries (maxima and exponential sums)
    # from which acceptance works without scanning the logits again; same outputs
    summaries = packed and args.summaries != "off" and step.sblocks > 0 and (args.summaries == "on" or fused)

    def run(k, events=None):
        """One step.  `events`: None, or five events recorded around the four calls (None entries are skipped)."""
        events = events or (None,) * 5
        pt, sl, fl, fc = states[k]
        kc, vc = b["k_caches"][k % kv_copies], b["v_caches"][k % kv_copies]
        if events[0]: events[0].record()
        step.attn(b["q"], kc, vc, pt, sl, qo, b["scale"], want_lse=False)
        if events[1]: events[1].record()
        if summaries:
            step.lm_head_packed_summary(b["hidden"], Wp, b["temperature"], qo)
        elif fused and packed:
            step.lm_head_packed_stats(b["hidden"], Wp)
        elif fused:
            step.lm_head_stats(b["hidden"], b["W"])
        elif packed:
            step.lm_head_packed(b["hidden"], Wp)
        else:
            step.lm_head(b["hidden"], b["W"])
        if events[2]: events[2].record()
        if summaries:
            step.accept_summary(tokens, draft_probs, b["temperature"], seeds, 0, qo)
        elif fused and packed:
            step.accept_packed_stats(tokens, draft_probs, b["temperature"], seeds, 0, qo)
        elif fused:
            step.accept_stats(tokens, draft_probs, b["temperature"], seeds, 0, qo)
        else:
            step.accept(tokens, draft_probs, b["temperature"], seeds, 0, qo)
        if events[3]: events[3].record()
        step.commit(pt, sl, qo, fl, fc, cfg.P)
        if events[4]: events[4].record()

    if args.copy_probe and extras:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # Warm-up: every call bracketed by events, which gives the per-call breakdown and names the dominant call.  An event
    # record costs a few microseconds of a step, so the timed region keeps only the two around that call.
    new_event = lambda: torch.cuda.Event(enable_timing=True)
    ev_warm = [[new_event() for _ in range(5)] for _ in range(n_warm)]
    for k in range(n_warm):
        run(k, ev_warm[k])
    torch.cuda.synchronize()
    def call_samples(evs, i):
        return np.array([e[i].elapsed_time(e[i + 1]) for e in evs])
    settled = ev_warm[len(ev_warm) // 2:]                 # the first warm-up steps carry one-off costs
    warm_ms = {n: float(call_samples(settled, i).mean()) if settled else 0.0 for i, n in enumerate(NAMES)}
    dom = max(range(4), key=lambda i: warm_ms[NAMES[i]])
    ev = [[new_event() if i in (dom, dom + 1) else None for i in range(5)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        run(n_warm + k, ev[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    emitted = int(step.stats.cpu()[1])
    assert int(step.status.cpu()) == 0, "a kernel flagged bad input"
    samples = {n: (call_samples(ev, i) if i == dom else call_samples(settled, i)) for i, n in enumerate(NAMES)}
    per_call_ms = {n: float(v.mean()) if len(v) else 0.0 for n, v in samples.items()}
    per_call_spread = {n: {"median": float(np.median(v)), "p10": float(np.percentile(v, 10)), "p90": float(np.percentile(v, 90))}
                       for n, v in samples.items()}
    del ev, ev_warm, settled                              # hundreds of live events slow later launches down now and then

    # ---- roofline of each call (algorithmic bytes / flops per launch) -----------------------
    alg = algorithmic(cfg, b)
    rl = {
        "verify_attn": dict(bound="hbm", achieved=alg["attn_bytes"] / per_call_ms["verify_attn"] / 1e6, peak=HBM_PEAK_GBS, unit="GB/s"),
        "lm_head_hbm": dict(bound="hbm", achieved=alg["lm_bytes"] / per_call_ms["lm_head"] / 1e6, peak=HBM_PEAK_GBS, unit="GB/s"),
        "lm_head_mfma": dict(bound="mfma", achieved=alg["lm_flops"] / per_call_ms["lm_head"] / 1e9, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s"),
        "accept": dict(bound="hbm", achieved=alg["accept_bytes"] / per_call_ms["accept"] / 1e6, peak=HBM_PEAK_GBS, unit="GB/s"),
    }
    for r in rl.values():
        r["frac"] = r["achieved"] / r["peak"]

    b2b_ms, rowmajor_lm_ms = {}, None
    if extras:
        # Calls back to back (20 launches between two events, outside the timed region): free of the events' own cost
        def back_to_back(fn, n=20):
            for i in range(3):
                fn(i)
            e0, e1 = new_event(), new_event()
            e0.record()
            for i in range(n):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n
        if packed:                                        # the same LM head on the row-major matrix (spec_lm_head)
            rowmajor_lm_ms = back_to_back(lambda i: step.lm_head(b["hidden"], b["W"]), n=10)
            step.lm_head_packed(b["hidden"], Wp)          # leave the logits as the step left them
            torch.cuda.synchronize()
        pt0, sl0 = b["page_table"], b["seq_lens"]        # the pristine table: no commit runs here
        b2b_ms = {
            "verify_attn": back_to_back(lambda i: step.attn(b["q"], b["k_caches"][i % kv_copies], b["v_caches"][i % kv_copies],
                                                            pt0, sl0, qo, b["scale"], want_lse=False)),
            "accept": back_to_back(lambda i: step.accept(tokens, draft_probs, b["temperature"], seeds, 0, qo)),
        }
        for n, nbytes in (("verify_attn", alg["attn_bytes"]), ("accept", alg["accept_bytes"])):
            rl[n]["back_to_back_ms"] = b2b_ms[n]
            rl[n]["back_to_back_frac"] = nbytes / b2b_ms[n] / 1e6 / HBM_PEAK_GBS

    dominant = NAMES[dom]
    # the LM head is priced against the roof that binds it at this M: weight streaming (HBM) when the
    # arithmetic intensity is under the ridge, MFMA otherwise
    lm_key = "lm_head_hbm" if alg["lm_flops"] / alg["lm_bytes"] < MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS else "lm_head_mfma"
    dom_key = {"lm_head": lm_key, "kv_commit": "accept"}.get(dominant, dominant)
    traffic, kernel = load_traffic(cfg.name, dominant, packed)
    roofline = dict(call=dominant, kernel=kernel, **{k: rl[dom_key][k] for k in ("bound", "achieved", "peak", "unit", "frac")},
                    traffic=traffic)

    rec = {
        "workload": f"{cfg.name}: B={B} gamma={sorted(set(b['gammas'].tolist()))} M={M} ctx={cfg.ctx} "
                    f"Hq={cfg.Hq} Hkv={cfg.Hkv} D={cfg.D} page={cfg.P} H={H} V={V} "
                    f"temperature={cfg.temperature} seed={cfg.seed}",
        "ms_per_step": ms_per_step, "steps": steps, "warmup": n_warm, "emitted_tokens_per_step": emitted,
        "value": emitted / (ms_per_step * 1e-3), "scored_positions_per_step": M, "kv_tokens": alg["kv_tokens"],
        "kv_pool_copies": kv_copies, "kv_pool_bytes": pool_bytes, "lm_weights": "packed" if packed else "rowmajor",
        "lm_head_ms_on_rowmajor_weights_back_to_back": rowmajor_lm_ms,
        "roofline": roofline, "per_call_ms": per_call_ms,
        "per_call_ms_source": {n: ("timed region" if i == dom else "instrumented warm-up steps") for i, n in enumerate(NAMES)},
        "per_call_ms_spread": per_call_spread, "per_call_roofline": rl,
    }
    ctxobj = dict(cfg=cfg, b=b, step=step, tokens=tokens, draft_probs=draft_probs, seeds=seeds, emitted=emitted) if extras else None
    return rec, ctxobj


def add_measured_fracs(rec, peaks):
    """fraction of what the probes reach on this chip, beside every fraction of the datasheet peak"""
    if not peaks:
        return
    ref = {"hbm": peaks["hbm_linear_read_GBs"], "mfma": peaks["mfma_bf16_TFLOPs_random_operands"] }
    for r in [rec["roofline"], *rec["per_call_roofline"].values()]:
        r["frac_of_measured_peak"] = r["achieved"] / ref[r["bound"]]


def main():
    args = parse()
    if args.summarize_counters:
        return summarize_counters(args)
    if args.summarize_trace:
        return summarize_trace(args)
    if args.summarize_sq:
        return summarize_sq(args)
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives are implemented); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2605_08151_amd import binding as sv
    from paper_2605_08151_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.peaks:
        rec = {"measured_peaks": measure_peaks(torch, sv), "datasheet": {"hbm_GBs": HBM_PEAK_GBS, "mfma_bf16_TFLOPs": MFMA_BF16_PEAK_TFLOPS}}
        if args.peaks_md:
            write_peaks_md(args.peaks_md, rec)
        print(json.dumps(rec))
        return
    if args.attn_chunk:
        sv.spec_set_tuning("attn_chunk", args.attn_chunk)

    rec, ctx = measure(args, args.config, args.steps, args.warmup, extras=True)
    peaks = None if args.no_peaks else measure_peaks(torch, sv)
    add_measured_fracs(rec, peaks)

    # ---- CPU oracle on a bounded sample of the same workload ----------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(ctx["cfg"], ctx["b"], ctx["step"], ctx["tokens"], ctx["draft_probs"], ctx["seeds"],
                           emitted_per_step=ctx["emitted"])
    del ctx
    torch.cuda.empty_cache()

    # ---- the other workloads, briefly (same protocol, fewer steps) ----------------------------------
    per_config = {}
    if not args.no_per_config:
        for name in wl.CONFIGS:
            if name == args.config:
                continue
            try:
                r, _ = measure(args, name, min(args.steps, 30), min(max(args.warmup, 2), 6), extras=False)
                add_measured_fracs(r, peaks)
                per_config[name] = {k: r[k] for k in ("workload", "ms_per_step", "value", "steps", "warmup", "emitted_tokens_per_step",
                                                      "roofline", "per_call_ms", "per_call_roofline", "kv_pool_copies")}
            except Exception as e:                        # the headline line must still be printed
                per_config[name] = {"error": f"{type(e).__name__}: {e}"}
            torch.cuda.empty_cache()

    out = {
        "metric": "verified tokens/sec per GPU", "value": rec["value"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": rec["warmup"], "ms_per_step": rec["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": rec["workload"], "lm_weights": rec["lm_weights"],
                   "lm_head_ms_on_rowmajor_weights_back_to_back": rec["lm_head_ms_on_rowmajor_weights_back_to_back"],
                   "emitted_tokens_per_step": rec["emitted_tokens_per_step"],
                   "scored_positions_per_step": rec["scored_positions_per_step"],
                   "scored_positions_per_s": rec["scored_positions_per_step"] / (rec["ms_per_step"] * 1e-3),
                   "kv_tokens": rec["kv_tokens"], "kv_pool_copies": rec["kv_pool_copies"], "kv_pool_bytes": rec["kv_pool_bytes"]},
        "roofline": rec["roofline"],
        "cpu_baseline": cpu,
        "measured_peaks": peaks,
        "per_call_ms": rec["per_call_ms"],
        "per_call_ms_source": rec["per_call_ms_source"],
        "per_call_ms_spread": rec["per_call_ms_spread"],
        "per_call_roofline": rec["per_call_roofline"],
        "per_config": per_config,
    }
    print(json.dumps(out))


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, b, step, tokens, draft_probs, seeds, emitted_per_step, budget_s=8.0):
    """Times the oracle as it stands on this machine's host cores.  Each stage first runs on a small probe, then on
    the largest slice of the real workload that the probe says fits ~budget_s seconds (the whole stage if it
    fits), and is extrapolated linearly to full size."""
    import numpy as np
    import oracle
    from paper_2605_08151_amd import workloads as wl

    oracle.build()
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or os.cpu_count()
    B, M, V = b["B"], b["M"], cfg.V
    qo = b["qo_indptr"].cpu().numpy()
    ctx, gam = b["ctx"].numpy().astype(np.int64), b["gammas"].numpy().astype(np.int64)
    kbits, vbits = wl.bf16_bits(b["k_cache"]), wl.bf16_bits(b["v_cache"])
    qbits = wl.bf16_bits(b["q"])
    pt = b["page_table"].cpu().numpy()
    work = (ctx + gam + 1) * (gam + 1)                      # key-row products per request

    def attn_on(n_seq):
        rows = int(qo[n_seq])
        t = time.perf_counter()
        oracle.verify_attn(qbits[:rows], kbits, vbits, pt[:n_seq].copy(), ctx[:n_seq].astype(np.int32),
                           qo[:n_seq + 1].copy(), b["scale"])
        return time.perf_counter() - t

    n_probe = min(B, 2)
    t_probe = attn_on(n_probe)
    per_work = t_probe / float(work[:n_probe].sum())
    n_seq = int(np.searchsorted(np.cumsum(work) * per_work, budget_s)) + 1
    n_seq = max(n_probe, min(B, n_seq))
    t_attn_sample = attn_on(n_seq) if n_seq > n_probe else t_probe
    t_attn = t_attn_sample * float(work.sum()) / float(work[:n_seq].sum())

    hbits = wl.bf16_bits(b["hidden"])
    def lm_on(v_s):
        t = time.perf_counter()
        oracle.lm_head(hbits, wl.bf16_bits(b["W"][:v_s]))
        return time.perf_counter() - t
    v_probe = min(V, 512)
    t_probe = lm_on(v_probe)
    v_s = max(v_probe, min(V, int(v_probe * budget_s / max(t_probe, 1e-6))))
    t_lm_sample = lm_on(v_s) if v_s > v_probe else t_probe
    t_lm = t_lm_sample * V / v_s

    gl = step.logits.cpu().numpy()
    dp = None if draft_probs is None else draft_probs.cpu().numpy()
    sd = None if seeds is None else seeds.cpu().numpy().view(np.uint64)
    t = time.perf_counter()
    ref = oracle.accept(gl, tokens.cpu().numpy(), dp, b["temperature"].cpu().numpy(), sd, 0, qo, b["gamma_max"])
    t_acc = time.perf_counter() - t
    ptc, sl = pt.copy(), ctx.astype(np.int32).copy()
    fl, fc = b["free_list"].cpu().numpy().copy(), b["free_count"].cpu().numpy().copy()
    t = time.perf_counter()
    oracle.kv_commit(ptc, sl, qo, ref["accept_len"], fl, fc, cfg.P)
    t_commit = time.perf_counter() - t
    total = t_attn + t_lm + t_acc + t_commit
    return {"value": emitted_per_step / total, "unit": "tokens/s", "cores": threads, "cpu_model": cpu_model(), "kind": "oracle",
            "sample": f"attention on the first {n_seq} of {B} requests ({t_attn_sample:.2f} s, scaled by key*row count), "
                      f"LM head on all {M} rows x the first {v_s} of {V} vocabulary rows ({t_lm_sample:.2f} s, scaled by V), "
                      f"acceptance and commit on the whole batch; stage seconds at full size: "
                      f"attn {t_attn:.2f}, lm_head {t_lm:.2f}, accept {t_acc:.3f}, commit {t_commit:.4f}"}


# ------------------------------------------------------------------------------------------------------------
# rocprofv3 CSVs -> profiles/*.md and profiles/traffic.json (host only, no GPU)
# ------------------------------------------------------------------------------------------------------------
def _algorithmic_by_kernel(cfg_name):
    """algorithmic MB per launch of the kernels that carry a call's traffic (host arithmetic on the drawn lengths)"""
    import torch  # noqa: F401  (the generators are torch's)
    from paper_2605_08151_amd import workloads as wl
    cfg = wl.CONFIGS[cfg_name]
    gammas, ctx = wl.draw_lengths(cfg, wl._gen(cfg.seed, "cpu"))
    temp = [cfg.temperature[1]] * cfg.B if cfg.temperature[0] == "const" else [cfg.temperature[1 + (i & 1)] for i in range(cfg.B)]
    b = dict(M=int((gammas + 1).sum()), ctx=ctx, gammas=gammas, temperature=torch.tensor(temp))
    alg = algorithmic(cfg, b)
    n_stoch = int((b["temperature"] > 0).sum())
    return {"verify_attn_kernel": alg["attn_bytes"] / 1e6, "verify_attn_rows_kernel": alg["attn_bytes"] / 1e6,
            "lm_head_packed_kernel": alg["lm_bytes"] / 1e6,
            "lm_head_mfma_kernel": alg["lm_bytes"] / 1e6, "lm_head_big2_kernel": alg["lm_bytes"] / 1e6,
            "lm_head_skinny_kernel": alg["lm_bytes"] / 1e6,
            "accept_row_stats_kernel": b["M"] * cfg.V * 4 / 1e6,
            "accept_residual_sums_kernel": n_stoch * 2 * cfg.V * 4 / 1e6}


def summarize_counters(args):
    fetch_csv, write_csv = args.summarize_counters
    name = args.config

    def load(path, ctr):
        agg = collections.defaultdict(list)
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] == ctr:
                agg[r["Kernel_Name"]].append(float(r["Counter_Value"]))
        return agg
    F, W = load(fetch_csv, "FETCH_SIZE"), load(write_csv, "WRITE_SIZE")
    # calibration: the 1 GiB device copy of --copy-probe is the non-library kernel with the largest reading
    probe = lambda agg: max((max(v) for k, v in agg.items() if "specv::" not in k), default=0.0)
    pf, pw = probe(F), probe(W)
    assert pf > 0 and pw > 0, "no copy probe in the CSVs: run bench.py with --copy-probe"
    sf, sw = 1048576.0 / pf, 1048576.0 / pw
    alg = _algorithmic_by_kernel(name)
    rows, table = [], {}
    for k in sorted(F):
        if "specv::" not in k:
            continue
        short = short_kernel_name(k)
        f = sum(F[k]) / len(F[k])
        w = sum(W[k]) / len(W[k]) if k in W else 0.0
        fm, wm = f * sf * 1024 / 1e6, w * sw * 1024 / 1e6
        rows.append((k.replace("void ", "").split("(")[0], len(F[k]), f, w, fm, wm, alg.get(short)))
        if "probe" in short or "pack_kernel" in short:   # not part of a step
            continue
        assert f"{name}:{short}" not in table, f"two kernels named {short}: key them apart before summing anything"
        table[f"{name}:{short}"] = (fm + wm) * 1e6
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    cmd = args.profile_cmd or f"python3 bench.py --config {name} --steps 5 --warmup 2 --no-cpu-baseline --no-per-config --no-peaks --copy-probe"
    md = os.path.join(ROOT, "profiles", f"step_{name}_hbm_traffic.md")
    with open(md, "w") as o:
        o.write(f"# Verification step, workload '{name}': HBM traffic per launch from rocprofv3 counters\n\n")
        o.write("Commands (on the MI355X box, from the repository root, one counter per run):\n\n")
        o.write("    cd /tmp && export TMPDIR=/tmp && cd <repository root>; OUT=<a scratch directory>\n")
        for c in ("FETCH_SIZE", "WRITE_SIZE"):
            o.write(f"    rocprofv3 --pmc {c} --output-format csv -d $OUT/pmc_{c} -o {name} -- {cmd}\n")
        o.write(f"    python3 bench.py --config {name} --summarize-counters $OUT/pmc_FETCH_SIZE/{name}_counter_collection.csv "
                f"$OUT/pmc_WRITE_SIZE/{name}_counter_collection.csv\n")
        o.write(f"\nCalibration: the plain 1 GiB device copy of `--copy-probe` (1048576 KiB read, 1048576 KiB written) reads "
                f"FETCH_SIZE = {pf:.0f} and WRITE_SIZE = {pw:.0f}, so the counters are scaled by {sf:.3f} (fetch) and {sw:.3f} (write) to KiB.\n\n")
        o.write("| kernel | launches | FETCH_SIZE avg | WRITE_SIZE avg | fetched MB | written MB | algorithmic MB | traffic / algorithmic |\n|---|---|---|---|---|---|---|---|\n")
        for k, n, f, w, fm, wm, a in rows:
            ratio = f"{(fm + wm) / a:.3f}" if a else "n/a"
            o.write(f"| {k} | {n} | {f:.1f} | {w:.1f} | {fm:.1f} | {wm:.1f} | {f'{a:.1f}' if a else 'n/a'} | {ratio} |\n")
        o.write("\nfetched/written MB = counter x scale x 1024 / 1e6, per launch (average over the launches of the run).  "
                "`profiles/traffic.json` holds fetched + written bytes per launch under the key `workload:kernel`, one kernel per key.\n")
    old = json.load(open(TRAFFIC_JSON)) if os.path.exists(TRAFFIC_JSON) else {}
    old = {k: v for k, v in old.items() if not k.startswith(name + ":")}
    old.update(table)
    old["_note"] = ("HBM bytes per launch of ONE kernel (FETCH_SIZE + WRITE_SIZE of rocprofv3 --pmc, calibrated against a 1 GiB copy), "
                    "key = workload:kernel; written by `bench.py --summarize-counters`; tables in step_<workload>_hbm_traffic.md")
    json.dump(dict(sorted(old.items())), open(TRAFFIC_JSON, "w"), indent=1)
    print(open(md).read())


SQ_COUNTERS = ("SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_WAVE_CYCLES SQ_WAIT_ANY SQ_WAIT_INST_ANY "
               "SQ_ACTIVE_INST_VALU SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE GRBM_GUI_ACTIVE")


def summarize_sq(args):
    name = args.config
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(args.summarize_sq)):
        if "specv::" in r["Kernel_Name"]:
            k = r["Kernel_Name"].split("(")[0].replace("void ", "")
            agg[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
            if r["Counter_Name"] == "GRBM_GUI_ACTIVE":
                agg[k]["_us"].append((float(r["End_Timestamp"]) - float(r["Start_Timestamp"])) / 1e3)
    cmd = args.profile_cmd or f"python3 bench.py --config {name} --steps 5 --warmup 2 --no-cpu-baseline --no-per-config --no-peaks"
    md = os.path.join(ROOT, "profiles", f"step_{name}_sq_counters.md")
    rows = []
    for k, v in agg.items():
        a = {c: sum(x) / len(x) for c, x in v.items()}
        if a.get("_us", 0.0) < 4.0 or "probe" in k or "pack_kernel" in k:
            continue
        cyc, wc = a["GRBM_GUI_ACTIVE"] / 8, max(a["SQ_WAVE_CYCLES"], 1.0)
        rows.append((a["_us"], f"| {k} | {len(v['_us'])} | {a['_us']:.1f} | {cyc / a['_us'] / 1e3:.2f} | "
                     f"{a['SQ_VALU_MFMA_BUSY_CYCLES'] / (cyc * 1024) * 100:.1f} % | {a['SQ_INSTS_VALU_MFMA_MOPS_BF16'] * 512:.3e} | "
                     f"{a['SQ_ACTIVE_INST_VALU'] / wc:.2f} | {a['SQ_WAIT_INST_ANY'] / wc:.2f} | {a['SQ_WAIT_ANY'] / wc:.2f} | "
                     f"{a['SQ_LDS_IDX_ACTIVE']:.3e} | {a['SQ_LDS_BANK_CONFLICT'] / max(a['SQ_LDS_IDX_ACTIVE'], 1) * 100:.1f} % |\n"))
    with open(md, "w") as o:
        o.write(f"# Verification step, workload '{name}': wave, MFMA and LDS counters (rocprofv3 --pmc)\n\n")
        o.write("Commands (on the MI355X box, from the repository root):\n\n")
        o.write("    cd /tmp && export TMPDIR=/tmp && cd <repository root>; OUT=<a scratch directory>\n")
        o.write(f"    rocprofv3 --pmc {SQ_COUNTERS} --output-format csv -d $OUT/pmc_sq -o {name} -- {cmd}\n")
        o.write(f"    python3 bench.py --config {name} --summarize-sq $OUT/pmc_sq/{name}_counter_collection.csv\n\n")
        o.write("Reading: launches of 4 us or more, averages per launch.  GRBM_GUI_ACTIVE is summed over the 8 XCDs (/8 = cycles of the "
                "launch, 'clock' = cycles / us; it also counts the few microseconds around a dispatch, so the clock of a short kernel reads "
                "high).  SQ_VALU_MFMA_BUSY_CYCLES is summed over the 1024 SIMDs; one MFMA MOP is 512 flop.  VALU / wait columns are "
                "fractions of SQ_WAVE_CYCLES (cycles summed over resident waves): 'wait inst' = stalled at a wait-count instruction, "
                "'wait any' = waiting for anything (barriers included).\n\n")
        o.write("| kernel | launches | us | clock GHz | MFMA busy (of 1024 SIMDs) | MFMA flop | VALU active | wait inst | wait any | "
                "LDS active cycles (sum) | of which bank conflicts |\n|---|---|---|---|---|---|---|---|---|---|---|\n")
        for _, line in sorted(rows, reverse=True):
            o.write(line)
    print(open(md).read())


def write_peaks_md(path, rec):
    p = rec["measured_peaks"]
    with open(path, "w") as o:
        o.write("# Measured ceilings of the MI355X box (probes of the library, HIP events on the launch stream)\n\n")
        o.write("Command (on the MI355X box, from the repository root; OUT = a scratch directory):\n\n    python3 bench.py --peaks --peaks-md $OUT/peaks.md\n\n")
        o.write("| probe | measured | datasheet | ratio |\n|---|---|---|---|\n")
        hb, mf = rec["datasheet"]["hbm_GBs"], rec["datasheet"]["mfma_bf16_TFLOPs"]
        o.write(f"| linear read of 2 GiB (`spec_probe_read`, 16-byte loads, 4 KB per workgroup step), median | {p['hbm_linear_read_GBs']:.0f} GB/s | {hb:.0f} GB/s | {p['hbm_linear_read_GBs'] / hb:.3f} |\n")
        o.write(f"| the same, best launch | {p['hbm_linear_read_GBs_best']:.0f} GB/s | {hb:.0f} GB/s | {p['hbm_linear_read_GBs_best'] / hb:.3f} |\n")
        o.write(f"| the same 2 GiB as 4 KB pages through an index list, in order (`spec_probe_read_pages`) | {p['hbm_4k_pages_in_order_GBs']:.0f} GB/s | {hb:.0f} GB/s | {p['hbm_4k_pages_in_order_GBs'] / hb:.3f} |\n")
        o.write(f"| 4 KB pages in a random permutation (what a paged K/V pool looks like) | {p['hbm_4k_pages_random_order_GBs']:.0f} GB/s | {hb:.0f} GB/s | {p['hbm_4k_pages_random_order_GBs'] / hb:.3f} |\n")
        o.write(f"| MFMA only, v_mfma_f32_16x16x32_bf16, random bf16 operands (`spec_probe_mfma`) | {p['mfma_bf16_TFLOPs_random_operands']:.0f} TFLOP/s | {mf:.0f} TFLOP/s | {p['mfma_bf16_TFLOPs_random_operands'] / mf:.3f} |\n")
        o.write(f"| MFMA only, constant operands | {p['mfma_bf16_TFLOPs_constant_operands']:.0f} TFLOP/s | {mf:.0f} TFLOP/s | {p['mfma_bf16_TFLOPs_constant_operands'] / mf:.3f} |\n")
        o.write(f"\n{p['hbm_probe']}; {p['hbm_pages_probe']}; {p['mfma_probe']}.\n")
        o.write("\nThe MFMA rate depends on the operand data (toggling costs power, and the clock follows): the random-operand figure "
                "is the ceiling a GEMM on real data can be held against.  `bench.py` prints `frac_of_measured_peak` beside every "
                "datasheet `frac`: HBM-bound calls against the linear read, the LM head against the random-operand MFMA rate.\n")


def summarize_trace(args):
    name = args.config
    rows = [r for r in csv.DictReader(open(args.summarize_trace)) if "specv::" in r["Name"]]
    rows.sort(key=lambda r: -float(r["TotalDurationNs"]))
    cmd = args.profile_cmd or f"python3 bench.py --config {name} --steps 30 --warmup 5 --no-cpu-baseline --no-per-config"
    md = os.path.join(ROOT, "profiles", f"step_{name}_kernel_trace.md")
    with open(md, "w") as o:
        o.write(f"# Verification step, workload '{name}': rocprofv3 kernel trace\n\n")
        o.write("Command (on the MI355X box, from the repository root):\n\n")
        o.write(f"    OUT=<a scratch directory>; cd /tmp && export TMPDIR=/tmp && cd <repository root> && rocprofv3 --kernel-trace --stats --output-format csv "
                f"-d $OUT/prof -o {name} -- {cmd}\n")
        o.write(f"    python3 bench.py --config {name} --summarize-trace $OUT/prof/{name}_kernel_stats.csv\n\n")
        o.write("Kernel-trace statistics of the library's kernels (durations in microseconds):\n\n")
        o.write("| kernel | calls | avg us | min us | max us | stddev us |\n|---|---|---|---|---|---|\n")
        for r in rows:
            k = r["Name"].replace("void ", "").split("(")[0]
            o.write(f"| {k} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.2f} | {float(r['MinNs']) / 1e3:.2f} | "
                    f"{float(r['MaxNs']) / 1e3:.2f} | {float(r['StdDev']) / 1e3:.2f} |\n")
    print(open(md).read())


if __name__ == "__main__":
    main()
