#!/usr/bin/env python3
"""Benchmark of the verification step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config mid]

A step is one pass of the whole hot path over one synthetic batch, inputs resident in HBM:
spec_verify_attn -> spec_lm_head -> spec_accept -> spec_kv_commit.  Prints ONE JSON line: verified
tokens/s (sum of accepted drafts + bonus tokens per wall-clock second), the roofline figures of the
dominant kernel measured with HIP events on the launch stream, per-call timings, and the CPU oracle
timed on a bounded sample of the same workload on this machine's host cores.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="mid", help="workload name in paper_2605_08151_amd.workloads.CONFIGS")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--attn-chunk", type=int, default=0, help="override keys per kv split (0 = library heuristic)")
    ap.add_argument("--fused-stats", action="store_true",
                    help="the LM head also leaves per-block maxima (spec_lm_head_stats or spec_lm_head_packed_stats) and "
                         "greedy acceptance reads those instead of the logits (spec_accept_stats); same outputs")
    ap.add_argument("--lm-weights", choices=("auto", "packed", "rowmajor"), default="auto",
                    help="layout of the vocabulary matrix: packed (spec_lm_head_packed; re-laid once before the timed "
                         "region, as at model load) or rowmajor (spec_lm_head); auto = packed whenever the kernel takes "
                         "the shape (H a multiple of 256)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy 3 times (untimed): under rocprofv3 --pmc its FETCH_SIZE / "
                         "WRITE_SIZE readings calibrate the counters against a known byte count")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives are implemented); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2605_08151_amd import binding as sv
    from paper_2605_08151_amd import workloads as wl
    from paper_2605_08151_amd.step import VerifyStep

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = wl.CONFIGS[args.config]
    if args.attn_chunk:
        sv.spec_set_tuning("attn_chunk", args.attn_chunk)

    # ---- inputs (untimed) ------------------------------------------------------------------
    kv_copies = 2
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
    n_warm = max(args.warmup, 2)                          # the breakdown below needs a few instrumented steps
    total = args.steps + n_warm
    states = [(b["page_table"].clone(), b["seq_lens"].clone(), b["free_list"].clone(), b["free_count"].clone())
              for _ in range(total)]

    names = ("verify_attn", "lm_head", "accept", "kv_commit")
    fused = args.fused_stats            # same outputs; greedy acceptance reads the LM head's block maxima instead of the logits

    def run(k, events=None):
        """One step.  `events`: None, or five events recorded around the four calls (None entries are skipped)."""
        events = events or (None,) * 5
        pt, sl, fl, fc = states[k]
        kc, vc = b["k_caches"][k % kv_copies], b["v_caches"][k % kv_copies]
        if events[0]: events[0].record()
        step.attn(b["q"], kc, vc, pt, sl, qo, b["scale"], want_lse=False)
        if events[1]: events[1].record()
        if fused and packed:
            step.lm_head_packed_stats(b["hidden"], Wp)
        elif fused:
            step.lm_head_stats(b["hidden"], b["W"])
        elif packed:
            step.lm_head_packed(b["hidden"], Wp)
        else:
            step.lm_head(b["hidden"], b["W"])
        if events[2]: events[2].record()
        if fused and packed:
            step.accept_packed_stats(tokens, draft_probs, b["temperature"], seeds, 0, qo)
        elif fused:
            step.accept_stats(tokens, draft_probs, b["temperature"], seeds, 0, qo)
        else:
            step.accept(tokens, draft_probs, b["temperature"], seeds, 0, qo)
        if events[3]: events[3].record()
        step.commit(pt, sl, qo, fl, fc, cfg.P)
        if events[4]: events[4].record()

    if args.copy_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # Warm-up: every call bracketed by events, which gives the per-call breakdown and names the dominant call.  An event
    # record costs a few microseconds of a 0.4 ms step, so the timed region keeps only the two around that call.
    new_event = lambda: torch.cuda.Event(enable_timing=True)
    ev_warm = [[new_event() for _ in range(5)] for _ in range(n_warm)]
    for k in range(n_warm):
        run(k, ev_warm[k])
    torch.cuda.synchronize()
    def call_samples(evs, i):
        return np.array([e[i].elapsed_time(e[i + 1]) for e in evs])
    settled = ev_warm[len(ev_warm) // 2:]                 # the first warm-up steps carry one-off costs
    warm_ms = {n: float(call_samples(settled, i).mean()) if settled else 0.0 for i, n in enumerate(names)}
    dom = max(range(4), key=lambda i: warm_ms[names[i]])
    ev = [[new_event() if i in (dom, dom + 1) else None for i in range(5)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        run(n_warm + k, ev[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    emitted = int(step.stats.cpu()[1])
    assert int(step.status.cpu()) == 0, "a kernel flagged bad input"
    samples = {n: (call_samples(ev, i) if i == dom else call_samples(settled, i)) for i, n in enumerate(names)}
    per_call_ms = {n: float(v.mean()) if len(v) else 0.0 for n, v in samples.items()}
    per_call_spread = {n: {"median": float(np.median(v)), "p10": float(np.percentile(v, 10)), "p90": float(np.percentile(v, 90))}
                       for n, v in samples.items()}

    del ev, ev_warm, settled                              # hundreds of live events slow later launches down now and then

    # Calls back to back (20 launches between two events, outside the timed region)
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
    # the same LM head on the row-major matrix (spec_lm_head), for comparison with the packed call
    rowmajor_lm_ms = None
    if packed:
        rowmajor_lm_ms = back_to_back(lambda i: step.lm_head(b["hidden"], b["W"]))
        step.lm_head_packed(b["hidden"], Wp)              # leave the logits as the step left them
        torch.cuda.synchronize()
    # attention (K/V pools rotating) and acceptance: their in-step figures above carry the events' own few microseconds,
    # which is several per cent of these two calls
    pt0, sl0 = b["page_table"], b["seq_lens"]            # the pristine table: no commit runs here
    b2b_ms = {
        "verify_attn": back_to_back(lambda i: step.attn(b["q"], b["k_caches"][i % kv_copies], b["v_caches"][i % kv_copies],
                                                        pt0, sl0, qo, b["scale"], want_lse=False)),
        "accept": back_to_back(lambda i: step.accept(tokens, draft_probs, b["temperature"], seeds, 0, qo)),
    }

    # ---- roofline of each call (algorithmic bytes / flops per launch) -----------------------
    kv_tokens = int((b["ctx"] + b["gammas"] + 1).sum())
    attn_bytes = kv_tokens * cfg.Hkv * cfg.D * 2 * 2 + 2 * M * cfg.Hq * cfg.D * 2
    lm_bytes = V * H * 2 + M * H * 2 + M * V * 4
    lm_flops = 2.0 * M * H * V
    n_stoch = int((b["temperature"] > 0).sum())
    accept_bytes = M * V * 4 + n_stoch * 2 * V * 4
    rl = {
        "verify_attn": dict(bound="hbm", achieved=attn_bytes / per_call_ms["verify_attn"] / 1e6, peak=HBM_PEAK_GBS, unit="GB/s"),
        "lm_head_hbm": dict(bound="hbm", achieved=lm_bytes / per_call_ms["lm_head"] / 1e6, peak=HBM_PEAK_GBS, unit="GB/s"),
        "lm_head_mfma": dict(bound="mfma", achieved=lm_flops / per_call_ms["lm_head"] / 1e9, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s"),
        "accept": dict(bound="hbm", achieved=accept_bytes / per_call_ms["accept"] / 1e6, peak=HBM_PEAK_GBS, unit="GB/s"),
    }
    for r in rl.values():
        r["frac"] = r["achieved"] / r["peak"]
    for n, nbytes in (("verify_attn", attn_bytes), ("accept", accept_bytes)):
        rl[n]["back_to_back_ms"] = b2b_ms[n]
        rl[n]["back_to_back_frac"] = nbytes / b2b_ms[n] / 1e6 / HBM_PEAK_GBS
    dominant = names[dom]
    # the LM head is priced against the roof that binds it at this M: weight streaming (HBM) when the
    # arithmetic intensity is under the ridge, MFMA otherwise
    lm_key = "lm_head_hbm" if lm_flops / lm_bytes < MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS else "lm_head_mfma"
    dom_key = {"lm_head": lm_key, "kv_commit": "accept"}.get(dominant, dominant)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(f"{cfg.name}:{dominant}")
    roofline = dict(kernel=dominant, **rl[dom_key], traffic=traffic)

    # ---- CPU oracle on a bounded sample of the same workload ----------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, b, step, tokens, draft_probs, seeds, emitted_per_step=emitted)

    out = {
        "metric": "verified tokens/sec per GPU", "value": emitted / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": n_warm, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={B} gamma={sorted(set(b['gammas'].tolist()))} M={M} ctx={cfg.ctx} "
                               f"Hq={cfg.Hq} Hkv={cfg.Hkv} D={cfg.D} page={cfg.P} H={H} V={V} "
                               f"temperature={cfg.temperature} seed={cfg.seed}",
                   "lm_weights": "packed" if packed else "rowmajor",
                   "lm_head_ms_on_rowmajor_weights_back_to_back": rowmajor_lm_ms,
                   "emitted_tokens_per_step": emitted, "scored_positions_per_step": M,
                   "scored_positions_per_s": M / (ms_per_step * 1e-3), "kv_tokens": kv_tokens},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "per_call_ms": per_call_ms,
        "per_call_ms_source": {n: ("timed region" if i == dom else "instrumented warm-up steps") for i, n in enumerate(names)},
        "per_call_ms_spread": per_call_spread,
        "per_call_roofline": rl,
    }
    print(json.dumps(out))


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
    v_probe = min(V, 2048)
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
    return {"value": emitted_per_step / total, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"attention on the first {n_seq} of {B} requests ({t_attn_sample:.2f} s, scaled by key*row count), "
                      f"LM head on all {M} rows x the first {v_s} of {V} vocabulary rows ({t_lm_sample:.2f} s, scaled by V), "
                      f"acceptance and commit on the whole batch; stage seconds at full size: "
                      f"attn {t_attn:.2f}, lm_head {t_lm:.2f}, accept {t_acc:.3f}, commit {t_commit:.4f}"}


if __name__ == "__main__":
    main()
