"""Benchmark of the PillarAttn hot path on one MI355X.

One "step" is one pass of the whole path over the batch: verification
attention with the score statistic, Top-K selection, one sparse draft step
(paper Section 4.1).  Inputs are synthetic and already resident in HBM when
the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps 50] [--warmup 10] [--config 3]
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

HBM_PEAK_GBPS = 8000.0
METRIC = "verify+draft attention µs/step and achieved HBM GB/s (% of peak) at batch 128"


def cpu_baseline(w, target_s: float = 12.0) -> dict:
    """Time the fp64 oracle, as it stands, on the leading requests of the SAME
    workload: whole requests are added four at a time until about `target_s`
    seconds of work are done (or the batch is exhausted); the time is scaled
    to the whole batch by context-token count."""
    import numpy as np
    import oracle
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        blas_threads = 1
    total_tokens = int(w.seq_lens.sum())
    done, wall, cpu = 0, 0.0, 0.0
    while done < w.B and wall < target_s:
        req = list(range(done, min(w.B, done + 4)))
        t0, c0 = time.perf_counter(), time.process_time()
        _, _, scores = oracle.verify_attn(w, requests=req)
        idx = np.full((w.B, w.Hkv, int(w.budgets.max())), -1, dtype=np.int32)
        counts = np.zeros(w.B, dtype=np.int32)
        idx[req], counts[req] = oracle.select_topk(scores[req], w.seq_lens[req], w.budgets[req],
                                                   max_budget=int(w.budgets.max()))
        oracle.sparse_decode(w, idx, counts, requests=req)
        wall += time.perf_counter() - t0
        cpu += time.process_time() - c0
        done = req[-1] + 1
    tok = int(w.seq_lens[:done].sum())
    scaled_us = wall * (total_tokens / tok) * 1e6
    return {"value": round(scaled_us, 1), "unit": "µs/step", "cores": max(1, round(cpu / max(wall, 1e-9))),
            "kind": "oracle",
            "sample": f"fp64 numpy oracle, verify + top-K + one draft step on the first {done} of {w.B} requests "
                      f"({tok} of {total_tokens} context tokens) of the same workload: {wall:.2f} s wall, scaled by "
                      f"token count; cores = CPU time / wall time; host has {os.cpu_count()} cpus, BLAS threads "
                      f"{blas_threads}",
            "sample_seconds": round(wall, 3)}


def measured_ceilings(pa, torch, dev) -> dict:
    """HBM read rates of THIS box with a plain read kernel (pillar_bench_read): a sequential stream over 2 GiB and
    the same bytes as 4 KiB chunks in random order (the access pattern of 16-token pages of one KV head)."""
    nbytes = 2 << 30
    buf = torch.ones(nbytes // 4, dtype=torch.int32, device=dev)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    n = nbytes // 4096
    order = torch.randperm(n, device=dev, generator=torch.Generator(device=dev).manual_seed(1)).to(torch.int32)
    res = {}
    for name, o in (("stream_read", None), ("random_4KiB_chunks", order)):
        best = 0.0
        for blocks in (1024, 2048, 4096):
            pa.pillar_bench_read(buf, n, 4096, o, blocks, sink)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                pa.pillar_bench_read(buf, n, 4096, o, blocks, sink)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, 5 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        res[name + "_GBps"] = round(best, 1)
    del buf, order
    return res


def recorded_traffic(config: int):
    """HBM bytes per step of the verification stage as rocprofv3's FETCH_SIZE / WRITE_SIZE counters gave
    them (scaled by a copy kernel of known size) for this workload: a recorded figure, read from the
    committed summary of those runs; None when there is none for the workload."""
    path = os.path.join(ROOT, "profiles", f"bench_config{config}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("verify_stage_traffic_bytes:"):
                return int(line.split(":")[1])
    except OSError:
        pass
    return None


def mixed_mode(args, w, run, gen, pa, torch) -> dict:
    """A unified batch of paper Section 4.2 on the same workload: every (k+1)-th request is in its verification
    phase, the others draft on the lists of their last verification.  Times pillar_mixed_step (one grid for both
    phases) against the same work as two calls on one stream and as two calls on two streams."""
    import numpy as np
    dev = run.dev
    ver = [b for b in range(w.B) if b % w.n_q == 0]
    dra = [b for b in range(w.B) if b % w.n_q != 0]
    v_ids = torch.tensor(ver, dtype=torch.int32, device=dev)
    d_ids = torch.tensor(dra, dtype=torch.int32, device=dev)
    run.verify_select()                                   # every request owns a list before the timed steps
    torch.cuda.synchronize()
    kv, k = run.dw.kv, w.spec_k

    def call(v, d, stream=None):
        pa.pillar_mixed_step(kv, v, d, run.dw.q, k, run.out, run.lse, run.scores, run.dw.budgets, run.max_budget, run.indices,
                             run.counts, run.dw.q_draft, run.d_out, run.d_lse, run.workspace, stream=stream)

    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()

    def fused():
        call(v_ids, d_ids)

    def sequential():
        call(v_ids, None)
        call(None, d_ids)

    def two_streams():
        side.wait_stream(main)
        call(v_ids, None)
        with torch.cuda.stream(side):
            call(None, d_ids, stream=side)
        main.wait_stream(side)

    def time_us(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        per = []
        for _ in range(args.steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main)
            fn()
            e1.record(main)
            per.append((e0, e1))
        torch.cuda.synchronize()
        t = sorted(a.elapsed_time(b) * 1e3 for a, b in per)
        return t[len(t) // 2], sum(t) / len(t)

    res = {}
    for name, fn in (("fused", fused), ("sequential", sequential), ("two_streams", two_streams)):
        med, mean = time_us(fn)
        res[name] = {"median_us": round(med, 2), "mean_us": round(mean, 2)}
    pa.pillar_profile_reset()
    pa.pillar_profile_enable(True)
    for _ in range(args.steps):
        fused()
    torch.cuda.synchronize()
    pa.pillar_profile_enable(False)
    prof = pa.pillar_profile_read()
    kern = {k_: {"launches": n, "avg_us": round(ms * 1e3 / max(n, 1), 2)} for k_, (n, ms) in prof.items()}
    tok_v = int(w.seq_lens[ver].astype(np.int64).sum())
    e = w.kv_elem_bytes()
    vb = tok_v * w.Hkv * (2 * w.D * e + 4) + 2 * len(ver) * w.n_q * w.Hq * w.D * w.q_elem_bytes()
    rows_d = int(np.minimum(w.budgets[dra], w.seq_lens[dra]).astype(np.int64).sum()) * w.Hkv
    db = rows_d * (2 * w.D * e + 4) + 2 * len(dra) * w.Hq * w.D * w.q_elem_bytes()
    us = res["fused"]["median_us"]
    gbps = (vb + db) / (us * 1e-6) / 1e9
    return {
        "metric": METRIC, "value": us, "unit": "µs/step", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us * 1e-3, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.kv_dtype == "bf16" else w.kv_dtype, "data": "synthetic",
        "config": {"workload": f"config {args.config}, unified batch: {len(ver)} of {w.B} requests verify (every {w.n_q}th), "
                               f"{len(dra)} draft: {gen.CONFIGS[args.config]}",
                   "calls": "pillar_mixed_step", "batch": w.B, "verifying": len(ver), "drafting": len(dra)},
        "mixed": {**res, "fused_vs_sequential": round(res["sequential"]["median_us"] / us, 3),
                  "fused_vs_two_streams": round(res["two_streams"]["median_us"] / us, 3),
                  "note": "per-step HIP-event times on the launch stream, median of the timed steps; sequential = "
                          "pillar_mixed_step with only the verifying list, then with only the drafting list"},
        "algorithmic_bytes": {"verify": vb, "draft": db},
        "kernels": kern,
        "roofline": {"bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                     "kernel": "whole unified step (all kernels of pillar_mixed_step)", "avg_us": us,
                     "algorithmic_bytes": vb + db},
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--batch", type=int, default=None, help="truncate the batch (debugging only; marks the run)")
    ap.add_argument("--three-calls", action="store_true",
                    help="verify, Top-K and draft as three calls (the statistic goes through HBM between the first two) "
                         "instead of pillar_verify_select + pillar_sparse_decode")
    ap.add_argument("--index-source", choices=["pillar", "window"], default="pillar",
                    help="window: the sliding-window draft the paper compares against -- verification without the "
                         "statistic, a static list of 4 sinks + the most recent tokens with the same budgets, draft")
    ap.add_argument("--mixed", action="store_true",
                    help="a unified draft / verify batch (paper Section 4.2): every (k+1)-th request verifies, the others "
                         "draft; pillar_mixed_step against the same work as two calls and on two streams")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB -> 1 GiB float copy kernel (for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE readings; not timed, not part of any reported figure)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU only (the path shards by request or KV head with no "
              "exchange, so a second GPU would only run a second copy). Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import gen
    import paper_2512_01278_amd as pa
    from paper_2512_01278_amd.runner import GpuRun

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    t_gen = time.perf_counter()
    w = gen.make_workload(args.config, batch=args.batch)
    print(f"[bench] generated {w.name}: B={w.B} tokens={int(w.seq_lens.sum())} in {time.perf_counter()-t_gen:.1f}s",
          file=sys.stderr, flush=True)
    run = GpuRun(w)
    torch.cuda.synchronize()
    if args.mixed:
        print(json.dumps(mixed_mode(args, w, run, gen, pa, torch), ensure_ascii=False))
        return 0
    stream = torch.cuda.current_stream()

    def step():
        if args.index_source == "window":
            run.verify(with_scores=False)
            pa.pillar_window_indices(run.dw.kv.seq_lens, run.dw.budgets, w.Hkv, 4, run.max_budget, run.indices, run.counts)
        elif args.three_calls:
            run.verify()
            run.topk()
        else:
            run.verify_select()
        run.decode()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly `steps` steps, nothing but the three entry points between the clocks
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = ev0.elapsed_time(ev1)

    # the same `steps` steps once more, each between its own event pair on the launch stream: median per step
    pairs_ev = []
    for _ in range(args.steps):
        a_ev, b_ev = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a_ev.record(stream)
        step()
        b_ev.record(stream)
        pairs_ev.append((a_ev, b_ev))
    torch.cuda.synchronize()
    per_step_us = sorted(x.elapsed_time(y) * 1e3 for x, y in pairs_ev)
    median_us = per_step_us[len(per_step_us) // 2]

    # the same `steps` steps again with a HIP event pair around every kernel (recorded by the
    # library on the launch stream): per-kernel durations; the events themselves stretch the step
    pa.pillar_profile_reset()
    pa.pillar_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof_wall_ms = (time.perf_counter() - t0) * 1e3
    pa.pillar_profile_enable(False)
    prof = pa.pillar_profile_read()

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)                                          # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = wall_ms / args.steps
    kern = {k: {"launches": n, "avg_us": round(ms * 1e3 / max(n, 1), 2)} for k, (n, ms) in prof.items()}
    stage_us = {"verify": 0.0, "topk": 0.0, "draft": 0.0}
    for k, (n, ms) in prof.items():
        per_step = ms * 1e3 / args.steps
        stage = "verify" if k.startswith("verify") else "topk" if k.startswith(("topk", "window")) else "draft"
        stage_us[stage] += per_step
    vb, db, tb = w.verify_bytes(), w.draft_bytes(), w.topk_bytes()
    verify_gbps = vb / (stage_us["verify"] * 1e-6) / 1e9 if stage_us["verify"] else 0.0
    draft_gbps = db / (stage_us["draft"] * 1e-6) / 1e9 if stage_us["draft"] else 0.0
    step_bytes = vb + db + tb
    step_gbps = step_bytes / (ms_per_step * 1e-3) / 1e9
    q_tokens = w.B * w.n_q + w.B          # query tokens served per step: k+1 verified + 1 drafted per request

    ceil = measured_ceilings(pa, torch, run.dev)
    stream_ceiling = ceil["stream_read_GBps"]
    dom = max(prof, key=lambda k: prof[k][1], default=None)
    dom_us = prof[dom][1] * 1e3 / max(prof[dom][0], 1) if dom else 0.0
    dom_bytes = vb if dom and dom.startswith("verify") else db if dom and dom.startswith("decode") else tb
    dom_gbps = dom_bytes / (dom_us * 1e-6) / 1e9 if dom_us else 0.0
    out = {
        "metric": METRIC,
        "value": round(ms_per_step * 1e3, 2),
        "unit": "µs/step",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"f32": "f32", "bf16": "bf16", "fp8_e4m3": "bf16 (fp8 e4m3 KV)"}[w.kv_dtype],
        "data": "synthetic",
        "config": {"workload": f"config {args.config}: {gen.CONFIGS[args.config]}",
                   "index_source": args.index_source,
                   "calls": "pillar_verify_attn (no statistic) + pillar_window_indices + pillar_sparse_decode"
                            if args.index_source == "window" else
                            "pillar_verify_attn + pillar_select_topk + pillar_sparse_decode" if args.three_calls
                            else "pillar_verify_select + pillar_sparse_decode",
                   "batch": w.B, "context_tokens": int(w.seq_lens.sum()), "spec_len_k": w.spec_k,
                   "selected_rows": w.selected_rows(), "truncated": args.batch is not None},
        "tokens_per_s": round(q_tokens / (ms_per_step * 1e-3), 1),
        "gpu_ms_per_step": round(gpu_ms / args.steps, 5),
        "median_us_per_step": round(median_us, 2),
        "ms_per_step_with_kernel_events": round(prof_wall_ms / args.steps, 5),
        "stage_us": {k: round(v, 2) for k, v in stage_us.items()},
        # a round of the method = one verification (with selection) and spec_len_k draft steps on its lists
        "round_us": round(stage_us["verify"] + stage_us["topk"] + w.spec_k * stage_us["draft"], 2),
        "query_tokens_per_s": {"verify": round(w.B * (w.spec_k + 1) / max((stage_us["verify"] + stage_us["topk"]) * 1e-6, 1e-12), 1),
                               "draft": round(w.B / max(stage_us["draft"] * 1e-6, 1e-12), 1)},
        "stage_gbps": {"verify": round(verify_gbps, 1), "draft": round(draft_gbps, 1), "step": round(step_gbps, 1)},
        "stage_frac_of_peak": {"verify": round(verify_gbps / HBM_PEAK_GBPS, 4),
                               "draft": round(draft_gbps / HBM_PEAK_GBPS, 4),
                               "step": round(step_gbps / HBM_PEAK_GBPS, 4)},
        "measured_ceilings": ceil,
        "stage_frac_of_stream_ceiling": {"verify": round(verify_gbps / stream_ceiling, 4),
                                         "draft": round(draft_gbps / stream_ceiling, 4),
                                         "step": round(step_gbps / stream_ceiling, 4)},
        "cache_state": "steps run back to back on the same pools and lists: a verification streams 4-10x the 256 MB "
                       "Infinity Cache, so no KV byte of one verification survives to the next; the rows a draft step "
                       "gathers (selected rows, 5-7 % of the KV) are still cached when the next verification reads them, "
                       "as they are in serving, where the draft steps of a round precede its verification",
        "algorithmic_bytes": {"verify": vb, "topk": tb, "draft": db},
        "kernels": kern,
        "roofline": {"bound": "hbm", "achieved": round(verify_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(verify_gbps / HBM_PEAK_GBPS, 4),
                     "frac_of_stream_ceiling": round(verify_gbps / stream_ceiling, 4),
                     "traffic": None if args.batch is not None else recorded_traffic(args.config),
                     "kernel": "verification stage = " + " + ".join(sorted(k for k in prof if k.startswith("verify"))),
                     "avg_us": round(stage_us["verify"], 2), "algorithmic_bytes": vb,
                     "stage_includes_selection": not args.three_calls,
                     "dominant_kernel": {"name": dom, "avg_us": round(dom_us, 2), "achieved": round(dom_gbps, 1),
                                         "frac": round(dom_gbps / HBM_PEAK_GBPS, 4)},
                     "note": "algorithmic bytes of the verification stage (every KV row once + one fp32 score per "
                             "token and KV head + Q and O) over the SUM of the average durations of all its kernels "
                             "(HIP events on the launch stream): the method needs the finish kernel (log-sum-exp, scores) as "
                             "much as the streaming pass, so the stage, not its longest kernel, is priced against the roofline; "
                             "dominant_kernel prices the same bytes against the longest kernel alone; with "
                             "pillar_verify_select the stage's time also contains the Top-K selection (its finish "
                             "kernel selects from on-chip scores) while its bytes do not; traffic is not "
                             "measured by this run: it is the HBM byte count (reads + writes, all kernels of the "
                             "stage, one step) that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command "
                             "recorded, see profiles/"},
    }
    if not args.no_cpu_baseline and args.index_source == "pillar":
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out, ensure_ascii=False))
    return 0


if __name__ == "__main__":
    sys.exit(main())
