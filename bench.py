#!/usr/bin/env python3
"""Benchmark of the PPSD decode hot path on one MI355X.

One "step" = one generation: prefill of the workload's prompt (untimed; the paper's speed metric is
decode-phase tokens/s, Sec. 5.1) followed by the timed ppsd_decode of the workload's decode length.
Prints ONE JSON line.

Default run: the headline is workload C4 (13B shape, prompt 512, decode 512: the largest one that runs on
one GPU), value = committed tokens/s of the PPSD schedule chosen BEFORE measuring from the table below;
that schedule is timed with the --steps / --warmup given, vanilla GPU decode and the other schedules with
a few generations each.  The same line carries the dominant kernel's HBM-roofline fraction (live HIP-event
timing), the per-committed-token fraction, the CPU oracle timed on this host, and sub-records for
workloads C2 (7B) and C5 (8B GQA, prompt 8192) under "workloads".  --workload NAME reports that workload
alone (C1, C2, C4, C5, a C3 cell such as C3_E8_a70, or C3 = the whole exit-layer x acceptance grid).
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
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_per_kernel.txt")

# Which PPSD schedule to run, decided before anything is measured.  Rows: the draft stage's share of the model,
# E / N; columns: acceptance below 0.6, 0.6 to 0.8, 0.8 and above.  Measured on the 7B exit-layer x acceptance
# grid (tokens/s relative to vanilla decode, two-stage / paper's ceil(N/E) stages / three stages):
#   E/N = 1/8:  0.87 / 0.47 / 0.86    0.91 / 0.60 / 0.95    0.96 / 0.95 / 1.12
#   E/N = 1/4:  0.91 / 0.72 / 0.83    0.96 / 0.87 / 0.95    1.02 / 1.16 / 1.15
#   E/N = 1/2:  0.91 / 0.93 / 0.70    1.01 / 1.02 / 0.84    1.09 / 1.11 / 0.99
# "three_stage" = the pipeline schedule with the layers behind the draft stage cut into two halves; at E/N = 1/2
# the paper's partition has two stages and differs from "overlap" in the kernels' prefetch depth only.
SCHEDULE_TABLE = (
    (0.1875, ("overlap", "three_stage", "three_stage")),
    (0.375, ("overlap", "overlap", "three_stage")),
    (1.0, ("pipeline", "pipeline", "pipeline")),
)


def choose_schedule(w, alpha_expected: float) -> str:
    frac = w.exit_layer / w.n_layers
    col = 0 if alpha_expected < 0.6 else 1 if alpha_expected < 0.8 else 2
    for upper, row in SCHEDULE_TABLE:
        if frac <= upper:
            return row[col]
    return "overlap"


def schedule_sessions(w, P):
    """name -> (library mode, extra configuration)."""
    half = -(-(w.n_layers - w.exit_layer) // 2)
    return {"vanilla": (P.MODE_VANILLA, {}), "serial": (P.MODE_SERIAL, {}), "overlap": (P.MODE_OVERLAP, {}),
            "pipeline": (P.MODE_PIPELINE, {}), "three_stage": (P.MODE_PIPELINE, {"pipeline_stage_layers": half}),
            "eesd": (P.MODE_EESD, {})}


SCHEDULE_TEXT = {"overlap": "two-stage verify-while-draft: draft stage and verify stage on two streams",
                 "pipeline": "the paper's ceil(N/E) stages of E layers, one stream per stage up to four",
                 "three_stage": "pipeline schedule with the layers behind the draft stage in two halves (three stages, three streams)",
                 "serial": "draft stage then verify stage on one stream", "vanilla": "autoregressive decode, no draft",
                 "eesd": "draft-then-verify rounds (Sec. 3.1), not PPSD"}


def algorithmic_bytes(w, mean_ctx: float):
    """Weights once + KV once per committed token (vanilla), plus PPSD's own extras."""
    layer = w.layer_weight_bytes()
    head = w.head_weight_bytes()
    kv = w.kv_bytes_per_position() * mean_ctx
    kv_draft = w.kv_bytes_per_position(w.exit_layer) * mean_ctx
    embed_row = w.d_model * w.elem_bytes
    vanilla = w.n_layers * layer + head + kv + embed_row
    xb = layer + w.kv_bytes_per_position(1) * mean_ctx if w.exit_block else 0   # the transformer-layer exit head
    accept_step = vanilla + head + xb                              # + exit head
    reject_extra = w.exit_layer * layer + head + xb + kv_draft + embed_row   # the wasted draft pass
    return dict(vanilla=vanilla, accept_step=accept_step, reject_extra=reject_extra, layer=layer, head=head, kv=kv)


def kernel_bytes(w, mean_ctx: float):
    """Algorithmic bytes per launch of each kernel kind (weights + vectors in/out)."""
    B, d, f = w.elem_bytes, w.d_model, w.d_ffn
    nq = w.n_heads * w.head_dim
    return {
        "qkv": w.qkv_rows * d * B + 4 * d + 4 * nq + 2 * w.n_kv_heads * w.head_dim * B,
        "attention": 2 * w.n_kv_heads * w.head_dim * B * mean_ctx + 8 * nq,
        "o_proj": d * nq * B + 4 * nq + 8 * d,
        "gate_up": 2 * f * d * B + 4 * d + 4 * f,
        "down": d * f * B + 4 * f + 8 * d,
        "head": w.vocab * d * B + 4 * d,
    }


def offline_traffic():
    """HBM bytes per dispatch from the tracked counter summary: {(workload, kernel kind): bytes}.

    The file holds raw FETCH_SIZE / WRITE_SIZE readings of rocprofv3 --pmc runs of ppsd_cli (the library's own
    kernels) plus the readings of a copy kernel of known size from the same runs, which give the bytes per unit."""
    if not os.path.exists(TRAFFIC_FILE):
        return {}, None
    rows, cal = [], None
    for line in open(TRAFFIC_FILE):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "calibration":
            cal = dict(fetch=float(t[2]), write=float(t[3]), bytes_read=float(t[6]), bytes_written=float(t[8]))
        else:
            rows.append((t[0], t[1], float(t[2]), float(t[3])))
    if cal is None:
        return {}, None
    fu, wu = cal["bytes_read"] / cal["fetch"], cal["bytes_written"] / cal["write"]
    return {(wl, k): f * fu + wr * wu for wl, k, f, wr in rows}, dict(fetch_unit_bytes=fu, write_unit_bytes=wu)


def progress(msg):
    """Progress lines on stderr (stdout carries the one JSON line)."""
    print("bench.py: " + msg, file=sys.stderr, flush=True)


def run_generations(ss, prompt, n_decode, steps, warmup, torch):
    times = []
    stats = None
    toks = None
    ss.prefill_ms = []
    for it in range(warmup + steps):
        torch.cuda.synchronize()
        tp = time.perf_counter()
        first = ss.ppsd_prefill(prompt)
        torch.cuda.synchronize()
        ss.prefill_ms.append(1e3 * (time.perf_counter() - tp))
        t0 = time.perf_counter()
        out = ss.ppsd_decode(n_decode)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        if it >= warmup:
            times.append(dt)
        stats = ss.ppsd_stats()
        toks = [first] + out
    return times, stats, toks


def cpu_oracle_baseline(w, W_gpu, prompt, torch, budget_s=25.0):
    """The CPU oracle as it stands, on a bounded sample of the same workload."""
    from oracle import decoder_fp64 as O
    W = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in W_gpu.items()}
    dec = O.Decoder(w, W)
    t0 = time.perf_counter()
    O.greedy_decode(dec, prompt[:2], 1)                      # 2 positions: sizes the sample
    per_pos = (time.perf_counter() - t0) / 2
    n_pos = int(max(2, min(24, budget_s / max(per_pos, 1e-6))))
    t0 = time.perf_counter()
    O.greedy_decode(dec, prompt[:n_pos], 1)                  # n_pos positions through the full model
    dt = time.perf_counter() - t0
    return dict(value=n_pos / dt, unit="tokens/s", cores=torch.get_num_threads(), kind="oracle",
                sample=f"fp64 oracle (KV-cache greedy decode, one position at a time), full {w.name} model, the first "
                       f"{n_pos} positions of the workload's prompt (context 1..{n_pos}, not the workload's context of "
                       f"{w.prompt_len}+: the oracle's time per position is dominated by its fp64 weight products, which "
                       f"do not depend on the context); tokens/s = positions / wall time ({dt:.1f} s)")


def measure(w, W, prompt, plan, args, torch, P, engine=None):
    """Runs the schedules of `plan` (name -> (steps, warmup)) and returns name -> result, plus the token streams."""
    n = w.decode_len
    n_stages = -(-w.n_layers // w.exit_layer)
    max_seq = w.prompt_len + 1 + n + max(1, n_stages - 1, 4)  # + the positions drafted ahead of the last commit
    sessions = schedule_sessions(w, P)
    engine = P.ENGINE_STREAMS if engine is None else engine
    res, streams = {}, {}
    for name, (steps, warmup) in plan.items():
        mode, extra = sessions[name]
        if mode == P.MODE_PIPELINE and (engine != P.ENGINE_STREAMS or n_stages > 16):
            continue
        if mode == P.MODE_EESD and (engine != P.ENGINE_STREAMS or 4 * 4 * w.d_model > 150 * 1024):
            continue
        if engine != P.ENGINE_STREAMS and name == "three_stage":
            continue
        kw = dict(extra)
        if mode == P.MODE_PIPELINE and args.pipeline_streams:
            kw["pipeline_streams"] = args.pipeline_streams
        if mode == P.MODE_EESD and args.gamma:
            kw["eesd_gamma"] = args.gamma
        ss = P.Session(w, W, max_seq=max_seq, mode=mode, engine=engine, prefill_loop=args.prefill_loop,
                       tune_wgs_per_cu=args.wgs_per_cu, tune_attn_split=args.attn_split,
                       tune_draft_share=args.draft_share, temperature=args.temperature, sample_seed=args.sample_seed, **kw)
        info = ss.launch_info()
        times, st, toks = run_generations(ss, prompt, n, steps, warmup, torch)
        prefill_ms = min(ss.prefill_ms)
        ss.close()
        total = sum(times)
        ts = sorted(times)
        progress(f"{w.name} {name}: {steps * n / total:.1f} tokens/s over {steps} generation(s) of {n} tokens")
        res[name] = dict(tokens_per_s=steps * n / total, ms_per_generation=1e3 * total / steps,
                         ms_per_token=1e3 * total / (steps * n), stats=st, prefill_ms=prefill_ms, steps=steps, warmup=warmup,
                         ms_per_generation_min=1e3 * ts[0], ms_per_generation_median=1e3 * ts[len(ts) // 2], launch=info)
        streams[name] = toks
    # vanilla and the PPSD schedules run the same kernels per token: their streams must be identical.  The batched
    # verify pass of the eesd mode keeps the per-token order of operations too; how far its stream agrees with the
    # others is reported rather than enforced.
    exact = {k: v for k, v in streams.items() if k != "eesd" and not (args.temperature > 0 and k == "vanilla")}
    if len(exact) > 1:
        first = next(iter(exact.values()))
        if any(s != first for s in exact.values()):
            print(f"bench.py: {w.name}: schedules disagree on the token stream", file=sys.stderr)
            sys.exit(1)
    if "eesd" in streams and exact:
        ref = next(iter(exact.values()))
        same = 0
        while same < len(ref) and streams["eesd"][same] == ref[same]:
            same += 1
        res["eesd"]["tokens_equal_to_vanilla_stream"] = same
    return res, streams, max_seq


def kernel_timing(w, W, prompt, max_seq, args, P, traffic):
    """Live per-kernel timing: vanilla decode of 32 tokens with direct launches on one stream and one HIP event
    between consecutive kernels (recorded on that stream by the library); an interval holds one kernel and one
    event, and the event's own cost, measured live on the same stream, is taken off."""
    n = min(w.decode_len, 32)
    ss = P.Session(w, W, max_seq=max_seq, mode=P.MODE_VANILLA, use_graph=False, time_kernels=True,
                   tune_wgs_per_cu=args.wgs_per_cu, tune_attn_split=args.attn_split)
    ss.ppsd_prefill(prompt)
    ss.ppsd_decode(n)
    kt = ss.kernel_times()
    ss.close()
    kb = kernel_bytes(w, w.prompt_len + 1 + n / 2.0)
    ev_us = kt.pop("event_overhead_us")
    ktimes = {}
    for k, v in kt.items():
        if v["launches"] and k in kb:
            raw = v["total_us"] / v["launches"]
            us = raw - ev_us
            ktimes[k] = dict(avg_us=us, avg_interval_us=raw, launches=v["launches"], bytes=kb[k], gbps=kb[k] / us / 1e3,
                             frac_of_peak=kb[k] / us / 1e3 / HBM_PEAK_GBPS)
    dom = max((k for k in ktimes), key=lambda k: ktimes[k]["avg_us"] * ktimes[k]["launches"])
    roofline = dict(bound="hbm", kernel=dom, achieved=ktimes[dom]["gbps"], peak=HBM_PEAK_GBPS, unit="GB/s",
                    frac=ktimes[dom]["gbps"] / HBM_PEAK_GBPS, traffic=traffic.get((w.name, dom)),
                    traffic_source="profiles/hbm_traffic_per_kernel.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of the "
                                   "library's kernels under ppsd_cli, scaled by a copy kernel of known size in the same runs "
                                   "(offline; null for shapes the file does not hold)",
                    avg_launch_us=ktimes[dom]["avg_us"], bytes_per_launch=ktimes[dom]["bytes"],
                    event_interval_us=ktimes[dom]["avg_interval_us"], event_overhead_us=ev_us)
    return ktimes, roofline


def workload_record(w, res, chosen, ab, n_stages):
    """What one workload measured: every schedule, the chosen one's fractions, acceptance."""
    r = res[chosen]
    st = r["stats"]
    alpha = st["accepted"] / st["drafts_compared"] if st["drafts_compared"] else None
    moved = None
    if chosen in ("pipeline", "three_stage"):
        S_run = r["launch"]["pipeline_stages"]
        # weights and KV of one stage run (the stages differ in size; the mean is exact for a full tick)
        per_stage_run = (ab["vanilla"] - ab["head"]) / S_run
        moved = (st["stage_runs"] * per_stage_run + st["pipeline_ticks"] * ab["head"] + st["committed"] * ab["head"]) / st["committed"]
    elif alpha is not None:
        moved = ab["accept_step"] + (1 - alpha) * ab["reject_extra"]
    van = res.get("vanilla")
    modes = {}
    for k, v in res.items():
        s = v["stats"]
        m = {"tokens_per_s": v["tokens_per_s"], "ms_per_token": v["ms_per_token"], "generations_timed": v["steps"],
             "hbm_frac_per_committed_token": v["tokens_per_s"] * ab["vanilla"] / (HBM_PEAK_GBPS * 1e9),
             "speedup_vs_vanilla_gpu": v["tokens_per_s"] / van["tokens_per_s"] if van else None,
             "steps_draft_only": s["steps_draft_only"], "accepted": s["accepted"], "rejected": s["rejected"],
             "schedule": SCHEDULE_TEXT[k]}
        if k in ("pipeline", "three_stage"):
            m.update(stages=v["launch"]["pipeline_stages"], streams=v["launch"]["streams"], ticks=s["pipeline_ticks"],
                     stage_runs=s["stage_runs"], flushed_tokens=s["flushed_tokens"])
        if k == "overlap":
            m["draft_share_of_256"] = v["launch"]["draft_share_of_256"]
        if k == "eesd":
            m.update(gamma=v["launch"]["eesd_gamma"], rounds=s["eesd_rounds"],
                     tokens_per_round=s["committed"] / max(1, s["eesd_rounds"]),
                     leading_tokens_equal_to_the_other_modes=v.get("tokens_equal_to_vanilla_stream"))
        modes[k] = m
    ppsd = [k for k in ("overlap", "pipeline", "three_stage") if k in res]
    best = max(ppsd, key=lambda k: res[k]["tokens_per_s"]) if ppsd else None
    return dict(
        schedule=chosen, schedule_text=SCHEDULE_TEXT[chosen], tokens_per_s=r["tokens_per_s"], ms_per_token=r["ms_per_token"],
        acceptance_rate=alpha, speedup_vs_vanilla_gpu=r["tokens_per_s"] / van["tokens_per_s"] if van else None,
        vanilla_tokens_per_s=van["tokens_per_s"] if van else None,
        hbm_frac_per_committed_token=r["tokens_per_s"] * ab["vanilla"] / (HBM_PEAK_GBPS * 1e9),
        hbm_frac_vanilla=van["tokens_per_s"] * ab["vanilla"] / (HBM_PEAK_GBPS * 1e9) if van else None,
        hbm_frac_per_moved_byte=moved and r["tokens_per_s"] * moved / (HBM_PEAK_GBPS * 1e9),
        bytes_per_token={"vanilla": ab["vanilla"], "ppsd_accept_step": ab["accept_step"], "ppsd_extra_per_reject": ab["reject_extra"],
                         "moved_by_the_chosen_schedule": moved},
        fastest_ppsd_schedule_measured=best, attention_splits=r["launch"]["attn_splits"],
        prefill={"ms": r["prefill_ms"], "tokens_per_s": w.prompt_len / r["prefill_ms"] * 1e3,
                 "path": "MFMA GEMMs and attention over chunks of %d positions" % r["launch"]["prefill_chunk"]
                 if r["launch"]["prefill_matrix_core"] else "looped decode kernels"},
        modes=modes), moved


def describe(w, n):
    return (f"{w.name}: {w.n_layers}-layer d={w.d_model} decoder ({w.dtype}), {w.n_heads}/{w.n_kv_heads} heads x {w.head_dim}, "
            f"exit layer {w.exit_layer}, prompt {w.prompt_len}, decode {n} tokens, batch 1, damp {w.damp}, exit head {w.exit_head}"
            + (f" behind a transformer layer (damp {w.exit_block_damp})" if w.exit_block else ""))


def plan_for(chosen, names, steps, warmup, short=(3, 1)):
    """The chosen schedule gets the run's --steps / --warmup, every other schedule a few generations."""
    return {k: ((steps, warmup) if k == chosen else (min(steps, short[0]), min(warmup, short[1]))) for k in names}


def c3_grid_report(args, torch, S, P):
    """Exit layer x acceptance grid on the 7B shape: PPSD speedup over vanilla GPU decode per cell and schedule."""
    from oracle import speedup_model as M
    cells_out = []
    vanilla_tps = None
    for w in S.c3_grid():
        W = S.make_weights(w, device="cuda")
        prompt = S.make_prompt(w)
        n = w.decode_len
        ab = algorithmic_bytes(w, w.prompt_len + 1 + n / 2.0)
        chosen = choose_schedule(w, w.acceptance_target)
        names = ["overlap", "pipeline", "three_stage"] + (["vanilla"] if vanilla_tps is None else [])
        res, _, _ = measure(w, W, prompt, {k: (args.steps, args.warmup) for k in names}, args, torch, P)
        if vanilla_tps is None:          # depends on the shape only
            vanilla_tps = res["vanilla"]["tokens_per_s"]
        st = res["overlap"]["stats"]
        alpha = st["accepted"] / st["drafts_compared"]
        per = {k: {"tokens_per_s": res[k]["tokens_per_s"], "speedup": res[k]["tokens_per_s"] / vanilla_tps,
                   "stages": res[k]["launch"]["pipeline_stages"] if k != "overlap" else 2} for k in ("overlap", "pipeline", "three_stage")}
        cells_out.append({
            "cell": w.name, "exit_layer": w.exit_layer, "damp": w.damp, "acceptance_target": w.acceptance_target,
            "acceptance_rate": alpha, "schedule_chosen_beforehand": chosen, "tokens_per_s": per[chosen]["tokens_per_s"],
            "speedup_vs_vanilla_gpu": per[chosen]["speedup"], "schedules": per,
            "fastest_schedule_measured": max(per, key=lambda k: per[k]["tokens_per_s"]),
            "byte_model_ratio": ab["vanilla"] / (ab["accept_step"] + (1 - alpha) * ab["reject_extra"]),
            "paper_eq7_gain_one_gpu_per_stage": M.ppsd_gain(alpha, w.exit_layer, w.n_layers)})
        del W
        torch.cuda.empty_cache()
    best = max(cells_out, key=lambda c: c["tokens_per_s"])
    print(json.dumps({
        "metric": "committed tokens/sec at batch 1 (PPSD decode), exit-layer x acceptance grid on the 7B shape",
        "value": best["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * 256 / best["tokens_per_s"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C3: 7B shape bf16, prompt 256, decode 256, batch 1; value = best cell " + best["cell"],
                   "schedule_table": SCHEDULE_TABLE},
        "vanilla_tokens_per_s": vanilla_tps, "cells": cells_out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=None,
                    help="default: headline C4 with sub-records C2 and C5; a name reports that workload alone")
    ap.add_argument("--damp", type=float, default=None, help="override the workload's damp")
    ap.add_argument("--exit-layer", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-sub-workloads", action="store_true", help="default run: skip the C2 and C5 sub-records")
    ap.add_argument("--modes", default="vanilla,overlap,pipeline,three_stage,eesd",
                    help="schedules to run: vanilla, serial, overlap (two-stage), pipeline (the paper's ceil(N/E) stages), "
                         "three_stage, eesd (draft-then-verify rounds, the method the paper compares against)")
    ap.add_argument("--schedule", default=None, choices=["overlap", "pipeline", "three_stage"],
                    help="override the schedule the table would choose for the headline")
    ap.add_argument("--exit-head", default=None, choices=["tied", "independent", "blend"],
                    help="override the workload's exit-head initialisation (independent: acceptance near 0)")
    ap.add_argument("--exit-block", type=float, default=None, metavar="DAMP",
                    help="use the transformer-layer early-exit head; DAMP scales its output projections "
                         "(0 = identity block: the norm head's drafts at the block's cost)")
    ap.add_argument("--temperature", type=float, default=0.0,
                    help="> 0: stochastic verification (sampled drafts, Eq. 2) in every mode")
    ap.add_argument("--sample-seed", type=int, default=2509)
    ap.add_argument("--gamma", type=int, default=0, help="drafts per round of the eesd mode (0 = library default, 3)")
    ap.add_argument("--engine", default="streams", choices=["streams", "persistent"])
    ap.add_argument("--pipeline-streams", type=int, default=0, help="streams of the pipeline mode (0 = library default)")
    ap.add_argument("--wgs-per-cu", type=int, default=0, help="launch tuning of the weight-streaming kernels (0 = defaults)")
    ap.add_argument("--draft-share", type=int, default=0,
                    help="launch tuning of the overlap mode: percent of its workgroups the draft stage works with beside the "
                         "verify stage (0 = default)")
    ap.add_argument("--attn-split", type=int, default=0, help="launch tuning: positions of capacity per attention split (0 = default)")
    ap.add_argument("--prefill-loop", action="store_true", help="prefill with the decode kernels, one position at a time")
    ap.add_argument("--prompt-len", type=int, default=None, help="override the workload's prompt length")
    ap.add_argument("--decode-len", type=int, default=None, help="override the workload's decode length")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the pipeline stages share one MI355X); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth_inputs as S
    import paper_2509_19368_amd as P
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    P.load_library()

    cells = {c.name: c for c in S.c3_grid()}
    if args.workload == "C3":
        return c3_grid_report(args, torch, S, P)
    default_run = args.workload is None
    name = "C4" if default_run else args.workload
    w = cells[name] if name in cells else S.WORKLOADS[name]
    if args.damp is not None:
        w = w.replace(damp=args.damp)
    if args.exit_layer is not None:
        w = w.replace(exit_layer=args.exit_layer)
    if args.exit_head is not None:
        w = w.replace(exit_head=args.exit_head, exit_beta=1.0 if args.exit_head == "blend" else 0.0)
    if args.exit_block is not None:
        w = w.replace(exit_block=True, exit_block_damp=args.exit_block)
    if args.prompt_len is not None:
        w = w.replace(prompt_len=args.prompt_len)
    if args.decode_len is not None:
        w = w.replace(decode_len=args.decode_len)
    traffic, traffic_units = offline_traffic()
    engine = P.ENGINE_PERSISTENT if args.engine == "persistent" else P.ENGINE_STREAMS

    def one_workload(w, steps, warmup, headline):
        progress(f"{w.name}: generating weights")
        t0 = time.perf_counter()
        W = S.make_weights(w, device="cuda")
        torch.cuda.synchronize()
        gen_s = time.perf_counter() - t0
        prompt = S.make_prompt(w)
        n = w.decode_len
        n_stages = -(-w.n_layers // w.exit_layer)
        ab = algorithmic_bytes(w, w.prompt_len + 1 + n / 2.0)
        alpha_expected = w.acceptance_target or 0.8
        if args.exit_head == "independent":
            alpha_expected = 0.0
        if args.damp == 0.0:
            alpha_expected = 1.0
        chosen = (headline and args.schedule) or choose_schedule(w, alpha_expected)
        if engine != P.ENGINE_STREAMS or n_stages > 16:
            chosen = "overlap"
        names = [k for k in args.modes.split(",") if k]
        if chosen not in names:
            names.append(chosen)
        res, streams, max_seq = measure(w, W, prompt, plan_for(chosen, names, steps, warmup), args, torch, P, engine)
        rec, moved = workload_record(w, res, chosen, ab, n_stages)
        rec["distinct_tokens_in_stream"] = len(set(next(iter(streams.values()))))
        rec["weight_generation_s"] = gen_s
        rec["workload"] = describe(w, n)
        rec["schedule_chosen_from"] = (f"table in bench.py at E/N = {w.exit_layer}/{w.n_layers}, expected acceptance "
                                       f"{alpha_expected}" if not (headline and args.schedule) else "--schedule")
        ktimes = roofline = None
        if not args.no_kernel_timing and engine == P.ENGINE_STREAMS:
            progress(f"{w.name}: per-kernel timing pass")
            ktimes, roofline = kernel_timing(w, W, prompt, max_seq, args, P, traffic)
            roofline["frac_per_committed_token"] = rec["hbm_frac_per_committed_token"]
        elif not args.no_kernel_timing:
            # persistent engine: the whole decode call is ONE launch; its duration is the library's own event pair
            st = res[chosen]["stats"]
            mv = n * (moved or ab["vanilla"])
            gbps = mv / st["device_ms"] / 1e6
            roofline = dict(bound="hbm", kernel=f"k_mega ({chosen} decode of {n} tokens in one launch)", achieved=gbps,
                            peak=HBM_PEAK_GBPS, unit="GB/s", frac=gbps / HBM_PEAK_GBPS, traffic=None,
                            avg_launch_us=st["device_ms"] * 1e3, bytes_per_launch=mv,
                            frac_per_committed_token=rec["hbm_frac_per_committed_token"])
        return W, prompt, res, rec, ktimes, roofline, chosen

    W, prompt, res, rec, ktimes, roofline, chosen = one_workload(w, args.steps, args.warmup, True)
    r = res[chosen]
    # what a pure streaming read reaches on this chip (the library's probe kernel over 4 GiB, 10 launches)
    probe = torch.empty(4 << 30, dtype=torch.uint8, device="cuda").fill_(0x3c)
    probe_ms = P.hbm_read_probe(probe, iters=10)
    stream_gbps = probe.numel() / probe_ms / 1e6
    del probe
    cpu = None
    if not args.no_cpu_baseline:
        progress(f"{w.name}: CPU oracle baseline (about half a minute)")
        cpu = cpu_oracle_baseline(w, W, prompt, torch)
        progress(f"{w.name}: CPU oracle {cpu['value']:.3f} tokens/s on {cpu['cores']} threads")
    del W
    torch.cuda.empty_cache()

    subs = {}
    if default_run and not args.no_sub_workloads:
        for sub in ("C2", "C5"):
            sw = S.WORKLOADS[sub]
            sW, _, sres, srec, skt, sroof, _ = one_workload(sw, min(args.steps, 3), min(args.warmup, 1), False)
            del sW
            torch.cuda.empty_cache()
            srec["roofline_dominant_kernel"] = sroof
            srec["kernels"] = skt
            subs[sub] = srec

    moved = rec["bytes_per_token"]["moved_by_the_chosen_schedule"]
    out = {
        "metric": "committed tokens/sec at batch 1 (PPSD decode on one GPU; schedule chosen beforehand, named in config.schedule)",
        "value": r["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_generation"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": rec["workload"], "schedule": chosen + ": " + SCHEDULE_TEXT[chosen],
                   "schedule_chosen_from": rec["schedule_chosen_from"], "engine": args.engine, "tokens_per_step": w.decode_len,
                   **({"temperature": args.temperature, "sample_seed": args.sample_seed,
                       "verification": "stochastic (Eq. 2)"} if args.temperature > 0 else {})},
        "acceptance_rate": rec["acceptance_rate"],
        "ms_per_token": r["ms_per_token"],
        "speedup_vs_vanilla_gpu": rec["speedup_vs_vanilla_gpu"],
        "vanilla_tokens_per_s": rec["vanilla_tokens_per_s"],
        "hbm_frac_per_committed_token": rec["hbm_frac_per_committed_token"],
        "hbm_frac_vanilla": rec["hbm_frac_vanilla"],
        "hbm_frac_per_moved_byte": rec["hbm_frac_per_moved_byte"],
        "hbm_stream_read_ceiling_gbps": stream_gbps,
        "frac_of_stream_read_ceiling_per_moved_byte": moved and r["tokens_per_s"] * moved / (stream_gbps * 1e9),
        "fastest_ppsd_schedule_measured": rec["fastest_ppsd_schedule_measured"],
        "modes": rec["modes"], "bytes_per_token": rec["bytes_per_token"],
        "distinct_tokens_in_stream": rec["distinct_tokens_in_stream"],
        "ms_per_generation_min": r["ms_per_generation_min"], "ms_per_generation_median": r["ms_per_generation_median"],
        "prefill": rec["prefill"], "attention_splits": rec["attention_splits"],
        "roofline": roofline, "kernels": ktimes, "cpu_baseline": cpu,
        "counter_units": traffic_units, "weight_generation_s": rec["weight_generation_s"],
        "schedule_table": {"rows_E_over_N_up_to": [row[0] for row in SCHEDULE_TABLE],
                           "columns_acceptance": ["< 0.6", "0.6 - 0.8", ">= 0.8"], "schedules": [row[1] for row in SCHEDULE_TABLE]},
        "workloads": subs or None,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
