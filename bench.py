#!/usr/bin/env python3
"""Benchmark of the PPSD decode hot path on one MI355X.

One "step" = one generation: prefill of the workload's prompt (untimed; the paper's speed metric
is decode-phase tokens/s) followed by the timed ppsd_decode of the workload's decode length.
Prints ONE JSON line.  value = committed tokens/s of PPSD (overlapped draft/verify stages);
the same line carries vanilla GPU decode, the acceptance rate, the HBM-roofline fraction of the
dominant kernel (live HIP-event timing) and the CPU oracle timed on this host.
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

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE (scaled by reference
# dispatches of known size: one FETCH_SIZE unit = 2 KiB, one WRITE_SIZE unit = 1 KiB), at the 7B, 13B and
# 8B-GQA shapes: profiles/weight_streaming_kernels_7B_shapes_pmc.md
MEASURED_TRAFFIC_BYTES = {
    ("C2", "gate_up"): 88233.2 * 2048 + 43.1 * 1024,
    ("C2", "qkv"): 49329.5 * 2048 + 48.0 * 1024,
    ("C2", "head"): 128176.9 * 2048 + 20.9 * 1024,
    ("C2", "o_proj"): 16519.5 * 2048 + 16.0 * 1024,
    ("C2", "down"): 44281.1 * 2048 + 16.0 * 1024,
    ("C4", "gate_up"): 138442.7 * 2048 + 54.1 * 1024,
    ("C4", "qkv"): 77018.4 * 2048 + 60.0 * 1024,
    ("C4", "head"): 160208.9 * 2048 + 20.8 * 1024,
    ("C4", "o_proj"): 25759.6 * 2048 + 20.0 * 1024,
    ("C4", "down"): 69417.7 * 2048 + 20.0 * 1024,
    ("C5", "gate_up"): 114857.5 * 2048 + 56.2 * 1024,
    ("C5", "qkv"): 24753.5 * 2048 + 24.0 * 1024,
    ("C5", "head"): 513205.9 * 2048 + 22.8 * 1024,
    ("C5", "o_proj"): 16519.6 * 2048 + 16.0 * 1024,
    ("C5", "down"): 57646.1 * 2048 + 16.0 * 1024,
}


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
    return dict(vanilla=vanilla, accept_step=accept_step, reject_extra=reject_extra, layer=layer, head=head)


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
                sample=f"fp64 oracle (KV-cache greedy decode), full {w.name} model, the first {n_pos} positions "
                       f"of the workload's prompt, one position at a time; tokens/s = positions / wall time "
                       f"({dt:.1f} s)")


def c3_grid_report(args, torch, S, P):
    """Exit layer x acceptance grid on the 7B shape: PPSD speedup over vanilla GPU decode per cell."""
    from oracle import speedup_model as M
    cells_out = []
    vanilla_tps = None
    engine = P.ENGINE_PERSISTENT if args.engine == "persistent" else P.ENGINE_STREAMS
    for w in S.c3_grid():
        W = S.make_weights(w, device="cuda")
        prompt = S.make_prompt(w)
        n_stages = -(-w.n_layers // w.exit_layer)
        n, max_seq = w.decode_len, w.prompt_len + 1 + w.decode_len + max(1, n_stages - 1)
        ab = algorithmic_bytes(w, w.prompt_len + 1 + n / 2.0)
        if vanilla_tps is None:          # depends on the shape only
            ss = P.Session(w, W, max_seq=max_seq, mode=P.MODE_VANILLA, engine=engine)
            t, _, _ = run_generations(ss, prompt, n, args.steps, args.warmup, torch)
            ss.close()
            vanilla_tps = args.steps * n / sum(t)
        ss = P.Session(w, W, max_seq=max_seq, mode=P.MODE_OVERLAP, engine=engine)
        t, st, _ = run_generations(ss, prompt, n, args.steps, args.warmup, torch)
        ss.close()
        tps2 = args.steps * n / sum(t)
        alpha = st["accepted"] / st["drafts_compared"]
        tps3 = None
        if engine == P.ENGINE_STREAMS and n_stages <= 16:
            ss = P.Session(w, W, max_seq=max_seq, mode=P.MODE_PIPELINE, engine=engine)
            t, _, _ = run_generations(ss, prompt, n, args.steps, args.warmup, torch)
            ss.close()
            tps3 = args.steps * n / sum(t)
        tps = max(tps2, tps3 or 0.0)
        cells_out.append({
            "cell": w.name, "exit_layer": w.exit_layer, "damp": w.damp, "acceptance_rate": alpha, "tokens_per_s": tps,
            "speedup_vs_vanilla_gpu": tps / vanilla_tps,
            "two_stage": {"tokens_per_s": tps2, "speedup": tps2 / vanilla_tps},
            "pipeline": {"stages": n_stages, "tokens_per_s": tps3, "speedup": tps3 and tps3 / vanilla_tps},
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
                   "engine": args.engine},
        "vanilla_tokens_per_s": vanilla_tps, "cells": cells_out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--damp", type=float, default=None, help="override the workload's damp")
    ap.add_argument("--exit-layer", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--modes", default="vanilla,serial,overlap,pipeline,eesd",
                    help="pipeline = the full ceil(N/E)-stage schedule; eesd = draft-then-verify rounds (the method the "
                         "paper compares against), both reported beside the two-stage path")
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
    ap.add_argument("--draft-share", type=int, default=0, help="launch tuning of the overlap mode: percent of its workgroups the draft stage works with beside the verify stage (0 = default)")
    ap.add_argument("--attn-split", type=int, default=0, help="launch tuning: positions of capacity per attention split (0 = default)")
    ap.add_argument("--prefill-loop", action="store_true", help="prefill with the decode kernels, one position at a time")
    ap.add_argument("--prompt-len", type=int, default=None, help="override the workload's prompt length")
    ap.add_argument("--decode-len", type=int, default=None, help="override the workload's decode length")
    ap.add_argument("--calibrate", action="store_true",
                    help="first run a 1 GiB device copy and a 1 GiB streaming read (reference dispatches for "
                         "scaling rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the two pipeline stages share one MI355X); "
              "--gpus must be 1", file=sys.stderr)
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
    w = cells[args.workload] if args.workload in cells else S.WORKLOADS[args.workload]
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
    if args.calibrate:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)                       # reads 1 GiB, writes 1 GiB
        P.hbm_read_probe(src, iters=1)       # k_read_probe twice (warm-up + 1): reads 1 GiB each
        torch.cuda.synchronize()
        del src, dst
    t0 = time.perf_counter()
    W = S.make_weights(w, device="cuda")
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0
    prompt = S.make_prompt(w)
    n = w.decode_len
    n_stages = -(-w.n_layers // w.exit_layer)
    max_seq = w.prompt_len + 1 + n + max(1, n_stages - 1, 4)  # + the positions drafted ahead of the last commit
    mean_ctx = w.prompt_len + 1 + n / 2.0
    ab = algorithmic_bytes(w, mean_ctx)

    engine = P.ENGINE_PERSISTENT if args.engine == "persistent" else P.ENGINE_STREAMS
    res = {}
    streams = {}
    for name, mode in (("vanilla", P.MODE_VANILLA), ("serial", P.MODE_SERIAL), ("overlap", P.MODE_OVERLAP),
                       ("pipeline", P.MODE_PIPELINE), ("eesd", P.MODE_EESD)):
        if name not in args.modes.split(","):
            continue
        if mode == P.MODE_PIPELINE and (engine != P.ENGINE_STREAMS or n_stages > 16):
            continue
        if mode == P.MODE_EESD and (engine != P.ENGINE_STREAMS or 4 * 4 * w.d_model > 150 * 1024):
            continue
        ss = P.Session(w, W, max_seq=max_seq, mode=mode, engine=engine, prefill_loop=args.prefill_loop,
                       pipeline_streams=args.pipeline_streams if mode == P.MODE_PIPELINE else 0,
                       tune_wgs_per_cu=args.wgs_per_cu, tune_attn_split=args.attn_split, tune_draft_share=args.draft_share,
                       eesd_gamma=args.gamma if mode == P.MODE_EESD else 0,
                       temperature=args.temperature, sample_seed=args.sample_seed)
        times, st, toks = run_generations(ss, prompt, n, args.steps, args.warmup, torch)
        prefill_ms = min(ss.prefill_ms)
        ss.close()
        total = sum(times)
        ts = sorted(times)
        res[name] = dict(tokens_per_s=args.steps * n / total, ms_per_generation=1e3 * total / args.steps,
                         ms_per_token=1e3 * total / (args.steps * n), stats=st, prefill_ms=prefill_ms,
                         ms_per_generation_min=1e3 * ts[0], ms_per_generation_median=1e3 * ts[len(ts) // 2])
        streams[name] = toks
    # vanilla and the PPSD schedules run the same kernels per token: their streams must be identical.  The
    # batched verify pass of the eesd mode keeps the per-token order of operations too; how far its stream
    # agrees with the others is reported rather than enforced.
    exact = {k: v for k, v in streams.items() if k != "eesd" and not (args.temperature > 0 and k == "vanilla")}
    if len(exact) > 1:
        first = next(iter(exact.values()))
        if any(s != first for s in exact.values()):
            print("bench.py: modes disagree on the token stream", file=sys.stderr)
            sys.exit(1)
    if "eesd" in streams and exact:
        ref = next(iter(exact.values()))
        same = 0
        while same < len(ref) and streams["eesd"][same] == ref[same]:
            same += 1
        res["eesd"]["tokens_equal_to_vanilla_stream"] = same

    # the headline is the fastest PPSD schedule the library has (two-stage verify-while-draft on two
    # streams, or the full ceil(N/E)-stage schedule on up to four streams); every mode is listed
    ppsd_modes = [k for k in ("overlap", "pipeline") if k in res]
    main_mode = max(ppsd_modes, key=lambda k: res[k]["tokens_per_s"]) if ppsd_modes else next(iter(res))
    r = res[main_mode]
    st = r["stats"]
    alpha = st["accepted"] / st["drafts_compared"] if st["drafts_compared"] else None

    # live per-kernel timing (HIP events around every launch, serial single-stream pass)
    roofline = None
    ktimes = None
    if not args.no_kernel_timing and engine == P.ENGINE_PERSISTENT:
        # the whole decode call is ONE kernel launch; its duration comes from the HIP event pair the
        # library records on the launching stream around it (ppsd_stats.device_ms of the last call)
        moved = n * ab["accept_step"] + st["rejected"] * ab["reject_extra"] if main_mode != "vanilla" else n * ab["vanilla"]
        dur_ms = st["device_ms"]
        gbps = moved / dur_ms / 1e6
        roofline = dict(bound="hbm", kernel=f"k_mega ({main_mode} decode of {n} tokens in one launch)", achieved=gbps,
                        peak=HBM_PEAK_GBPS, unit="GB/s", frac=gbps / HBM_PEAK_GBPS, traffic=None,
                        avg_launch_us=dur_ms * 1e3, bytes_per_launch=moved)
    elif not args.no_kernel_timing:
        ss = P.Session(w, W, max_seq=max_seq, mode=P.MODE_VANILLA, use_graph=False, time_kernels=True,
                       tune_wgs_per_cu=args.wgs_per_cu, tune_attn_split=args.attn_split)
        ss.ppsd_prefill(prompt)
        ss.ppsd_decode(min(n, 32))
        kt = ss.kernel_times()
        ss.close()
        ctx_t = w.prompt_len + 1 + min(n, 32) / 2.0
        kb = kernel_bytes(w, ctx_t)
        # an interval between two events holds one kernel and one event; the event's own cost, measured
        # live on the same stream (events back to back, no kernel), is taken off
        ev_us = kt.pop("event_overhead_us")
        ktimes = {}
        for k, v in kt.items():
            if v["launches"] and k in kb:
                raw = v["total_us"] / v["launches"]
                us = raw - ev_us
                ktimes[k] = dict(avg_us=us, avg_interval_us=raw, launches=v["launches"], bytes=kb[k], gbps=kb[k] / us / 1e3)
        dom = max((k for k in ktimes), key=lambda k: ktimes[k]["avg_us"] * ktimes[k]["launches"])
        roofline = dict(bound="hbm", kernel=dom, achieved=ktimes[dom]["gbps"], peak=HBM_PEAK_GBPS, unit="GB/s",
                        frac=ktimes[dom]["gbps"] / HBM_PEAK_GBPS,
                        traffic=MEASURED_TRAFFIC_BYTES.get((w.name, dom)),
                        avg_launch_us=ktimes[dom]["avg_us"], bytes_per_launch=ktimes[dom]["bytes"],
                        event_interval_us=ktimes[dom]["avg_interval_us"], event_overhead_us=ev_us)

    # bytes the schedule really moved per committed token (wasted drafts included)
    moved_per_token = None
    if main_mode == "pipeline":
        per_stage_run = (ab["vanilla"] - ab["head"]) / n_stages          # E layers of weights + their KV reads
        moved_per_token = (st["stage_runs"] * per_stage_run + st["pipeline_ticks"] * ab["head"]
                           + st["committed"] * ab["head"]) / st["committed"]
    elif alpha is not None:
        moved_per_token = ab["accept_step"] + (1 - alpha) * ab["reject_extra"]
    # what a pure streaming read reaches on this chip (the library's probe kernel over 4 GiB, 10 launches)
    probe = torch.empty(4 << 30, dtype=torch.uint8, device="cuda").fill_(0x3c)
    probe_ms = P.hbm_read_probe(probe, iters=10)
    stream_gbps = probe.numel() / probe_ms / 1e6
    del probe
    distinct = len(set(next(iter(streams.values())))) if streams else None
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_oracle_baseline(w, W, prompt, torch)

    out = {
        "metric": "committed tokens/sec at batch 1 (PPSD decode on one GPU; fastest of the PPSD schedules, named in config.mode)",
        "value": r["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_generation"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_layers}-layer d={w.d_model} decoder ({w.dtype}), exit layer "
                               f"{w.exit_layer}, prompt {w.prompt_len}, decode {n} tokens, batch 1, damp {w.damp}, "
                               f"exit head {w.exit_head}" + (f" behind a transformer layer (damp {w.exit_block_damp})"
                                                              if w.exit_block else ""),
                   "mode": main_mode + (f" ({n_stages} stages of {w.exit_layer} layers, one stream per stage up to 4)"
                                        if main_mode == "pipeline" else " (draft stage + verify stage on two streams)"
                                        if main_mode == "overlap" else ""),
                   "engine": args.engine, "tokens_per_step": n,
                   **({"temperature": args.temperature, "sample_seed": args.sample_seed,
                       "verification": "stochastic (Eq. 2)"} if args.temperature > 0 else {})},
        "acceptance_rate": alpha,
        "ms_per_token": r["ms_per_token"],
        "modes": {k: {"tokens_per_s": v["tokens_per_s"], "ms_per_token": v["ms_per_token"],
                      "steps_draft_only": v["stats"]["steps_draft_only"], "accepted": v["stats"]["accepted"],
                      "rejected": v["stats"]["rejected"], "device_ms": v["stats"]["device_ms"],
                      **({"stages": n_stages, "ticks": v["stats"]["pipeline_ticks"], "stage_runs": v["stats"]["stage_runs"],
                          "flushed_tokens": v["stats"]["flushed_tokens"]} if k == "pipeline" else {}),
                      **({"gamma": args.gamma or 3, "rounds": v["stats"]["eesd_rounds"],
                          "tokens_per_round": v["stats"]["committed"] / max(1, v["stats"]["eesd_rounds"]),
                          "speedup_vs_vanilla_gpu": (v["tokens_per_s"] / res["vanilla"]["tokens_per_s"]) if "vanilla" in res else None,
                          "leading_tokens_equal_to_the_other_modes": v.get("tokens_equal_to_vanilla_stream"),
                          "note": "draft-then-verify early-exit speculative decoding (Sec. 3.1), not PPSD"}
                         if k == "eesd" else {})}
                  for k, v in res.items()},
        "speedup_vs_vanilla_gpu": (r["tokens_per_s"] / res["vanilla"]["tokens_per_s"]) if "vanilla" in res else None,
        "bytes_per_token": {"vanilla": ab["vanilla"], "ppsd_accept_step": ab["accept_step"],
                            "ppsd_extra_per_reject": ab["reject_extra"]},
        "hbm_frac_per_committed_token": r["tokens_per_s"] * ab["vanilla"] / (HBM_PEAK_GBPS * 1e9),
        "hbm_frac_vanilla": (res["vanilla"]["tokens_per_s"] * ab["vanilla"] / (HBM_PEAK_GBPS * 1e9))
        if "vanilla" in res else None,
        "hbm_stream_read_ceiling_gbps": stream_gbps,
        "frac_of_stream_read_ceiling_per_moved_byte": moved_per_token and r["tokens_per_s"] * moved_per_token / (stream_gbps * 1e9),
        "distinct_tokens_in_stream": distinct,
        "ms_per_generation_min": r["ms_per_generation_min"], "ms_per_generation_median": r["ms_per_generation_median"],
        "hbm_frac_per_moved_byte": moved_per_token and r["tokens_per_s"] * moved_per_token / (HBM_PEAK_GBPS * 1e9),
        "prefill": {"ms": r["prefill_ms"], "tokens_per_s": w.prompt_len / r["prefill_ms"] * 1e3,
                    "path": "looped decode kernels" if args.prefill_loop else "MFMA GEMMs and attention over chunks of up to 4096 positions (when eligible)"},
        "roofline": roofline, "kernels": ktimes, "cpu_baseline": cpu,
        "weight_generation_s": gen_s,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
