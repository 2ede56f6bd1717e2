#!/usr/bin/env python3
"""Benchmark of the SPAR-K decode hot path on one MI355X.

A "step" is one decoding step (one generated token) of the whole path: schedule/dispatch, layers
1..e on the new position, then either the layer-specific head (early exit) or the batched pass of
pending rows through layers e+1..L and the final head.  Default workload: the Step-Audio-2-mini
shape of the paper's Sec. V-A (28 layers), bf16, random-init weights, batch 1, 512-token prompt,
interleave 1 text : 2 speech, exit layer 20, refresh period 4.

Prints ONE JSON line: decode tokens/s with the weights, KV cache and prompt resident in HBM, the
HBM roofline of the dominant kernel (the gate/up projection) from HIP events recorded on the
library's stream, and the CPU oracle timed on the host cores as a reported baseline.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

import workloads as wl

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak
MFMA_BF16_PEAK_TFLOPS = 2500.0   # dense bf16


def measured_traffic(shape):
    """HBM bytes per launch of the gate/up kernel from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, scaled), if there is one for this shape; else None"""
    import pathlib
    import re
    f = pathlib.Path(__file__).resolve().parent / "profiles" / f"gateup_gemv_{shape.name}_hbm_traffic.txt"
    if not f.exists():
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*(\d+)", f.read_text(), flags=re.M)
    return int(m.group(1)) if m else None


def step_bytes(shape, sched, ctx_len: float):
    """algorithmic HBM bytes of one early-exit step and one full-depth step at context length T:
    each needed weight matrix once, plus the KV of the layers that run"""
    esz = 2 if shape.dtype == wl.DTYPE_BF16 else 4
    d, F, V = shape.d_model, shape.d_ffn, shape.vocab
    q, kv = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    w_layer = ((q + 2 * kv) * d + d * q + 2 * F * d + d * F) * esz
    w_head = V * d * esz
    kv_tok = 2 * kv * esz
    ee = sched.exit_layer * w_layer + d * d * esz + w_head + sched.exit_layer * ctx_len * kv_tok
    full = shape.n_layers * w_layer + w_head + shape.n_layers * ctx_len * kv_tok
    return ee, full, w_layer


def short_leg(Spark, torch, name, dev_w, batch, aligned, steps, warmup, prompt_len=None):
    """a short decode of another benchmark configuration, so that its rate is part of the same
    record: `steps` timed steps after `warmup`, inputs resident, same conventions as the headline"""
    w = wl.WORKLOADS[name]
    shape, sched = w.shape, w.schedule
    if batch > 1:
        plens = [int(x) for x in wl.make_prompt_lengths(batch, 256, 2048, seed=3)]
    else:
        plens = [prompt_len or w.prompt_len]
    max_seq = min(16384, (max(plens) + warmup + steps + 64 + 63) // 64 * 64)
    sp = Spark(shape, sched, dev_w, max_batch=batch, max_seq_len=max_seq, kv_page_tokens=64, device="cuda:0")
    cyc = sched.n_text + sched.n_speech
    sids = [sp.seq_open(i % cyc if batch > 1 and not aligned else 0) for i in range(batch)]
    t0 = time.perf_counter()
    for i, (s_, n) in enumerate(zip(sids, plens)):
        sp.prefill(s_, wl.make_prompt(shape, n, seed=1 + i, ids=w.prompt_ids))
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    sp.decode(warmup, sids)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    tok, dep = sp.decode(steps, sids)
    torch.cuda.synchronize()
    el = time.perf_counter() - t1
    esz = 2 if shape.dtype == wl.DTYPE_BF16 else 4
    ctx = float(np.mean(plens)) + warmup + steps / 2
    ee_b, full_b, w_layer = step_bytes(shape, sched, ctx)
    head_b = shape.vocab * shape.d_model * esz
    any_full = int((dep == shape.n_layers).any(axis=1).sum())
    any_ee = int((dep != shape.n_layers).any(axis=1).sum())
    kv_b = (sched.exit_layer * steps + (shape.n_layers - sched.exit_layer) * any_full) * \
        sum(plens) * 2 * shape.n_kv_heads * shape.head_dim * esz / steps
    avg_bytes = (steps * sched.exit_layer * w_layer + any_full * ((shape.n_layers - sched.exit_layer) * w_layer + head_b)
                 + any_ee * (head_b + shape.d_model ** 2 * esz)) / steps + kv_b
    out = {"workload": f"{name}, batch {batch}, prompts {plens[0] if batch == 1 else '256..2048'}, "
                       f"{'aligned' if aligned and batch > 1 else 'mixed' if batch > 1 else 'single'} cycle offsets, "
                       f"e={sched.exit_layer}, K={sched.period_k}",
           "steps": steps, "warmup": warmup, "tokens_per_s": round(steps * batch / el, 1),
           "ms_per_step": round(el * 1e3 / steps, 4), "prefill_tokens_per_s": round(sum(n - 1 for n in plens) / prefill_s, 1),
           "steps_with_a_full_depth_row": any_full, "steps_with_an_early_exit_row": any_ee,
           "algorithmic_GB_per_step": round(avg_bytes / 1e9, 3),
           "frac_of_hbm_peak": round(avg_bytes / (el / steps) / 1e9 / HBM_PEAK_GBS, 4)}
    sp.close()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1024)
    ap.add_argument("--warmup", type=int, default=36)
    ap.add_argument("--workload", default="step_audio_2_mini", choices=sorted(wl.WORKLOADS))
    ap.add_argument("--prompt-len", type=int, default=None)
    ap.add_argument("--cpu-steps", type=int, default=16, help="oracle steps timed for cpu_baseline (0 = skip)")
    ap.add_argument("--other-configs", type=int, default=1,
                    help="1 (default, headline workload only): after the headline measurement also time short legs "
                         "of the GLM-4-Voice shape at batch 1 and of batch 32 at the Step-Audio-2-mini shape "
                         "(mixed and aligned cycle offsets); 0 = skip")
    ap.add_argument("--profile-steps", type=int, default=48)
    ap.add_argument("--batch", type=int, default=1,
                    help="sequences decoded together (default 1: the headline workload); >1 gives "
                         "random prompt lengths in 256..2048 and mixed cycle offsets")
    ap.add_argument("--exit-layer", type=int, default=None, help="override the workload's exit layer e")
    ap.add_argument("--period", type=int, default=None, help="override the refresh period K (phase becomes K-1)")
    ap.add_argument("--text-period", type=int, default=None,
                    help="apply the periodic rule to text positions too, with this period and phase 0")
    ap.add_argument("--aligned", action="store_true",
                    help="batch > 1: every sequence starts at cycle offset 0 (phase-aligned schedules)")
    ap.add_argument("--speech-share", type=float, default=0.0,
                    help="e.g. 0.795: the text ends early, so that this share of the warm-up + timed tokens is "
                         "speech (the interleave alone gives n_speech / (n_text + n_speech))")
    ap.add_argument("--align-phases", action="store_true",
                    help="batch > 1 with --speech-share: once every sequence is in its speech tail (after the "
                         "warm-up), move the phases so that the full-depth steps of the batch coincide")
    ap.add_argument("--temperature", type=float, default=0.0,
                    help="> 0: draw tokens by temperature / nucleus sampling instead of the arg-max")
    ap.add_argument("--top-p", type=float, default=0.9)
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE",
                    help="a kernel-selection switch of the library (spark_tune), for A/B measurements")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (no collectives, no "
              "sharding across devices are part of it)", file=sys.stderr)
        return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    from paper_2603_09215_amd import Spark

    w = wl.WORKLOADS[args.workload]
    shape, sched = w.shape, w.schedule
    if args.exit_layer is not None:
        sched = dataclasses.replace(sched, exit_layer=args.exit_layer)
    if args.period is not None:
        sched = dataclasses.replace(sched, period_k=args.period, phase=args.period - 1)
    if args.text_period is not None:
        sched = dataclasses.replace(sched, text_period_k=args.text_period, text_phase=0)
    prompt_len = args.prompt_len or w.prompt_len
    K, W = args.steps, args.warmup
    device = torch.device("cuda:0")
    max_seq = prompt_len + W + K + 4 * args.profile_steps + 64
    max_seq = min(16384, (max_seq + 63) // 64 * 64)

    t0 = time.time()
    if shape.dtype == wl.DTYPE_BF16:
        dev_w = wl.make_weights_on_device(shape, seed=0, device="cuda:0")
    else:
        dev_w = wl.make_weights(shape, seed=0)
    B = args.batch
    if B > 1:
        plens = [args.prompt_len] * B if args.prompt_len else \
            [int(x) for x in wl.make_prompt_lengths(B, 256, 2048, seed=3)]
        max_seq = min(16384, (max(plens) + W + K + 4 * args.profile_steps + 64 + 63) // 64 * 64)
    else:
        plens = [prompt_len]
    sp = Spark(shape, sched, dev_w, max_batch=B, max_seq_len=max_seq, kv_page_tokens=64, device="cuda:0")
    for t in args.tune:
        name, value = t.split("=")
        sp.tune(name, int(value))
    cyc = sched.n_text + sched.n_speech
    sids = [sp.seq_open(i % cyc if B > 1 and not args.aligned else 0) for i in range(B)]
    prompts = [wl.make_prompt(shape, n, seed=1 + i, ids=w.prompt_ids) for i, n in enumerate(plens)]
    prompt = prompts[0]
    sid = sids[0]
    torch.cuda.synchronize()
    tp0 = time.perf_counter()
    for s_, p_ in zip(sids, prompts):
        sp.prefill(s_, p_)
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - tp0
    print(f"[bench] weights + prefill({sum(plens)} tokens) ready in {time.time() - t0:.1f}s "
          f"(prefill {prefill_s * 1e3:.1f} ms)", file=sys.stderr, flush=True)
    # useful flops of the prompt pass: 2 per weight element and row, plus causal attention
    esz_ = 2 if shape.dtype == wl.DTYPE_BF16 else 4
    qd = shape.n_q_heads * shape.head_dim
    kvd = shape.n_kv_heads * shape.head_dim
    w_elems_layer = (qd + 2 * kvd) * shape.d_model + shape.d_model * qd + 3 * shape.d_ffn * shape.d_model
    pre_rows = sum(n - 1 for n in plens)
    pre_flops = 2.0 * w_elems_layer * shape.n_layers * pre_rows + \
        sum(2.0 * (n - 1) ** 2 * qd * shape.n_layers for n in plens)
    prefill = {"tokens": pre_rows, "ms": round(prefill_s * 1e3, 2),
               "tokens_per_s": round(pre_rows / prefill_s, 1),
               "useful_TFLOPs": round(pre_flops / prefill_s / 1e12, 2),
               "frac_of_mfma_bf16_peak": round(pre_flops / prefill_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}

    # ---- warm-up, then the timed region: exactly K steps, tokens fed back on the device
    text_budget = 0
    if args.speech_share > 0:
        text_budget = max(1, round((1.0 - args.speech_share) * (W + K)))
        for i_, s_ in enumerate(sids):   # a batch: the responses' texts differ in length (+- a third, seeded)
            sp.seq_text_budget(s_, text_budget if B == 1 else max(1, round(text_budget * (2 / 3 + 2 / 3 * i_ / (B - 1)))))
    sampled = args.temperature > 0
    if sampled:   # one 64-bit random word per step and sequence, drawn ahead of the timed region
        sp.set_sampling(args.temperature, args.top_p)
        words = np.random.Generator(np.random.Philox(7)).integers(0, 2 ** 64, size=(K + W, B), dtype=np.uint64)
        decode = lambda n, first: sp.decode_sampled(n, sids, words[first:first + n])
    else:
        decode = lambda n, first: sp.decode(n, sids)
    decode(W, 0)
    if args.align_phases:
        sp.align_phases(sids)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    tok, dep = decode(K, W)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    ms_per_step = elapsed * 1e3 / K
    value = K * B / elapsed

    # ---- per-class step times (one synchronous spark_step per token), same sequence continues
    # classes: early exit, full depth with m rows in the pass (m - 1 pending positions completed)
    n_cls = min(2 * args.profile_steps, 96)
    cls = {}
    ctx_now = prompt_len - 1 + W + K
    pending = sp.seq_state(sid)["pending"] if B == 1 else 0
    for i in range(n_cls if B == 1 else 0):
        torch.cuda.synchronize()
        a = time.perf_counter()
        t_, d_ = sp.step([sid])
        b = time.perf_counter()
        if d_[0] != shape.n_layers:
            cls.setdefault("ee", []).append((b - a) * 1e3)
        else:
            cls.setdefault("full", []).append((b - a) * 1e3)
            cls.setdefault(f"full_m{pending + 1}", []).append((b - a) * 1e3)
        pending = sp.seq_state(sid)["pending"]
    ee_b, full_b, w_layer = step_bytes(shape, sched, ctx_now + n_cls / 2)
    classes = {}
    for key, ts in cls.items():
        med = float(np.median(ts))
        by = ee_b if key == "ee" else full_b
        classes[key] = {"ms": round(med, 4), "steps": len(ts), "algorithmic_GB": round(by / 1e9, 3),
                        "GBps": round(by / med / 1e6, 1), "frac_of_hbm_peak": round(by / med / 1e6 / HBM_PEAK_GBS, 4)}

    # ---- roofline of the dominant kernel: gate/up projection, HIP events on the library's stream
    esz = 2 if shape.dtype == wl.DTYPE_BF16 else 4
    gateup_bytes = 2 * shape.d_ffn * shape.d_model * esz
    sp.profile_select("gateup")
    if args.profile_steps > 0:
        sp.decode(args.profile_steps, sids)
    n_launch, tot_ms, empty_ms = sp.profile_read()
    sp.profile_select(-1)
    # the launch duration is the whole event bracket (it includes the bracket's own cost, about a
    # microsecond, so the figure errs low); the bracket net of an empty one is reported beside it
    avg_ms = tot_ms / max(1, n_launch)
    net_ms = (tot_ms - empty_ms) / max(1, n_launch)
    achieved = gateup_bytes / (avg_ms * 1e-3) / 1e9 if n_launch else 0.0
    # what a plain streaming read gets on this device, next to the published peak: all gate
    # matrices of the model (several GB, far beyond the last-level cache), non-temporal loads
    ceiling_nt, _ = sp.measure_read(sp.dev_weights["wg"], reps=4, nontemporal=True)
    ceiling_plain, _ = sp.measure_read(sp.dev_weights["wg"], reps=4, nontemporal=False)
    # the same reader over as many bytes as one gate/up launch streams (the gate matrices of two
    # layers), one launch per repetition: what a launch of that size can reach, its start and
    # drain included
    wg = sp.dev_weights["wg"]
    same_size = wg.reshape(-1)[:gateup_bytes // wg.element_size()]
    ceiling_same, _ = sp.measure_read(same_size, reps=16, nontemporal=True)
    roofline = {"bound": "hbm", "kernel": "gemv_rows_k<gate/up + SwiGLU>", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(shape),
                "traffic_source": "profiles/ (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs), not this run",
                "bytes_per_launch": gateup_bytes, "avg_launch_ms": round(avg_ms, 5),
                "avg_launch_ms_net_of_an_empty_bracket": round(net_ms, 5),
                "launches_timed": int(n_launch),
                "measured_read_ceiling_GBps": round(ceiling_nt, 1),
                "measured_read_ceiling_plain_loads_GBps": round(ceiling_plain, 1),
                "frac_of_measured_ceiling": round(achieved / max(ceiling_nt, 1e-9), 4),
                "measured_read_of_the_launch_bytes_GBps": round(ceiling_same, 1),
                "frac_of_read_of_the_launch_bytes": round(achieved / max(ceiling_same, 1e-9), 4)}

    sampler = None
    if sampled and args.profile_steps > 0:
        sp.profile_select("sample")
        decode(args.profile_steps, 0)
        n_s, ms_s, _ = sp.profile_read()
        sp.profile_select(-1)
        sampler = {"temperature": args.temperature, "top_p": args.top_p,
                   "avg_launch_ms": round(ms_s / max(1, n_s), 5), "launches_timed": int(n_s)}

    depth_all = dep[:, 0]
    mix = {"full_steps": int((depth_all == shape.n_layers).sum()), "ee_steps": int((depth_all != shape.n_layers).sum())}
    stats = sp.get_stats(sid)
    if B > 1:   # any full-depth row in a step streams the upper layers; both heads usually run
        any_full = int((dep == shape.n_layers).any(axis=1).sum())
        any_ee = int((dep != shape.n_layers).any(axis=1).sum())
        head_b = shape.vocab * shape.d_model * esz
        lower = sched.exit_layer * w_layer
        upper = (shape.n_layers - sched.exit_layer) * w_layer
        avg_bytes = (K * lower + any_full * (upper + head_b) +
                     any_ee * (head_b + shape.d_model ** 2 * esz)) / K
        mix = {"steps_with_a_full_depth_row": any_full, "steps_with_an_early_exit_row": any_ee}
    else:
        avg_bytes = (mix["full_steps"] * full_b + mix["ee_steps"] * ee_b) / K
    whole = {"algorithmic_GB_per_step": round(avg_bytes / 1e9, 3),
             "GBps": round(avg_bytes / (ms_per_step * 1e-3) / 1e9, 1),
             "frac_of_hbm_peak": round(avg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload
    cpu = None
    if args.cpu_steps > 0:
        from oracle import binding as ob
        host_w = wl.device_weights_to_host(sp.dev_weights)
        om = ob.Model(shape, sched, host_w, max_seq_len=64 + args.cpu_steps)
        osq = om.open(0)
        osq.prefill(prompt[:32])
        c0 = time.perf_counter()
        for _ in range(args.cpu_steps):
            rc, *_ = osq.step(want_logits=False)
            assert rc == 0
        cpu_s = time.perf_counter() - c0
        cpu = {"value": round(args.cpu_steps / cpu_s, 4), "unit": "tokens/s", "cores": ob.num_threads(),
               "kind": "oracle",
               "sample": f"{args.cpu_steps} decode steps after a 32-token prompt, same shape, weights and schedule"}
        osq.close(); om.close()

    if "ee" in classes and "full" in classes:
        classes["ee_over_full"] = {"measured": round(classes["ee"]["ms"] / classes["full"]["ms"], 4),
                                   "from_bytes": round(ee_b / full_b, 4)}
    line = {
        "metric": f"decode tokens/s per GPU (batch {B})", "value": round(value, 2), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == wl.DTYPE_BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"{shape.name}: L={shape.n_layers} d={shape.d_model} "
                               f"{shape.n_q_heads}q/{shape.n_kv_heads}kv hd={shape.head_dim} F={shape.d_ffn} "
                               f"V={shape.vocab}; prompt {prompt_len if B == 1 or args.prompt_len else '256..2048'}, decode {K}, batch {B}, "
                               f"{sched.n_text}:{sched.n_speech} text:speech, e={sched.exit_layer}, "
                               f"K={sched.period_k}, phase={sched.phase}, "
                               f"{'K_text=' + str(sched.text_period_k) + ', ' if sched.text_period_k > 1 else ''}"
                               f"scope={'chunk' if sched.scope == 0 else 'stream'}"
                               f"{', cycle offsets aligned' if args.aligned and B > 1 else ''}"
                               f"{f', text ends after {text_budget} tokens (speech share {args.speech_share})' if text_budget else ''}"
                               f"{', phases aligned after the warm-up' if args.align_phases else ''}"
                               f"{f', sampled T={args.temperature} top_p={args.top_p}' if sampled else ', greedy'}",
                   "weights": "random N(0,0.02), fp32 accumulation", "kv_cache": "paged, 64 tokens/page",
                   "step_mix": mix, "mean_speech_depth": stats["mean_speech_depth"],
                   "speech_layer_saving_pct": round(stats["speech_layer_saving"], 2),
                   "prefill": prefill},
        "roofline": roofline, "whole_step": whole, "step_classes": classes, "cpu_baseline": cpu,
    }
    if sampler:
        line["sampler"] = sampler
    sp.close()
    # ---- the other benchmark configurations, short legs (outside the headline's timed region)
    default_run = (args.workload == "step_audio_2_mini" and B == 1 and not sampled and args.exit_layer is None
                   and args.period is None and args.text_period is None and not args.speech_share)
    if args.other_configs and default_run:
        others = {}
        others["batch32_mixed"] = short_leg(Spark, torch, "step_audio_2_mini", dev_w, 32, False, 48, 16)
        others["batch32_aligned"] = short_leg(Spark, torch, "step_audio_2_mini", dev_w, 32, True, 48, 16)
        del dev_w
        torch.cuda.empty_cache()
        glm_w = wl.make_weights_on_device(wl.WORKLOADS["glm_4_voice"].shape, seed=0, device="cuda:0")
        others["glm_4_voice_batch1"] = short_leg(Spark, torch, "glm_4_voice", glm_w, 1, False, 78, 39)
        line["other_configs"] = others
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
