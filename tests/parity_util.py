"""Teacher-forced comparison of the HIP path (through the C ABI) with the CPU oracle."""
from __future__ import annotations

import pathlib
import sys
import time

import numpy as np

import workloads as wl
from oracle import binding as ob

# max-abs logit tolerance: fp32 models 1e-4, bf16 models 2e-2
TOL = {wl.DTYPE_FP32: 1e-4, wl.DTYPE_BF16: 2e-2}


def kv_tolerance(shape, want):
    """element-wise bound for a cached key / value entry.  fp32 caches: the logit tolerance.  bf16
    caches: both sides round the entry to bf16 when they store it, so where their fp32 / fp64 values
    straddle a rounding boundary the stored entries differ by one unit in the last place, 2^-7 of
    the value (0.031 for an entry of magnitude 4); on top of that the logit tolerance, which bounds
    what the layers below may have moved the unrounded value by."""
    if shape.dtype == wl.DTYPE_FP32:
        return TOL[wl.DTYPE_FP32]
    return TOL[wl.DTYPE_BF16] + 2.0 ** -7 * np.abs(want)


_PROGRESS = pathlib.Path(__file__).resolve().parent.parent / "gpurun_out" / "test_progress.log"


def say(msg: str) -> None:
    """progress of a long case: to stdout, and appended to a log file that a harness watching for
    signs of life can see while pytest holds stdout back"""
    print(msg, flush=True)
    sys.stdout.flush()
    try:
        _PROGRESS.parent.mkdir(exist_ok=True)
        with open(_PROGRESS, "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass


_cache: dict = {}


def full_weights(name):
    """(device, host) copies of one benchmark backbone's weights, drawn once per test session (both
    backbones together are 37 GB on either side).  Gains are drawn away from 1 so that a wrong or
    missing gain shows."""
    import torch
    if name not in _cache:
        w = wl.WORKLOADS[name]
        t0 = time.time()
        dev_w = wl.make_weights_on_device(w.shape, seed=0)
        g = torch.Generator(device="cuda:0")
        g.manual_seed(5)
        for k in wl.GAIN_TENSORS:
            dev_w[k] = 1.0 + 0.1 * torch.randn(dev_w[k].shape, generator=g, dtype=torch.float32, device="cuda:0")
        host_w = wl.device_weights_to_host(dev_w)
        say(f"  {name}: weights on device and host in {time.time() - t0:.1f}s")
        _cache[name] = (dev_w, host_w)
    return _cache[name]


def release_full_weights():
    import torch
    _cache.clear()
    if torch.cuda.is_available():
        torch.cuda.empty_cache()


def compare_run(spark, shape, sched, weights, prompts, offsets, n_steps, forced_seed=2,
                check_kv_every=0, chunk=1, oracle_kind="f32", label="", kv_round_bf16=None,
                text_budgets=None, beside_f32_steps=0, trace_steps=False, kv_all_positions=False):
    """Run len(prompts) sequences for n_steps teacher-forced steps on both sides.

    chunk > 1 uses spark_decode with that many steps per call.  text_budgets: per sequence, the
    number of text tokens after which it generates speech only (0: none).  Returns a dict of what
    was seen.
    beside_f32_steps > 0 (with oracle_kind="f64"): the oracle's fp32 build runs the same stream next
    to its fp64 twin for that many steps, and the three distances GPU-f64, GPU-f32 and f32-f64 are
    logged; only GPU-f64 is asserted.  trace_steps logs the worst distance of every step.
    kv_all_positions: the cache check covers every position of the sequence instead of the last
    2K + 1 (for short contexts).
    Asserts: depths bit-exact; logits within tolerance of the oracle's; tokens equal except at
    logged near-ties (oracle gap between its own argmax and the GPU's token <= 2 * tol)."""
    tol = TOL[shape.dtype]
    B = len(prompts)
    max_len = max(len(p) for p in prompts) + n_steps + 1
    if kv_round_bf16 is None:     # the KV cache of a bf16 model stores bf16 on both sides
        kv_round_bf16 = shape.dtype == wl.DTYPE_BF16
    om = ob.Model(shape, sched, weights, max_seq_len=max_len, kind=oracle_kind,
                  kv_round_bf16=kv_round_bf16)
    oseqs = [om.open(off) for off in offsets]
    om32 = oseqs32 = None
    if beside_f32_steps > 0:
        assert oracle_kind == "f64"
        om32 = ob.Model(shape, sched, weights, max_seq_len=max_len, kind="f32", kv_round_bf16=kv_round_bf16)
        oseqs32 = [om32.open(off) for off in offsets]
    sids = [spark.seq_open(off) for off in offsets]
    forced = np.stack([wl.make_forced_stream(shape, n_steps, sched.n_text, sched.n_speech, off,
                                             seed=forced_seed + 17 * b)
                       for b, off in enumerate(offsets)], axis=1)          # [n_steps, B]
    for b in range(B):
        assert oseqs[b].prefill(prompts[b]) == 0
        if oseqs32:
            assert oseqs32[b].prefill(prompts[b]) == 0
        spark.prefill(sids[b], prompts[b])
        if text_budgets is not None and text_budgets[b] > 0:
            assert oseqs[b].text_budget(text_budgets[b]) == 0
            spark.seq_text_budget(sids[b], text_budgets[b])
    worst, near_ties, depths = 0.0, [], []
    worst_g32 = worst_32_64 = 0.0
    step = 0
    while step < n_steps:
        k = min(chunk, n_steps - step)
        if k == 1:
            tok, dep = spark.step(sids, forced[step])
            tok, dep = tok[None], dep[None]
        else:
            tok, dep = spark.decode(k, sids, forced[step:step + k])
        for s in range(k):
            last = s == k - 1
            step_worst = 0.0
            for b in range(B):
                rc, otok, odep, ologits = oseqs[b].step(forced_next=int(forced[step + s, b]))
                assert rc == 0
                assert dep[s, b] == odep, (label, step + s, b, dep[s, b], odep)
                if last:   # logits of the latest position are readable
                    glogits, head = spark.get_logits(sids[b])
                    assert head == odep
                    err = float(np.max(np.abs(glogits.astype(np.float64) - ologits)))
                    worst = max(worst, err)
                    step_worst = max(step_worst, err)
                    if oseqs32 and step + s < beside_f32_steps:
                        rc32, _, dep32, lg32 = oseqs32[b].step(forced_next=int(forced[step + s, b]))
                        assert rc32 == 0 and dep32 == odep
                        worst_g32 = max(worst_g32, float(np.max(np.abs(glogits.astype(np.float64) - lg32))))
                        worst_32_64 = max(worst_32_64, float(np.max(np.abs(lg32 - ologits))))
                    assert err <= tol, (label, step + s, b, err)
                    assert int(np.argmax(glogits)) == tok[s, b]      # fused argmax, lowest index
                if tok[s, b] != otok:
                    gap = float(ologits[otok] - ologits[tok[s, b]])
                    near_ties.append((step + s, b, int(otok), int(tok[s, b]), gap))
                    assert gap <= 2 * tol, (label, "token mismatch beyond a near tie", step + s, b, gap)
                if last:
                    st = spark.seq_state(sids[b])
                    assert st["len"] == oseqs[b].len and st["pending"] == oseqs[b].pending
                    assert st["upper_valid"] == oseqs[b].upper_valid
                    if check_kv_every and odep == shape.n_layers and (step + s) % check_kv_every == 0:
                        pos_hi = st["len"] - 1
                        for l in range(shape.n_layers):
                            for p in range(0 if kv_all_positions else max(0, pos_hi - 2 * sched.period_k), pos_hi + 1):
                                k1, v1 = spark.get_kv(sids[b], l, p)
                                k2, v2 = oseqs[b].kv(l, p)
                                for got, want, nm in ((k1, k2, "K"), (v1, v2, "V")):
                                    bad = np.abs(got - want) - kv_tolerance(shape, want)
                                    assert np.all(bad <= 0), (label, nm, l, p, float(bad.max()))
            depths.append(dep[s].copy())
            if trace_steps and last:
                say(f"    {label} step {step + s}: depth {list(map(int, dep[s]))} worst |dlogit| {step_worst:.3g}")
        step += k
    stats = []
    for b in range(B):
        gs, os_ = spark.get_stats(sids[b]), oseqs[b].stats()
        assert gs["text"] == os_["text"] and gs["speech_full"] == os_["speech_full"]
        assert gs["text_ee"] == os_["text_ee"]
        assert gs["speech_ee"] == os_["speech_ee"] and gs["flush_hist"] == os_["flush_hist"]
        stats.append(gs)
        spark.seq_close(sids[b])
        oseqs[b].close()
    om.close()
    if oseqs32:
        for q in oseqs32:
            q.close()
        om32.close()
        say(f"  {label}: first {beside_f32_steps} steps, max |dlogit|: GPU vs fp64 oracle {worst:.3g} (whole run), "
            f"GPU vs fp32 oracle {worst_g32:.3g}, fp32 oracle vs fp64 oracle {worst_32_64:.3g}")
    for t in near_ties:
        say(f"  near tie {label}: step {t[0]} seq {t[1]} oracle {t[2]} gpu {t[3]} gap {t[4]:.3g}")
    say(f"  {label}: {n_steps} steps x {B} seq, worst |dlogit| {worst:.3g} (tol {tol}), "
        f"{len(near_ties)} near ties")
    return {"worst": worst, "near_ties": near_ties, "depths": np.array(depths), "stats": stats,
            "worst_gpu_f32": worst_g32, "worst_f32_f64": worst_32_64}
