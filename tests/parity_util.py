"""Teacher-forced comparison of the HIP path (through the C ABI) with the CPU oracle."""
from __future__ import annotations

import sys

import numpy as np

import workloads as wl
from oracle import binding as ob

# max-abs logit tolerance: fp32 models 1e-4, bf16 models 2e-2
TOL = {wl.DTYPE_FP32: 1e-4, wl.DTYPE_BF16: 2e-2}


def say(msg: str) -> None:
    print(msg, flush=True)
    sys.stdout.flush()


def compare_run(spark, shape, sched, weights, prompts, offsets, n_steps, forced_seed=2,
                check_kv_every=0, chunk=1, oracle_kind="f32", label="", kv_round_bf16=None,
                text_budgets=None):
    """Run len(prompts) sequences for n_steps teacher-forced steps on both sides.

    chunk > 1 uses spark_decode with that many steps per call.  text_budgets: per sequence, the
    number of text tokens after which it generates speech only (0: none).  Returns a dict of what
    was seen.
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
    sids = [spark.seq_open(off) for off in offsets]
    forced = np.stack([wl.make_forced_stream(shape, n_steps, sched.n_text, sched.n_speech, off,
                                             seed=forced_seed + 17 * b)
                       for b, off in enumerate(offsets)], axis=1)          # [n_steps, B]
    for b in range(B):
        assert oseqs[b].prefill(prompts[b]) == 0
        spark.prefill(sids[b], prompts[b])
        if text_budgets is not None and text_budgets[b] > 0:
            assert oseqs[b].text_budget(text_budgets[b]) == 0
            spark.seq_text_budget(sids[b], text_budgets[b])
    worst, near_ties, depths = 0.0, [], []
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
            for b in range(B):
                rc, otok, odep, ologits = oseqs[b].step(forced_next=int(forced[step + s, b]))
                assert rc == 0
                assert dep[s, b] == odep, (label, step + s, b, dep[s, b], odep)
                if last:   # logits of the latest position are readable
                    glogits, head = spark.get_logits(sids[b])
                    assert head == odep
                    err = float(np.max(np.abs(glogits.astype(np.float64) - ologits)))
                    worst = max(worst, err)
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
                            for p in range(max(0, pos_hi - 2 * sched.period_k), pos_hi + 1):
                                k1, v1 = spark.get_kv(sids[b], l, p)
                                k2, v2 = oseqs[b].kv(l, p)
                                kv_tol = tol if shape.dtype == wl.DTYPE_FP32 else 2e-2
                                assert np.max(np.abs(k1 - k2)) <= kv_tol, (label, "K", l, p)
                                assert np.max(np.abs(v1 - v2)) <= kv_tol, (label, "V", l, p)
            depths.append(dep[s].copy())
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
    for t in near_ties:
        say(f"  near tie {label}: step {t[0]} seq {t[1]} oracle {t[2]} gpu {t[3]} gap {t[4]:.3g}")
    say(f"  {label}: {n_steps} steps x {B} seq, worst |dlogit| {worst:.3g} (tol {tol}), "
        f"{len(near_ties)} near ties")
    return {"worst": worst, "near_ties": near_ties, "depths": np.array(depths), "stats": stats}
