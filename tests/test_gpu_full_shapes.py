"""GPU parity at the full model shapes of the two benchmark backbones, in the launch configuration
bench.py times (batch 1, 64-token KV pages), on shortened runs the oracle finishes in about a
minute: 32-token prompt, then a few interleave cycles teacher-forced; and one 200-token prompt."""
import time

import numpy as np
import pytest

import workloads as wl
from parity_util import compare_run, say

pytestmark = pytest.mark.gpu


def sampled_draws_match(sp, w, prompt, offset, n_steps=12, temperature=0.7, top_p=0.9):
    """temperature / nucleus sampling (Sec. V-A "Models") over the whole 158k-entry vocabulary,
    free running: each drawn token against the oracle's sampler on the GPU's logits of that step"""
    from oracle import binding as ob
    T, P = float(np.float32(temperature)), float(np.float32(top_p))
    rng = np.random.default_rng(21)
    sid = sp.seq_open(offset)
    sp.prefill(sid, prompt)
    sp.set_sampling(temperature, top_p)
    sizes, moved, crowd = [], 0, []
    for s in range(n_steps):
        omega = int(rng.integers(0, 2 ** 64, dtype=np.uint64))
        tok, _ = sp.decode_sampled(1, [sid], [omega])
        lg, _ = sp.get_logits(sid)
        otok, n, gap = ob.sample(lg, T, P, omega)
        sizes.append(n)
        moved += int(tok[0, 0] != int(np.argmax(lg)))
        # how many masses lie within 1/64 (relative) below the nucleus' last one
        m = np.sort(np.exp((lg.astype(np.float64) - float(lg.max())) / T))[::-1]
        crowd.append(int(np.sum((m <= m[n - 1]) & (m > m[n - 1] * (1 - 1 / 64)))))
        assert tok[0, 0] == otok or gap <= 4 * 2.0 ** -32, (s, int(tok[0, 0]), otok, gap)
    say(f"  sampled T={temperature}: {n_steps} draws, nucleus sizes {min(sizes)}..{max(sizes)}, {moved} away from "
        f"the arg-max, {min(crowd)}..{max(crowd)} masses within 1/64 below the nucleus' edge")
    assert moved > 0
    sp.set_sampling(0.0, 0.0)
    sp.seq_close(sid)


@pytest.mark.parametrize("name,n_steps,offset,n_prompt", [
    ("step_audio_2_mini", 36, 0, 32),    # 3 * (1 + 2) * 4 steps: flushes of 1, 2 and 3 rows
    ("glm_4_voice", 24, 10, 32),         # enters the cycle 3 text slots before a 26-slot speech chunk
    # a prompt longer than one pass of the prompt path (192 rows at this shape: three tiles of 64
    # rows on the MFMA units, then a ragged pass), and a context of several attention slices
    ("step_audio_2_mini", 8, 1, 200),
])
def test_full_shape_short_run(name, n_steps, offset, n_prompt):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_09215_amd import binding as sb
    w = wl.WORKLOADS[name]
    say(f"case full shape {name}: drawing weights")
    t0 = time.time()
    dev_w = wl.make_weights_on_device(w.shape, seed=0)
    host_w = wl.device_weights_to_host(dev_w)
    say(f"  weights on device and host in {time.time() - t0:.1f}s")
    sp = sb.Spark(w.shape, w.schedule, dev_w, max_batch=1, max_seq_len=n_prompt + 96, kv_page_tokens=64)
    prompt = wl.make_prompt(w.shape, n_prompt, seed=1, ids=w.prompt_ids)
    t0 = time.time()
    # Reference: the oracle's fp64 twin.  Its fp32 build sums 3584..18944-term dot products
    # sequentially, which leaves ~sqrt(n) * 2^-24 relative noise in K and V; re-rounding those to
    # bf16 for the cache turns that noise into rounding flips that eat most of the 2e-2 budget
    # (measured 0.018 / 0.022 on these two shapes), so the GPU's own error is measured against
    # the twin whose noise is negligible.
    res = compare_run(sp, w.shape, w.schedule, host_w, [prompt], [offset], n_steps,
                      check_kv_every=0, label=name, oracle_kind="f64")
    say(f"  compared in {time.time() - t0:.1f}s")
    depths = res["depths"][:, 0]
    assert set(np.unique(depths)) <= {w.schedule.exit_layer, w.shape.n_layers}
    assert n_steps < 12 or len(np.unique(depths)) == 2
    if name == "step_audio_2_mini" and n_prompt == 32:
        sampled_draws_match(sp, w, prompt, offset)
        # a flat distribution: tens of thousands of masses within 1/64 of each other, more than
        # the sampler's candidate list holds, so its general path decides
        sampled_draws_match(sp, w, prompt, offset, n_steps=6, temperature=5.0, top_p=0.9)
    sp.close()
    del dev_w, host_w
    torch.cuda.empty_cache()


def test_bench_configuration_properties():
    """The configuration bench.py times (Step-Audio-2-mini shape, 512-token prompt, 1024 decoded
    tokens in multi-step calls, 64-token pages, free running): too long for the oracle's model, so
    what holds at any size is checked: the depth of every step against the oracle's scheduler, the
    counters, the two validity frontiers of the cache, and that a second, identical run reproduces
    the tokens bit for bit (nothing in the path depends on timing or on atomics' order)."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import binding as ob
    from paper_2603_09215_amd import binding as sb
    w = wl.WORKLOADS["step_audio_2_mini"]
    say("case bench configuration")
    dev_w = wl.make_weights_on_device(w.shape, seed=0)
    n = w.decode_len
    want_depth, want_text = ob.schedule_run(w.shape, w.schedule, n, 0)
    prompt = wl.make_prompt(w.shape, w.prompt_len, seed=1, ids=w.prompt_ids)
    runs = []
    for rep in range(2):
        sp = sb.Spark(w.shape, w.schedule, dev_w, max_batch=1, max_seq_len=w.prompt_len + n + 64, kv_page_tokens=64)
        sid = sp.seq_open(0)
        sp.prefill(sid, prompt)
        tok, dep = sp.decode(n, [sid])
        assert np.array_equal(dep[:, 0], want_depth)
        assert tok.min() >= 0 and tok.max() < w.shape.vocab
        st = sp.get_stats(sid)
        assert st["text"] == int(want_text.sum())
        assert st["speech_full"] == int(((want_text == 0) & (want_depth == w.shape.n_layers)).sum())
        assert st["speech_ee"] == int((want_depth != w.shape.n_layers).sum())
        state = sp.seq_state(sid)
        trailing_ee = 0
        while want_depth[n - 1 - trailing_ee] != w.shape.n_layers:
            trailing_ee += 1
        assert state["len"] == w.prompt_len - 1 + n and state["pending"] == trailing_ee
        assert state["upper_valid"] == state["len"] - trailing_ee
        logits, head = sp.get_logits(sid)
        assert np.all(np.isfinite(logits)) and int(np.argmax(logits)) == tok[-1, 0]
        runs.append(tok.copy())
        sp.close()
    assert np.array_equal(runs[0], runs[1])
    del dev_w
    torch.cuda.empty_cache()


def test_batched_bench_configuration_properties():
    """bench.py --batch at the Step-Audio-2-mini shape (prompts of 256..2048 tokens, mixed cycle
    offsets, MFMA projections and attention with several pieces per workgroup): every sequence's
    depths against the oracle's scheduler, and a second run reproduces the tokens bit for bit"""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import binding as ob
    from paper_2603_09215_amd import binding as sb
    w = wl.WORKLOADS["step_audio_2_mini"]
    say("case batched bench configuration")
    dev_w = wl.make_weights_on_device(w.shape, seed=0)
    B, n = 12, 48
    cyc = w.schedule.n_text + w.schedule.n_speech
    plens = [int(x) for x in wl.make_prompt_lengths(B, 256, 2048, seed=3)]
    prompts = [wl.make_prompt(w.shape, p, seed=1 + i, ids=w.prompt_ids) for i, p in enumerate(plens)]
    runs = []
    for rep in range(2):
        sp = sb.Spark(w.shape, w.schedule, dev_w, max_batch=B, max_seq_len=2048 + n + 64, kv_page_tokens=64)
        sids = [sp.seq_open(i % cyc) for i in range(B)]
        for s_, p_ in zip(sids, prompts):
            sp.prefill(s_, p_)
        tok, dep = sp.decode(n, sids)
        for i in range(B):
            want_depth, _ = ob.schedule_run(w.shape, w.schedule, n, i % cyc)
            assert np.array_equal(dep[:, i], want_depth), i
            assert sp.seq_state(sids[i])["len"] == plens[i] - 1 + n
        assert tok.min() >= 0 and tok.max() < w.shape.vocab
        runs.append(tok.copy())
        sp.close()
    assert np.array_equal(runs[0], runs[1])
    del dev_w
    torch.cuda.empty_cache()
