"""spark_init_static, the entry point that allocates nothing (its scratch area is a static device
array inside the library), against spark_init with a caller's scratch buffer: the same prompt and
teacher-forced stream through both contexts give bit-identical tokens, depths and logits, on two
calls in a row, the second with a smaller configuration (a smaller model and batch, so the second
context finds the first one's leftovers in the shared array); then the refusals.

A context on a caller's buffer of the full size also holds a copy of the projection weights in MFMA
operand order, which the static area has no room for; the comparison switches that copy off
("mfma_tiled" = 0), so that both contexts run the same kernels with the same k ranges and the
results can be compared bit by bit."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def run_both(sb, shape, sched, weights, n_seq, n_prompt, n_steps, seed):
    prompts = [wl.make_prompt(shape, n_prompt + 3 * b, seed=seed + b) for b in range(n_seq)]
    offsets = [b % (sched.n_text + sched.n_speech) for b in range(n_seq)]
    forced = np.stack([wl.make_forced_stream(shape, n_steps, sched.n_text, sched.n_speech, off, seed=seed + 50 + b)
                       for b, off in enumerate(offsets)], axis=1)
    results = []
    for static in (True, False):
        sp = sb.Spark(shape, sched, weights, max_batch=n_seq, max_seq_len=n_prompt + 3 * n_seq + n_steps + 8,
                      kv_page_tokens=16, static_scratch=static)
        sp.tune("mfma_tiled", 0)
        sids = [sp.seq_open(o) for o in offsets]
        for s_, p_ in zip(sids, prompts):
            sp.prefill(s_, p_)
        tok, dep = sp.decode(n_steps - 1, sids, forced[:n_steps - 1])
        t1, d1 = sp.step(sids, forced[n_steps - 1])
        logits = np.stack([sp.get_logits(s_)[0] for s_ in sids])
        kv = np.concatenate(sp.get_kv(sids[0], shape.n_layers - 1, n_prompt))
        results.append((np.vstack([tok, t1[None]]), np.vstack([dep, d1[None]]), logits, kv))
        sp.close()
    a, b = results
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.array_equal(a[2], b[2]) and np.array_equal(a[3], b[3])
    assert len(np.unique(a[1])) == 2          # both early-exit and full-depth steps ran
    return a


def test_static_scratch_context_matches_caller_scratch_context():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_09215_amd import binding as sb
    w = wl.TINY
    # first call: a bf16 model on the MFMA path with 6 sequences; second call: the small fp32 model
    # with 2 sequences, which uses a prefix of the same array
    big = w.shape.replace(name="bf16-static", dtype=wl.DTYPE_BF16, n_layers=4, d_model=512, n_q_heads=4,
                          n_kv_heads=2, head_dim=128, d_ffn=1024 + 40, vocab_text=900, vocab_speech=301)
    run_both(sb, big, w.schedule, wl.make_weights(big, seed=8, gain_std=0.1), n_seq=6, n_prompt=20, n_steps=14, seed=70)
    run_both(sb, w.shape, w.schedule, wl.make_weights(w.shape, seed=0, gain_std=0.1), n_seq=2, n_prompt=9,
             n_steps=14, seed=80)


def test_static_scratch_refusals():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_09215_amd import binding as sb
    w = wl.TINY
    weights = wl.make_weights(w.shape, seed=0)
    sp = sb.Spark(w.shape, w.schedule, weights, max_batch=1, max_seq_len=64, kv_page_tokens=16, static_scratch=True)
    with pytest.raises(sb.SparkError) as ei:      # one context per device on the static area
        sb.Spark(w.shape, w.schedule, weights, max_batch=1, max_seq_len=64, kv_page_tokens=16, static_scratch=True)
    assert ei.value.code == -4
    sp.close()
    # a configuration whose scratch need exceeds the static area: refused, nothing touched
    wide = w.shape.replace(name="too-big", vocab_text=150000, vocab_speech=8000)
    with pytest.raises(sb.SparkError) as ei:
        sb.Spark(wide, w.schedule, {k: v for k, v in weights.items()}, max_batch=64, max_seq_len=64,
                 kv_page_tokens=16, static_scratch=True)
    assert ei.value.code == -3
    sp = sb.Spark(w.shape, w.schedule, weights, max_batch=1, max_seq_len=64, kv_page_tokens=16, static_scratch=True)
    sp.close()                                     # the area is free again after both refusals
