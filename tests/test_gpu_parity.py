"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on identical seeded
weights and token streams (teacher-forced).  Depths bit-exact, logits within 1e-4 (fp32 models) /
2e-2 (bf16 models) max-abs, tokens equal except at logged near-ties."""
import numpy as np
import pytest

import workloads as wl
from parity_util import compare_run, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sb():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_09215_amd import binding
    binding.load_library()
    return binding


@pytest.fixture(scope="module")
def tiny_weights():
    return wl.make_weights(wl.TINY.shape, seed=0, gain_std=0.1)


def test_tiny_workload_full_length(sb, tiny_weights):
    """the small fp32 workload end to end: 16-token prompt, 64 generated tokens, 2:4, e=2, K=4"""
    w = wl.TINY
    say("case tiny full length")
    sp = sb.Spark(w.shape, w.schedule, tiny_weights, max_batch=1, max_seq_len=128, kv_page_tokens=16)
    prompt = wl.make_prompt(w.shape, w.prompt_len, seed=1)
    res = compare_run(sp, w.shape, w.schedule, tiny_weights, [prompt], [0], w.decode_len,
                      check_kv_every=1, label="tiny")
    st = res["stats"][0]
    assert st["text"] == 22 and st["speech_full"] == 10 and st["speech_ee"] == 32
    assert st["flush_hist"] == {1: 22, 4: 10}
    assert st["mean_speech_depth"] == pytest.approx((32 * 2 + 10 * 4) / 42)
    assert st["speech_layer_saving"] == pytest.approx((1 - st["mean_speech_depth"] / 4) * 100)
    sp.close()


def test_tiny_with_unit_gains_as_specified(sb):
    w = wl.TINY
    say("case tiny unit gains")
    weights = wl.make_weights(w.shape, seed=0, gain_std=0.0)
    sp = sb.Spark(w.shape, w.schedule, weights, max_batch=1, max_seq_len=128, kv_page_tokens=16)
    compare_run(sp, w.shape, w.schedule, weights, [wl.make_prompt(w.shape, 16, seed=1)], [0], 30,
                label="tiny gamma=1")
    sp.close()


SCHEDULES = [
    dict(period_k=2, phase=0, n_text=1, n_speech=4),                                  # Even
    dict(period_k=2, phase=1, n_text=1, n_speech=4),                                  # Odd
    dict(period_k=3, phase=0, n_text=1, n_speech=4),                                  # Triple
    dict(period_k=4, phase=3, n_text=1, n_speech=2, scope=wl.SCOPE_STREAM),
    dict(period_k=3, phase=1, n_text=0, n_speech=5, exit_layer=1),                    # joined runs
    dict(period_k=5, phase=4, n_text=2, n_speech=4, exit_layer=3),                    # fixed layer
    dict(exit_layer=4),                                                               # e = L
    dict(period_k=1, phase=0),                                                        # K = 1
    dict(period_k=8, phase=7, n_text=3, n_speech=9, scope=wl.SCOPE_STREAM, exit_layer=1),
    # the periodic rule on text positions (Sec. V-C, row G10: text Even, speech at full depth)
    dict(text_period_k=2, text_phase=0, period_k=1, phase=0, n_text=3, n_speech=2),
    # both modalities scheduled: early-exit runs cross the modality boundary (up to 5 pending rows,
    # so flushes of 5 and 6 rows take the MFMA-path row count on bf16 models, the vector tiles here)
    dict(text_period_k=3, text_phase=0, period_k=4, phase=3, n_text=3, n_speech=4),
    dict(text_period_k=3, text_phase=0, period_k=2, phase=1, n_text=2, n_speech=3,
         scope=wl.SCOPE_STREAM),
    # the largest supported period: fifteen pending positions and the current one in one pass
    dict(period_k=16, phase=15, n_text=1, n_speech=20, scope=wl.SCOPE_STREAM, exit_layer=1),
]


@pytest.mark.parametrize("over", SCHEDULES, ids=lambda o: "-".join(f"{k}{v}" for k, v in o.items()))
def test_schedules_and_degenerate_cases(sb, tiny_weights, over):
    w = wl.TINY
    sched = w.schedule.replace(**over)
    say(f"case schedule {over}")
    sp = sb.Spark(w.shape, sched, tiny_weights, max_batch=1, max_seq_len=96, kv_page_tokens=16)
    prompt = wl.make_prompt(w.shape, 9, seed=5)
    res = compare_run(sp, w.shape, sched, tiny_weights, [prompt], [2], 36, check_kv_every=3,
                      label=str(over))
    if sched.exit_layer == w.shape.n_layers or (sched.period_k == 1 and sched.text_period_k <= 1):
        assert np.all(res["depths"] == w.shape.n_layers)
    if sched.text_period_k > 1:
        assert res["stats"][0]["text_ee"] > 0
    sp.close()


def test_batch_of_sequences_mixed_schedules_and_multi_step_calls(sb, tiny_weights):
    """several sequences with different prompt lengths and cycle offsets in the same steps: some
    rows exit early while others run full depth; spark_decode chunks equal single steps"""
    w = wl.TINY
    sched = w.schedule
    say("case batch mixed")
    prompts = [wl.make_prompt(w.shape, n, seed=10 + n) for n in (1, 16, 17, 33, 5)]
    offsets = [0, 1, 3, 5, 2]
    sp = sb.Spark(w.shape, sched, tiny_weights, max_batch=5, max_seq_len=96, kv_page_tokens=16)
    a = compare_run(sp, w.shape, sched, tiny_weights, prompts, offsets, 30, check_kv_every=5,
                    label="batch5 step")
    b = compare_run(sp, w.shape, sched, tiny_weights, prompts, offsets, 30, chunk=7,
                    label="batch5 decode(7)")
    assert np.array_equal(a["depths"], b["depths"])
    assert len(np.unique(a["depths"], axis=1)) > 1      # schedules really were mixed in a step
    # logits are readable after the last step of a call only: calls of 2, 3 and 5 steps end, between
    # them, on 22 of the 30 steps (every multiple of 2, 3 or 5), so the logits of steps enqueued
    # without a return to the host are compared with the oracle's at most positions of the run too
    for chunk in (2, 3, 5):
        c = compare_run(sp, w.shape, sched, tiny_weights, prompts, offsets, 30, chunk=chunk,
                        label=f"batch5 decode({chunk})")
        assert np.array_equal(a["depths"], c["depths"])
    sp.close()


def test_free_running_matches_oracle_until_a_near_tie(sb, tiny_weights):
    """no teacher forcing: the emitted token feeds the next step on both sides"""
    from oracle import binding as ob
    w = wl.TINY
    say("case free running")
    sp = sb.Spark(w.shape, w.schedule, tiny_weights, max_batch=1, max_seq_len=128, kv_page_tokens=16)
    prompt = wl.make_prompt(w.shape, 16, seed=1)
    sid = sp.seq_open(0)
    sp.prefill(sid, prompt)
    gtok, gdep = sp.decode(64, [sid])
    om = ob.Model(w.shape, w.schedule, tiny_weights, max_seq_len=128)
    os_ = om.open(0)
    os_.prefill(prompt)
    for i in range(64):
        rc, otok, odep, ologits = os_.step()
        assert rc == 0 and odep == gdep[i, 0]
        if otok != gtok[i, 0]:
            gap = float(ologits[otok] - ologits[gtok[i, 0]])
            say(f"  free-running streams part at step {i} on a near tie (gap {gap:.3g})")
            assert gap <= 2e-4
            break
    os_.close(); om.close(); sp.close()


@pytest.mark.parametrize("name,shape_kw,sched_kw", [
    ("bf16-tiny", dict(dtype=wl.DTYPE_BF16), dict()),
    # 7 query heads per KV head, head_dim 128, odd vocabulary, FFN width not a multiple of 512
    ("bf16-gqa7", dict(dtype=wl.DTYPE_BF16, n_layers=6, d_model=896, n_q_heads=7, n_kv_heads=1,
                       head_dim=128, d_ffn=1712, vocab_text=3001, vocab_speech=1000),
     dict(exit_layer=4, n_text=1, n_speech=2, scope=wl.SCOPE_STREAM)),
    ("bf16-gqa16", dict(dtype=wl.DTYPE_BF16, n_layers=5, d_model=1024, n_q_heads=16, n_kv_heads=1,
                        head_dim=64, d_ffn=2048 + 264, vocab_text=2000, vocab_speech=777),
     dict(exit_layer=3, period_k=3, phase=2, n_text=2, n_speech=7)),
    # MFMA attention (bf16 cache, head_dim 128) with 1, 4, 8 and 16 query heads per KV head
    ("bf16-hd128-g1", dict(dtype=wl.DTYPE_BF16, n_layers=3, d_model=256, n_q_heads=2, n_kv_heads=2, head_dim=128,
                           d_ffn=512), dict(exit_layer=2)),
    ("bf16-hd128-g4", dict(dtype=wl.DTYPE_BF16, n_layers=3, d_model=256, n_q_heads=4, n_kv_heads=1, head_dim=128,
                           d_ffn=512), dict(exit_layer=2)),
    ("bf16-hd128-g8", dict(dtype=wl.DTYPE_BF16, n_layers=3, d_model=512, n_q_heads=8, n_kv_heads=1, head_dim=128,
                           d_ffn=512), dict(exit_layer=1)),
    ("bf16-hd128-g16", dict(dtype=wl.DTYPE_BF16, n_layers=3, d_model=512, n_q_heads=16, n_kv_heads=1, head_dim=128,
                            d_ffn=768), dict(exit_layer=2, n_text=1, n_speech=2, scope=wl.SCOPE_STREAM)),
    ("fp32-wide", dict(n_layers=3, d_model=4096, n_q_heads=4, n_kv_heads=2, head_dim=128,
                       d_ffn=5000 - 8, vocab_text=700, vocab_speech=300),
     dict(exit_layer=2)),
])
def test_other_shapes(sb, name, shape_kw, sched_kw):
    shape = wl.TINY.shape.replace(name=name, **shape_kw)
    sched = wl.TINY.schedule.replace(**sched_kw)
    say(f"case shape {name}")
    weights = wl.make_weights(shape, seed=3, gain_std=0.1)
    sp = sb.Spark(shape, sched, weights, max_batch=2, max_seq_len=400, kv_page_tokens=32)
    prompts = [wl.make_prompt(shape, 70, seed=4), wl.make_prompt(shape, 300, seed=5)]
    compare_run(sp, shape, sched, weights, prompts, [0, 1], 20, check_kv_every=4, label=name)
    sp.close()


def test_edge_cases_and_errors(sb, tiny_weights):
    w = wl.TINY
    say("case edges")
    sp = sb.Spark(w.shape, w.schedule, tiny_weights, max_batch=2, max_seq_len=40, kv_page_tokens=16)
    a = sp.seq_open(0)
    with pytest.raises(sb.SparkError) as ei:
        sp.step([a])
    assert ei.value.code == -4                       # step before prefill
    with pytest.raises(sb.SparkError) as ei:
        sp.prefill(a, [])
    assert ei.value.code == -1
    with pytest.raises(sb.SparkError) as ei:
        sp.prefill(a, [w.shape.vocab])
    assert ei.value.code == -1
    with pytest.raises(sb.SparkError) as ei:
        sp.prefill(a, np.zeros(41, dtype=np.int32))
    assert ei.value.code == -3
    sp.prefill(a, wl.make_prompt(w.shape, 33, seed=1))     # 32 cached positions = 2 full pages
    with pytest.raises(sb.SparkError) as ei:
        sp.prefill(a, [1, 2])
    assert ei.value.code == -4
    with pytest.raises(sb.SparkError) as ei:
        sp.step([a, a])
    assert ei.value.code == -1
    with pytest.raises(sb.SparkError) as ei:
        sp.step([7])
    assert ei.value.code == -2
    b = sp.seq_open(1)
    with pytest.raises(sb.SparkError) as ei:
        sp.seq_open(0)
    assert ei.value.code == -2                       # both slots taken
    sp.prefill(b, [5])                               # single-token prompt: nothing cached
    assert sp.seq_state(b) == {"len": 0, "upper_valid": 0, "pending": 0}
    for _ in range(8):                               # a fills its context: 32 + 8 = 40
        sp.step([a, b])
    with pytest.raises(sb.SparkError) as ei:
        sp.step([a])
    assert ei.value.code == -3                       # context full
    tok, dep = sp.step([b])                          # b is unaffected
    assert dep[0] in (w.schedule.exit_layer, w.shape.n_layers)
    sp.seq_close(a)
    c = sp.seq_open(0)                               # slot and pages are reusable
    sp.prefill(c, wl.make_prompt(w.shape, 20, seed=2))
    sp.step([c, b])
    sp.close()


def test_reopened_slot_reproduces_a_fresh_run(sb, tiny_weights):
    w = wl.TINY
    say("case reuse")
    sp = sb.Spark(w.shape, w.schedule, tiny_weights, max_batch=1, max_seq_len=64, kv_page_tokens=16)
    prompt = wl.make_prompt(w.shape, 16, seed=1)
    runs = []
    for _ in range(2):
        sid = sp.seq_open(0)
        sp.prefill(sid, prompt)
        tok, dep = sp.decode(40, [sid])
        logits, _ = sp.get_logits(sid)
        runs.append((tok.copy(), dep.copy(), logits.copy()))
        sp.seq_close(sid)
    assert np.array_equal(runs[0][0], runs[1][0]) and np.array_equal(runs[0][1], runs[1][1])
    assert np.array_equal(runs[0][2], runs[1][2])    # bit-identical: no order-dependent reductions
    sp.close()


def test_text_schedule_with_long_flushes_on_a_bf16_model(sb):
    """text and speech both scheduled (Sec. V-C): runs of early exits cross the modality boundary,
    so one sequence completes up to six rows in a full-depth step; on a bf16 model four or more
    rows go through the MFMA kernels, fewer through the vector kernel"""
    shape = wl.TINY.shape.replace(name="bf16-textsched", dtype=wl.DTYPE_BF16, n_layers=4, d_model=512,
                                  n_q_heads=8, n_kv_heads=4, head_dim=64, d_ffn=1536 + 72,
                                  vocab_text=1500, vocab_speech=701)
    # text: full, early, early; speech: early, early, early, full -> five pending rows + the current
    sched = wl.TINY.schedule.replace(text_period_k=3, text_phase=0, period_k=4, phase=3, n_text=3,
                                     n_speech=4)
    say("case text schedule bf16")
    weights = wl.make_weights(shape, seed=8, gain_std=0.1)
    sp = sb.Spark(shape, sched, weights, max_batch=1, max_seq_len=128, kv_page_tokens=16)
    res = compare_run(sp, shape, sched, weights, [wl.make_prompt(shape, 21, seed=9)], [0], 42,
                      check_kv_every=5, label="text schedule bf16")
    hist = res["stats"][0]["flush_hist"]
    assert max(hist) >= 5 and res["stats"][0]["text_ee"] > 0
    sp.close()


@pytest.mark.parametrize("tiled", [1, 0])
def test_batched_decode_on_the_mfma_path(sb, tiled):
    """24 bf16 sequences with mixed schedules in every step: 24 rows through layers 1..e, the
    early-exit rows through the layer-specific head, the full-depth rows with their pending rows
    (up to 4 each) through layers e+1..L and the final head -- all as MFMA contractions, once with
    the weights taken from the copy in MFMA operand order (the default of a context with a
    full-size scratch area) and once with the kernel that stages the caller's rows through LDS
    (what a context on the static scratch area runs)"""
    shape = wl.TINY.shape.replace(name="bf16-batch", dtype=wl.DTYPE_BF16, n_layers=4, d_model=512,
                                  n_q_heads=8, n_kv_heads=4, head_dim=64, d_ffn=1536 + 72,
                                  vocab_text=1500, vocab_speech=701)
    sched = wl.TINY.schedule
    say("case batched mfma")
    weights = wl.make_weights(shape, seed=6, gain_std=0.1)
    B = 24
    lens = wl.make_prompt_lengths(B, 3, 90, seed=3)
    prompts = [wl.make_prompt(shape, int(n), seed=40 + i) for i, n in enumerate(lens)]
    offsets = [i % 6 for i in range(B)]
    sp = sb.Spark(shape, sched, weights, max_batch=B, max_seq_len=160, kv_page_tokens=16)
    sp.tune("mfma_tiled", tiled)
    a = compare_run(sp, shape, sched, weights, prompts, offsets, 14, check_kv_every=7,
                    label=f"batch24 bf16 tiled={tiled}")
    assert len(np.unique(a["depths"], axis=1)) > 1
    sp.close()


@pytest.mark.parametrize("rows,small_max_k", [(32, 32768), (96, 32768), (96, 8), (160, 8)])
def test_prompt_pass_row_counts_and_tile_shapes(sb, rows, small_max_k):
    """a 150-token prompt in passes of 32, 96 or 160 rows (one 32-row tile; a 64-row and a 32-row
    tile; ragged last tiles), with the 128-task tiles that matrices of few tiles get by default and
    with 256-task tiles forced for every projection (64 tasks, four A tiles, per wave); the decoding
    steps behind the prompt and cache entries across it are compared with the oracle"""
    shape = wl.TINY.shape.replace(name="bf16-prompt", dtype=wl.DTYPE_BF16, n_layers=4, d_model=512,
                                  n_q_heads=4, n_kv_heads=2, head_dim=128, d_ffn=1024 + 40,
                                  vocab_text=900, vocab_speech=301)
    sched = wl.TINY.schedule
    say(f"case prompt passes of {rows} rows, small tiles up to k = {small_max_k}")
    weights = wl.make_weights(shape, seed=8, gain_std=0.1)
    sp = sb.Spark(shape, sched, weights, max_batch=1, max_seq_len=256, kv_page_tokens=64)
    sp.tune("prefill_rows", rows)
    sp.tune("mfma_small_max_k", small_max_k)
    compare_run(sp, shape, sched, weights, [wl.make_prompt(shape, 150, seed=61)], [2], 8, check_kv_every=1,
                label=f"prompt150 rows={rows} small_k={small_max_k}", kv_all_positions=True)
    sp.close()


@pytest.mark.parametrize("B", [3, 4, 5, 7, 8])
def test_row_counts_around_the_mfma_threshold(sb, B):
    """bf16 sequences with the same cycle offset: every pass of the lower layers has exactly B rows
    (three and four: one pass of the vector kernel; five: the MFMA projections), the flushes B to
    4B rows; head size 128, so attention runs on its MFMA kernel throughout"""
    shape = wl.TINY.shape.replace(name="bf16-rows", dtype=wl.DTYPE_BF16, n_layers=4, d_model=512,
                                  n_q_heads=4, n_kv_heads=2, head_dim=128, d_ffn=1024 + 40,
                                  vocab_text=900, vocab_speech=301)
    sched = wl.TINY.schedule
    say(f"case {B} rows per pass")
    weights = wl.make_weights(shape, seed=8, gain_std=0.1)
    prompts = [wl.make_prompt(shape, 5 + 9 * i, seed=60 + i) for i in range(B)]
    sp = sb.Spark(shape, sched, weights, max_batch=B, max_seq_len=128, kv_page_tokens=64)
    compare_run(sp, shape, sched, weights, prompts, [0] * B, 13, check_kv_every=6, label=f"rows {B} bf16")
    sp.close()


def test_text_ends_before_the_speech(sb, tiny_weights):
    """Sec. IV-A: after a sequence's text budget every position is speech.  Per-chunk and stream
    counters, several sequences with different budgets and cycle offsets in one batch, multi-step
    calls; and a budget that is set between two steps."""
    w = wl.TINY
    say("case text budget")
    for scope in (wl.SCOPE_CHUNK, wl.SCOPE_STREAM):
        sched = w.schedule.replace(scope=scope)
        sp = sb.Spark(w.shape, sched, tiny_weights, max_batch=4, max_seq_len=160, kv_page_tokens=16)
        prompts = [wl.make_prompt(w.shape, 10 + 3 * b, seed=20 + b) for b in range(4)]
        res = compare_run(sp, w.shape, sched, tiny_weights, prompts, [0, 1, 4, 5], 60, chunk=5,
                          text_budgets=[3, 7, 0, 1], label=f"text budget scope {scope}")
        texts = [st["text"] for st in res["stats"]]
        assert texts[0] == 3 and texts[1] == 7 and texts[3] == 1 and texts[2] >= 20
        sp.close()
    # set between steps: "the text has just ended"
    from oracle import binding as ob
    sp = sb.Spark(w.shape, w.schedule, tiny_weights, max_batch=1, max_seq_len=96, kv_page_tokens=16)
    om = ob.Model(w.shape, w.schedule, tiny_weights, max_seq_len=96)
    sid, os_ = sp.seq_open(0), om.open(0)
    prompt = wl.make_prompt(w.shape, 8, seed=3)
    sp.prefill(sid, prompt)
    assert os_.prefill(prompt) == 0
    forced = wl.make_forced_stream(w.shape, 40, 2, 4, 0, seed=5)
    for i in range(40):
        if i == 8:      # two text tokens of the first cycle and two of the second are out
            with pytest.raises(sb.SparkError):
                sp.seq_text_budget(sid, 3)                   # fewer than already generated
            sp.seq_text_budget(sid, 4)
            assert os_.text_budget(4) == 0
            with pytest.raises(sb.SparkError):
                sp.seq_text_budget(sid, 9)                   # only once
        tok, dep = sp.step([sid], [forced[i]])
        rc, otok, odep, _ = os_.step(forced_next=int(forced[i]))
        assert rc == 0 and dep[0] == odep, (i, dep[0], odep)
    assert sp.get_stats(sid)["text"] == 4 == os_.stats()["text"]
    os_.close(); om.close(); sp.close()


@pytest.mark.parametrize("name,shape_kw,page,long_prompt", [
    # MFMA attention (bf16 cache, head_dim 128): 36 slices, a slice inside one 64-token page
    ("bf16-hd128-long", dict(dtype=wl.DTYPE_BF16, n_layers=3, d_model=512, n_q_heads=4, n_kv_heads=2,
                             head_dim=128, d_ffn=1024), 64, 2300),
    # the same kernel with slices that span four 16-token pages
    ("bf16-hd128-small-pages", dict(dtype=wl.DTYPE_BF16, n_layers=3, d_model=512, n_q_heads=4, n_kv_heads=2,
                                    head_dim=128, d_ffn=1024), 16, 900),
    # vector attention (fp32), 19 slices
    ("fp32-long", dict(), 64, 1200),
])
def test_long_contexts(sb, name, shape_kw, page, long_prompt):
    """contexts of many attention slices: the merge runs several rounds of eight partials, the
    prompt passes see rows whose contexts differ by a whole pass, a short sequence shares the batch"""
    shape = wl.TINY.shape.replace(name=name, **shape_kw)
    sched = wl.TINY.schedule.replace(exit_layer=2, n_text=1, n_speech=2, scope=wl.SCOPE_STREAM)
    say(f"case long context {name}")
    weights = wl.make_weights(shape, seed=6, gain_std=0.1)
    sp = sb.Spark(shape, sched, weights, max_batch=2, max_seq_len=long_prompt + 64, kv_page_tokens=page)
    prompts = [wl.make_prompt(shape, long_prompt, seed=7), wl.make_prompt(shape, 70, seed=8)]
    res = compare_run(sp, shape, sched, weights, prompts, [0, 2], 24, check_kv_every=8, chunk=3, label=name)
    assert len(np.unique(res["depths"])) == 2
    sp.close()


@pytest.mark.parametrize("pieces", [3, 8])
def test_attention_pieces_per_workgroup(sb, pieces):
    """the MFMA attention kernel with a fixed number of 64-token pieces per workgroup (the library
    picks 1, 2, 4 or 8 by the size of the launch; eight is what contexts of 4096 tokens and more
    get): a 2300-token context is 36 slices, so workgroups with all their pieces, with some, and
    the ragged last one all occur; prompt passes and decode steps"""
    shape = wl.TINY.shape.replace(name="bf16-hd128-pieces", dtype=wl.DTYPE_BF16, n_layers=3, d_model=512,
                                  n_q_heads=4, n_kv_heads=2, head_dim=128, d_ffn=1024)
    sched = wl.TINY.schedule.replace(exit_layer=2, n_text=1, n_speech=2, scope=wl.SCOPE_STREAM)
    say(f"case attention with {pieces} pieces per workgroup")
    weights = wl.make_weights(shape, seed=6, gain_std=0.1)
    sp = sb.Spark(shape, sched, weights, max_batch=2, max_seq_len=2300 + 64, kv_page_tokens=64)
    sp.tune("attn_pieces", pieces)
    with pytest.raises(sb.SparkError):
        sp.tune("no_such_switch", 1)
    prompts = [wl.make_prompt(shape, 2300, seed=7), wl.make_prompt(shape, 200, seed=8)]
    compare_run(sp, shape, sched, weights, prompts, [0, 2], 12, check_kv_every=6, chunk=3, label=f"pieces {pieces}")
    sp.close()


def test_moved_and_aligned_phases(sb, tiny_weights):
    """a sequence's speech phase moved between steps, and a batch aligned (Sec. IV-B.3: an
    early-exit step skips the upper layers only if no sequence of the batch needs them): depths,
    tokens and logits against the oracle with the same moves; after the alignment the sequences,
    all in their speech tail, run full depth on the same steps"""
    from oracle import binding as ob
    w = wl.TINY
    say("case moved phases")
    sched = w.schedule.replace(scope=wl.SCOPE_STREAM, n_text=1, n_speech=2)
    K = sched.period_k
    sp = sb.Spark(w.shape, sched, tiny_weights, max_batch=3, max_seq_len=160, kv_page_tokens=16)
    om = ob.Model(w.shape, sched, tiny_weights, max_seq_len=160)
    offsets, budgets = [0, 1, 2], [2, 4, 3]
    sids = [sp.seq_open(o) for o in offsets]
    oseqs = [om.open(o) for o in offsets]
    for b in range(3):
        prompt = wl.make_prompt(w.shape, 9 + 2 * b, seed=40 + b)
        sp.prefill(sids[b], prompt)
        assert oseqs[b].prefill(prompt) == 0
        sp.seq_text_budget(sids[b], budgets[b])
        assert oseqs[b].text_budget(budgets[b]) == 0
    n = 60
    forced = np.stack([wl.make_forced_stream(w.shape, n, 1, 2, offsets[b], seed=50 + b) for b in range(3)], axis=1)
    depths = []
    for i in range(n):
        if i == 7:                                   # one sequence alone
            sp.seq_set_phase(sids[1], 0)
            assert oseqs[1].set_phase(0) == 0
            with pytest.raises(sb.SparkError):
                sp.seq_set_phase(sids[1], K)
        if i == 24:                                  # the whole batch, all in their speech tail by now
            sp.align_phases(sids)
            for b in range(3):
                assert oseqs[b].set_phase((oseqs[b].j_stream + K - 1) % K) == 0
        tok, dep = sp.step(sids, forced[i])
        for b in range(3):
            rc, otok, odep, ologits = oseqs[b].step(forced_next=int(forced[i, b]))
            assert rc == 0 and dep[b] == odep, (i, b, dep[b], odep)
            glogits, _ = sp.get_logits(sids[b])
            assert np.max(np.abs(glogits - ologits)) <= 1e-4
            assert tok[b] == otok or ologits[otok] - ologits[tok[b]] <= 2e-4
        depths.append(dep.copy())
    depths = np.array(depths)
    tail = depths[24:]
    assert np.all(tail == tail[:, :1])                        # the same depth for all three, step by step
    full = np.flatnonzero(tail[:, 0] == w.shape.n_layers)
    assert full[0] == K - 1 and np.all(np.diff(full) == K)
    assert not np.all(depths[8:24] == depths[8:24, :1])       # before the alignment they differed
    for os_ in oseqs:
        os_.close()
    om.close(); sp.close()


def test_moved_phase_is_validated_and_pending_rows_cannot_outgrow_their_slots(sb, tiny_weights):
    """per-chunk counters on a pure-speech cycle of three slots with K = 4: a phase of 3 would never
    run full depth (refused, as spark_init refuses such a configuration); and a caller that keeps
    moving the phase away from the slot about to run never completes the pending positions: the
    step that would need a ninth hidden-state slot is refused before anything is enqueued, and the
    sequence can go on once a full-depth step is allowed"""
    w = wl.TINY
    say("case moved phase validation")
    sched = w.schedule.replace(scope=wl.SCOPE_CHUNK, n_text=0, n_speech=3, period_k=4, phase=0)
    sp = sb.Spark(w.shape, sched, tiny_weights, max_batch=1, max_seq_len=64, kv_page_tokens=16)
    sid = sp.seq_open(0)
    sp.prefill(sid, wl.make_prompt(w.shape, 5, seed=1))
    with pytest.raises(sb.SparkError) as ei:
        sp.seq_set_phase(sid, 3)
    assert ei.value.code == -1
    depths = []
    for g in range(7):                               # slot g % 3 runs next: keep the phase elsewhere
        sp.seq_set_phase(sid, (g % 3 + 1) % 3)
        depths.append(int(sp.step([sid])[1][0]))
    assert depths == [w.schedule.exit_layer] * 7 and sp.seq_state(sid)["pending"] == 7
    sp.seq_set_phase(sid, (7 % 3 + 1) % 3)
    with pytest.raises(sb.SparkError) as ei:         # 8 pending rows + the next position > 8 slots
        sp.step([sid])
    assert ei.value.code == -4
    assert sp.seq_state(sid) == {"len": 11, "upper_valid": 4, "pending": 7}   # nothing was enqueued
    sp.seq_set_phase(sid, 7 % 3)                     # the slot about to run is the full-depth one
    tok, dep = sp.step([sid])
    assert dep[0] == w.shape.n_layers and sp.seq_state(sid)["pending"] == 0
    assert sp.get_stats(sid)["flush_hist"] == {8: 1}
    sp.close()
