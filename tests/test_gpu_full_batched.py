"""GPU parity of batched decoding at the full shapes of the two benchmark backbones, against the
oracle's fp64 twin, element by element: several sequences per step, so that the projections of
layers 1..e, the batched pass of pending rows through layers e+1..L (Sec. IV-B.3) and both
vocabulary heads run on the MFMA path with the row counts a batch produces (5 to 24 rows, ragged),
with the k-split partial sums and the finishing launches the library itself selects at d = 3584 /
4096 and V = 158 497 / 167 936.  Prompts are short (the oracle walks every prompt token through
all layers); long contexts are covered in test_gpu_long_context.py."""
import time

import numpy as np
import pytest

import workloads as wl
from parity_util import compare_run, full_weights, say

pytestmark = pytest.mark.gpu

CASES = [
    # name, sequences, cycle offsets, steps
    # equal offsets: every row of a step takes the same head -> the MFMA lens head and the MFMA final
    # head see all 8 rows, and a full-depth step pushes 8..24 rows through the upper layers
    ("step_audio_2_mini", 8, "equal", 12),
    # mixed offsets: early-exit and full-depth rows in the same step (ragged exit), flushes of 1..3
    # rows per sequence, both heads in one step with few rows each
    ("step_audio_2_mini", 8, "mixed", 12),
    ("glm_4_voice", 6, "equal", 8),
    ("glm_4_voice", 6, "mixed", 8),
]


@pytest.mark.parametrize("name,B,offsets,n_steps", CASES)
def test_full_shape_batched_decode(name, B, offsets, n_steps):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_09215_amd import binding as sb
    w = wl.WORKLOADS[name]
    say(f"case full shape batched {name} B={B} offsets={offsets}")
    dev_w, host_w = full_weights(name)
    cyc = w.schedule.n_text + w.schedule.n_speech
    if offsets == "equal":
        # GLM: enter the cycle two text slots before its 26-slot speech chunk, so that 8 steps hold
        # full-depth text steps, early exits and a full-depth speech step with three pending rows
        offs = [0 if name == "step_audio_2_mini" else 11] * B
    else:
        # spread over the cycle; for GLM around the text/speech boundary so that both classes occur
        offs = [(i * 5) % cyc if name == "step_audio_2_mini" else 9 + i for i in range(B)]
    rng = np.random.default_rng(11)
    plens = [int(x) for x in rng.integers(4, 9, size=B)]
    prompts = [wl.make_prompt(w.shape, p, seed=31 + i, ids=w.prompt_ids) for i, p in enumerate(plens)]
    sp = sb.Spark(w.shape, w.schedule, dev_w, max_batch=B, max_seq_len=64, kv_page_tokens=64)
    t0 = time.time()
    res = compare_run(sp, w.shape, w.schedule, host_w, prompts, offs, n_steps, check_kv_every=1,
                      kv_all_positions=False, label=f"{name}/B{B}/{offsets}", oracle_kind="f64",
                      trace_steps=True)
    say(f"  compared in {time.time() - t0:.1f}s")
    depths = res["depths"]
    L, e = w.shape.n_layers, w.schedule.exit_layer
    assert set(np.unique(depths)) == {e, L}
    rows_full = (depths == L).sum(axis=1)
    rows_ee = (depths == e).sum(axis=1)
    if offsets == "equal":
        assert set(np.unique(rows_full)) == {0, B}            # a step is one class for the whole batch
    else:
        assert np.any((rows_full > 0) & (rows_ee > 0))        # ragged exit inside one step
    # rows through the upper layers in one pass: pending rows + their own, summed over the batch
    flushed = sum(m * n for st in res["stats"] for m, n in st["flush_hist"].items())
    say(f"  rows per step: full depth {rows_full.tolist()}, early exit {rows_ee.tolist()}; "
        f"{flushed} rows went through layers {e + 1}..{L}")
    sp.close()


@pytest.mark.parametrize("exit_layer,period", [(14, 8), (24, 2)])
def test_full_shape_batched_sweep_points(exit_layer, period):
    """the far corners of the batched benchmark's sweep (exit layer 14 / 20 / 24, period 2 / 4 / 8)
    at the full Step-Audio-2-mini shape: five sequences with mixed cycle offsets, so that the pass
    through the upper layers has 14 or 4 of them and flushes of up to 8 rows per sequence occur
    with the long period"""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_09215_amd import binding as sb
    w = wl.WORKLOADS["step_audio_2_mini"]
    sched = w.schedule.replace(exit_layer=exit_layer, period_k=period, phase=period - 1)
    say(f"case full shape batched sweep point e={exit_layer} K={period}")
    dev_w, host_w = full_weights("step_audio_2_mini")
    B, n_steps = 5, 10
    offs = [i % 3 for i in range(B)]
    prompts = [wl.make_prompt(w.shape, 3 + i, seed=71 + i, ids=w.prompt_ids) for i in range(B)]
    sp = sb.Spark(w.shape, sched, dev_w, max_batch=B, max_seq_len=64, kv_page_tokens=64)
    res = compare_run(sp, w.shape, sched, host_w, prompts, offs, n_steps, check_kv_every=2,
                      label=f"step_audio_2_mini/B{B}/e{exit_layer}K{period}", oracle_kind="f64", trace_steps=True)
    assert set(np.unique(res["depths"])) == {exit_layer, w.shape.n_layers}
    sp.close()
