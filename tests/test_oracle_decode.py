"""Pins for the oracle's decoding loops.

  * standard incremental decoding (KV cache) == full recomputation with a T x T causal mask
    (numpy definition) -- textbook identity;
  * SPAR-K with e = L, or with K = 1, == standard decoding, token for token and logit for logit;
  * teacher-forced SPAR-K: every full-depth step restores complete KV at all layers (end of
    Sec. IV-B.3), so its g_L logits at full-depth positions and its g_e logits at early-exit
    positions equal those computed from the hidden states of a plain full-depth pass, and its KV
    cache equals standard decoding's;
  * pending-set bookkeeping of Algorithm 1.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import binding as ob
from oracle import definition as od

TOL = {"f32": 2e-5, "f64": 1e-11}


@pytest.fixture(scope="module")
def tiny():
    w = wl.TINY
    weights = wl.make_weights(w.shape, seed=0, gain_std=0.1)
    prompt = wl.make_prompt(w.shape, w.prompt_len, seed=1)
    return w, weights, prompt


def stream_positions(prompt, forced):
    """the token at every position when `forced` is teacher-forced after `prompt`"""
    return np.concatenate([prompt, forced[:-1]])


@pytest.mark.parametrize("kind", ["f32", "f64"])
def test_standard_incremental_equals_full_recompute(tiny, kind):
    w, weights, prompt = tiny
    n_new = 24
    def_toks, def_logits = od.greedy_standard(w.shape, weights, prompt, n_new)
    m = ob.Model(w.shape, w.schedule, weights, max_seq_len=64, kind=kind)
    s = m.open()
    assert s.prefill(prompt) == 0
    for i in range(n_new):
        rc, tok, logits, _ = s.step_standard(forced_next=int(def_toks[i]))
        assert rc == 0
        assert np.max(np.abs(logits - def_logits[i])) < TOL[kind]
        gap = def_logits[i][def_toks[i]] - def_logits[i][tok]
        assert tok == def_toks[i] or gap < 2 * TOL[kind]
    if kind == "f64":   # free-running fp64 reproduces the definition's greedy tokens
        s2 = m.open()
        s2.prefill(prompt)
        assert [s2.step_standard()[1] for _ in range(n_new)] == list(def_toks)
        s2.close()
    s.close(); m.close()


@pytest.mark.parametrize("kind", ["f32", "f64"])
@pytest.mark.parametrize("degenerate", [dict(exit_layer=4), dict(period_k=1, phase=0)])
def test_spark_with_e_equal_L_or_K_equal_1_is_standard_decoding(tiny, kind, degenerate):
    w, weights, prompt = tiny
    sched = w.schedule.replace(**degenerate)
    m = ob.Model(w.shape, sched, weights, max_seq_len=64, kind=kind)
    a, b = m.open(), m.open()
    a.prefill(prompt); b.prefill(prompt)
    for _ in range(30):                       # free running: identical arithmetic, exact equality
        rc, tok, depth, logits = a.step()
        rc2, tok2, logits2, _ = b.step_standard()
        assert rc == 0 and rc2 == 0
        assert depth == w.shape.n_layers
        assert tok == tok2
        assert np.array_equal(logits, logits2)
        assert a.pending == 0 and a.upper_valid == a.len
    a.close(); b.close(); m.close()


CASES = [
    # (schedule overrides, cycle_offset)
    (dict(), 0),                                                      # tiny workload as specified
    (dict(period_k=2, phase=0, n_text=1, n_speech=4), 0),             # Even
    (dict(period_k=2, phase=1, n_text=1, n_speech=4), 3),             # Odd, entered mid-cycle
    (dict(period_k=3, phase=0, n_text=1, n_speech=4), 0),             # Triple, short last period
    (dict(period_k=4, phase=3, n_text=1, n_speech=2, scope=wl.SCOPE_STREAM), 0),
    (dict(period_k=3, phase=1, n_text=0, n_speech=5, exit_layer=1), 2),   # no text: joined runs
    (dict(period_k=5, phase=4, n_text=2, n_speech=4, exit_layer=3), 1),   # fixed-layer baseline
    # the periodic rule on text positions (Sec. V-C, Table II row G10: text Even, speech full depth)
    (dict(text_period_k=2, text_phase=0, period_k=1, phase=0, n_text=3, n_speech=2), 0),
    # both modalities scheduled: early-exit runs cross the modality boundary
    (dict(text_period_k=2, text_phase=1, period_k=4, phase=3, n_text=2, n_speech=4), 1),
    (dict(text_period_k=3, text_phase=0, period_k=2, phase=1, n_text=2, n_speech=3,
          scope=wl.SCOPE_STREAM), 0),
]


@pytest.mark.parametrize("kind", ["f32", "f64"])
@pytest.mark.parametrize("over,offset", CASES)
def test_teacher_forced_spark_equals_full_depth_pass(tiny, kind, over, offset):
    w, weights, prompt = tiny
    sched = w.schedule.replace(**over)
    L, e, K = w.shape.n_layers, sched.exit_layer, sched.period_k
    n = 40
    forced = wl.make_forced_stream(w.shape, n, sched.n_text, sched.n_speech, offset, seed=2)
    tokens = stream_positions(prompt, forced)
    hs = od.hidden_states(w.shape, weights, tokens)          # [L+1, T, d], one causal pass
    p0 = len(prompt) - 1

    m = ob.Model(w.shape, sched, weights, max_seq_len=len(tokens) + 1, kind=kind)
    s = m.open(offset)
    ref = m.open(offset)                                     # standard decoding on the same stream
    assert s.prefill(prompt) == 0 and ref.prefill(prompt) == 0
    want_depth, want_text = ob.schedule_run(w.shape, sched, n, offset)
    seen_pending = 0
    for i in range(n):
        rc, tok, depth, logits = s.step(forced_next=int(forced[i]))
        assert rc == 0
        rc, rtok, rlogits, h_e = ref.step_standard(forced_next=int(forced[i]), capture_layer=e)
        assert rc == 0
        assert depth == want_depth[i]
        pos = p0 + i
        assert np.max(np.abs(h_e - hs[e, pos])) < TOL[kind]
        if depth == L:
            want = od.final_logits(w.shape, weights, hs[L, pos])
            assert np.max(np.abs(logits - want)) < TOL[kind]
            assert np.max(np.abs(logits - rlogits)) < TOL[kind]
            # complete KV restored for every preceding position, at every layer
            assert s.pending == 0 and s.upper_valid == s.len == pos + 1
            for l in range(L):
                for p in range(max(0, pos - 2 * K), pos + 1):
                    k1, v1 = s.kv(l, p); k2, v2 = ref.kv(l, p)
                    assert np.max(np.abs(k1 - k2)) < TOL[kind]
                    assert np.max(np.abs(v1 - v2)) < TOL[kind]
        else:
            assert depth == e and (not want_text[i] or sched.text_period_k > 1)
            want = od.lens_logits(w.shape, weights, hs[e, pos])
            assert np.max(np.abs(logits - want)) < TOL[kind]
            assert np.max(np.abs(logits - m.lens_logits(h_e))) < TOL[kind]
            assert s.pending >= 1
            seen_pending = max(seen_pending, s.pending)
        # emitted token is the argmax of the head that ran (lowest index on ties)
        assert tok == int(np.argmax(logits))
        # bookkeeping: lower frontier = upper frontier + pending, pending bounded
        assert s.upper_valid + s.pending == s.len
        if sched.text_period_k > 1:
            assert s.pending <= 2 * (K - 1) + 2 * (sched.text_period_k - 1)
        else:
            assert s.pending <= (K - 1 if sched.n_text > 0 or sched.scope == wl.SCOPE_STREAM
                                 else 2 * K - 2)
    st = s.stats()
    assert st["text"] + st["text_ee"] == int(want_text.sum())
    assert st["text_ee"] == int(((want_depth == e) & (want_text == 1)).sum()) if e < L else True
    assert st["speech_ee"] == int(((want_depth == e) & (want_text == 0)).sum()) if e < L else True
    assert st["text"] + st["speech_full"] == sum(st["flush_hist"].values())
    assert sum(mm * c for mm, c in st["flush_hist"].items()) <= n
    if e < L and (K > 1 or sched.text_period_k > 1):
        assert seen_pending >= 1
    s.close(); ref.close(); m.close()


def test_lens_reduces_to_logit_lens_when_translator_is_identity(tiny):
    """A = 0, b = 0, gain and unembedding shared with the final head => g_e(h) == g_L(h)"""
    w, weights, prompt = tiny
    w2 = dict(weights)
    w2["lens_a"] = np.zeros_like(weights["lens_a"])
    w2["lens_b"] = np.zeros_like(weights["lens_b"])
    w2["lens_norm"] = weights["final_norm"]
    w2["lens_head"] = weights["lm_head"]
    h = np.random.default_rng(7).standard_normal(w.shape.d_model)
    m = ob.Model(w.shape, w.schedule, w2, max_seq_len=8, kind="f64")
    assert np.allclose(m.lens_logits(h), od.final_logits(w.shape, w2, h), rtol=0, atol=1e-12)
    m.close()


def test_fp32_oracle_tracks_its_fp64_twin(tiny):
    """bounds the fp32 oracle's own rounding noise on the tiny workload (teacher-forced)"""
    w, weights, prompt = tiny
    sched = w.schedule
    n = w.decode_len
    forced = wl.make_forced_stream(w.shape, n, sched.n_text, sched.n_speech, 0, seed=2)
    outs = {}
    for kind in ("f32", "f64"):
        m = ob.Model(w.shape, sched, weights, max_seq_len=w.prompt_len + n, kind=kind)
        s = m.open()
        s.prefill(prompt)
        outs[kind] = [s.step(forced_next=int(forced[i])) for i in range(n)]
        s.close(); m.close()
    worst = 0.0
    for a, b in zip(outs["f32"], outs["f64"]):
        assert a[2] == b[2]
        worst = max(worst, float(np.max(np.abs(a[3] - b[3]))))
    assert worst < 1e-5


def test_state_errors(tiny):
    w, weights, prompt = tiny
    m = ob.Model(w.shape, w.schedule, weights, max_seq_len=18, kind="f32")
    s = m.open()
    assert s.step()[0] == -2                     # step before prefill
    assert s.prefill(np.array([], dtype=np.int32)) == -1
    assert s.prefill(np.array([w.shape.vocab], dtype=np.int32)) == -1
    assert s.prefill(prompt) == 0
    assert s.prefill(prompt) == -2               # second prompt on a live sequence
    assert s.step()[0] == 0 and s.step()[0] == 0 and s.step()[0] == 0
    assert s.step()[0] == -3                     # context full (16 prompt + 3 = 18 + held input)
    s.close(); m.close()


def test_bf16_model_with_bf16_kv_storage():
    """bf16 weights and a KV cache that stores bf16 (rounded once, when written): standard
    decoding equals the numpy definition with the same storage rounding, and teacher-forced
    SPAR-K equals standard decoding, cache entry for cache entry"""
    w = wl.TINY
    shape = w.shape.replace(dtype=wl.DTYPE_BF16)
    sched = w.schedule
    weights = wl.make_weights(shape, seed=4, gain_std=0.1)
    prompt = wl.make_prompt(shape, 12, seed=1)
    n = 26
    forced = wl.make_forced_stream(shape, n, sched.n_text, sched.n_speech, 0, seed=2)
    tokens = stream_positions(prompt, forced)
    hs = od.hidden_states(shape, weights, tokens, kv_bf16=True)
    hs_plain = od.hidden_states(shape, weights, tokens, kv_bf16=False)
    assert np.max(np.abs(hs[-1] - hs_plain[-1])) > 1e-4          # the storage format matters
    p0 = len(prompt) - 1
    L, e = shape.n_layers, sched.exit_layer
    for kind, tol in (("f64", 1e-9), ("f32", 5e-4)):
        m = ob.Model(shape, sched, weights, max_seq_len=len(tokens) + 1, kind=kind, kv_round_bf16=True)
        s, ref = m.open(), m.open()
        s.prefill(prompt); ref.prefill(prompt)
        for i in range(n):
            rc, tok, depth, logits = s.step(forced_next=int(forced[i]))
            rc2, rtok, rlogits, h_e = ref.step_standard(forced_next=int(forced[i]), capture_layer=e)
            assert rc == 0 and rc2 == 0
            pos = p0 + i
            if depth == L:
                assert np.max(np.abs(logits - od.final_logits(shape, weights, hs[L, pos]))) < tol
                assert np.max(np.abs(logits - rlogits)) < tol
                for l in range(L):
                    for p in range(max(0, pos - 4), pos + 1):
                        k1, v1 = s.kv(l, p); k2, v2 = ref.kv(l, p)
                        assert np.array_equal(k1, k2) and np.array_equal(v1, v2)
                        # what is stored is representable in bf16
                        assert np.array_equal(k1, od.bf16_storage(k1))
            else:
                assert np.max(np.abs(logits - od.lens_logits(shape, weights, hs[e, pos]))) < tol
        s.close(); ref.close(); m.close()
