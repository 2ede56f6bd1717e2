"""Pins for the oracle's scheduler (Sec. IV-B.1) and depth statistics (Eq. 4): values the paper
prints, closed forms, and the statements the paper makes in prose."""
import itertools
import pathlib

import numpy as np
import pytest

import workloads as wl
from oracle import binding as ob

GOLDEN = pathlib.Path(__file__).parent / "golden" / "table2_exit_layers.txt"


def shape_with_layers(L):
    return wl.TINY.shape.replace(n_layers=L)


def run(L, e, K, phase, scope, nt, ns, n, off=0):
    sched = wl.Schedule(e, K, phase, scope, nt, ns)
    return ob.schedule_run(shape_with_layers(L), sched, n, off)


def golden_rows():
    rows = []
    for line in GOLDEN.read_text().splitlines():
        if not line.strip() or line.startswith("#"):
            continue
        f = line.split()
        rows.append((f[0], *map(int, f[1:7]), float(f[7]), float(f[8]), float(f[9])))
    return rows


@pytest.mark.parametrize("row", golden_rows(), ids=lambda r: r[0])
def test_table2_exit_layer_column(row):
    name, L, e, K, phase, nt, ns, mean_depth, saving, tol = row
    cycles = 50
    depth, is_text = run(L, e, K, phase, wl.SCOPE_CHUNK, nt, ns, cycles * (nt + ns))
    speech = depth[is_text == 0]
    assert len(speech) == cycles * ns
    assert abs(speech.mean() - mean_depth) <= tol, (name, speech.mean())
    # text column of the table: full depth at every text position
    assert np.all(depth[is_text == 1] == L)
    got_saving = ob.layer_saving(speech, L)
    assert abs(got_saving - saving) <= 0.5 + 1e-9 + 100 * tol / L, (name, got_saving)


def test_table2_text_exit_layer_row():
    """row G10: the periodic rule on text positions, speech at full depth"""
    path = GOLDEN.parent / "table2_text_exit_layers.txt"
    for line in path.read_text().splitlines():
        if not line.strip() or line.startswith("#"):
            continue
        f = line.split()
        L, e, kt, pt, nt, ns, scope = map(int, f[1:8])
        want, tol = float(f[8]), float(f[9])
        sched = wl.Schedule(e, 1, 0, scope, nt, ns, text_period_k=kt, text_phase=pt)
        depth, is_text = ob.schedule_run(shape_with_layers(L), sched, 40 * (nt + ns))
        assert np.all(depth[is_text == 0] == L)                 # speech column: 40
        assert abs(depth[is_text == 1].mean() - want) <= tol, (f[0], depth[is_text == 1].mean())


def brute_force_schedule(L, e, K, phase, kt, pt, scope, nt, ns, n, off):
    """the rule of Sec. IV-B.1 written out slot by slot, for both modalities"""
    pattern = ["t"] * nt + ["s"] * ns
    depth, is_text = [], []
    seen = {"t": 0, "s": 0}       # positions of each modality emitted so far
    for g in range(n):
        kind = pattern[(g + off) % len(pattern)]
        # the index inside the chunk is the slot's own (a sequence may enter the cycle mid-chunk)
        slot = (g + off) % len(pattern)
        idx_chunk = slot if kind == "t" else slot - nt
        idx = idx_chunk if scope == wl.SCOPE_CHUNK else seen[kind]
        period, ph = (kt, pt) if kind == "t" else (K, phase)
        if kind == "t" and kt <= 1:
            full = True
        else:
            full = e == L or period == 1 or idx % period == ph
        depth.append(L if full else e)
        is_text.append(1 if kind == "t" else 0)
        seen[kind] += 1
    return np.array(depth), np.array(is_text)


def test_schedule_against_brute_force_both_modalities():
    rng = np.random.default_rng(7)
    L = 12
    checked = 0
    for _ in range(300):
        e = int(rng.integers(1, L + 1))
        K, kt = int(rng.integers(1, 6)), int(rng.integers(0, 5))
        phase = int(rng.integers(0, K))
        pt = int(rng.integers(0, max(kt, 1)))
        nt, ns = int(rng.integers(0, 6)), int(rng.integers(0, 8))
        if nt + ns == 0:
            continue
        scope = int(rng.integers(0, 2))
        off = int(rng.integers(0, nt + ns))
        sched = wl.Schedule(e, K, phase, scope, nt, ns, text_period_k=kt, text_phase=pt)
        res = ob.schedule_run(shape_with_layers(L), sched, 5 * (nt + ns) + 3, off)
        want_d, want_t = brute_force_schedule(L, e, K, phase, kt, pt, scope, nt, ns,
                                              5 * (nt + ns) + 3, off)
        if res is None:
            # refused: counters restart per chunk and the cycle has no full-depth slot, or its
            # longest run of early exits does not fit the pending buffer
            assert scope == wl.SCOPE_CHUNK and e < L
            d0, _ = brute_force_schedule(L, e, K, phase, kt, pt, scope, nt, ns, 2 * (nt + ns), 0)
            runs = "".join("f" if x == L else "e" for x in d0).split("f")
            cap = 2 * K + (2 * kt if kt > 1 else 0)
            assert not (d0 == L).any() or max(len(r) for r in runs) + 1 > cap
            continue
        assert list(res[0]) == list(want_d) and list(res[1]) == list(want_t)
        checked += 1
    assert checked > 150


def test_text_policy_closed_forms():
    L, e = 12, 5
    for kt, nt, ns in itertools.product([2, 3, 4], [1, 3, 13], [2, 4]):
        for pt in range(kt):
            sched = wl.Schedule(e, 1, 0, wl.SCOPE_STREAM, nt, ns, text_period_k=kt, text_phase=pt)
            depth, is_text = ob.schedule_run(shape_with_layers(L), sched, kt * 6 * (nt + ns))
            text = depth[is_text == 1]
            assert len(text) % kt == 0
            assert text.mean() == pytest.approx(((kt - 1) * e + L) / kt, abs=1e-12)
            assert np.all(depth[is_text == 0] == L)
            sched = sched.replace(scope=wl.SCOPE_CHUNK)
            res = ob.schedule_run(shape_with_layers(L), sched, 6 * (nt + ns))
            depth, is_text = res
            n_full = int(((is_text == 1) & (depth == L)).sum())
            assert n_full == 6 * full_count_closed_form(nt, kt, pt)


def test_named_schedules_patterns():
    """Even / Odd / Triple as spelled out in Sec. IV-B.1, on Step-Audio-2's 4-slot chunk:
    each has two full-depth and two early-exit positions (discussion of schedule variants)."""
    L, e = 28, 22
    pats = {(2, 0): [L, e, L, e], (2, 1): [e, L, e, L], (3, 0): [L, e, e, L]}
    for (K, phase), want in pats.items():
        depth, is_text = run(L, e, K, phase, wl.SCOPE_CHUNK, 1, 4, 15)
        for c in range(3):
            assert is_text[5 * c] == 1 and depth[5 * c] == L
            assert list(depth[5 * c + 1:5 * c + 5]) == want
            assert list(is_text[5 * c + 1:5 * c + 5]) == [0] * 4


def full_count_closed_form(n_slots, K, phase):
    """number of j in [0, n_slots) with j mod K == phase"""
    return (n_slots - 1 - phase) // K + 1 if n_slots > phase else 0


@pytest.mark.parametrize("scope", [wl.SCOPE_CHUNK, wl.SCOPE_STREAM])
def test_full_slot_count_closed_form(scope):
    L, e = 12, 5
    for K, nt, ns in itertools.product([1, 2, 3, 4, 5, 8], [0, 1, 3], [1, 2, 4, 7, 26]):
        for phase in range(K):
            n = 6 * (nt + ns)
            res = run(L, e, K, phase, scope, nt, ns, n)
            if res is None:  # refused: a pure-speech cycle that never reaches a full-depth slot
                assert nt == 0 and scope == wl.SCOPE_CHUNK and K > 1 and phase >= ns
                continue
            depth, is_text = res
            n_speech = int((is_text == 0).sum())
            assert n_speech == 6 * ns
            n_full = int(((is_text == 0) & (depth == L)).sum())
            if K == 1:
                assert n_full == n_speech
            elif scope == wl.SCOPE_CHUNK:
                assert n_full == 6 * full_count_closed_form(ns, K, phase)
            else:
                assert n_full == full_count_closed_form(n_speech, K, phase)
            assert set(np.unique(depth)) <= {e, L}
            assert np.all(depth[is_text == 1] == L)


@pytest.mark.parametrize("L,e,K", [(28, 20, 4), (40, 32, 4), (4, 2, 4), (28, 14, 2), (28, 24, 8)])
def test_stream_scope_mean_speech_depth(L, e, K):
    """every K-th speech position is a refresh => mean speech depth ((K-1)e + L)/K over any
    whole number of periods"""
    for nt, ns in [(1, 2), (13, 26), (2, 4), (0, 5)]:
        for phase in (0, K - 1):
            n_cycles = 3 * K
            depth, is_text = run(L, e, K, phase, wl.SCOPE_STREAM, nt, ns, n_cycles * (nt + ns))
            speech = depth[is_text == 0]
            assert len(speech) % K == 0
            assert speech.mean() == pytest.approx(((K - 1) * e + L) / K, abs=1e-12)
            assert ob.layer_saving(speech, L) == pytest.approx(
                (1 - ((K - 1) * e + L) / K / L) * 100, abs=1e-9)


def test_degenerate_configs_are_full_depth():
    for L, e, K in [(28, 28, 4), (28, 20, 1), (4, 4, 1)]:
        depth, _ = run(L, e, K, 0, wl.SCOPE_STREAM, 1, 2, 60)
        assert np.all(depth == L)


def test_cycle_offset_shifts_the_pattern():
    L, e, K, nt, ns = 28, 22, 2, 1, 4
    base_d, base_t = run(L, e, K, 0, wl.SCOPE_CHUNK, nt, ns, 40)
    for off in range(1, 5):
        d, t = run(L, e, K, 0, wl.SCOPE_CHUNK, nt, ns, 30, off)
        assert list(d) == list(base_d[off:off + 30])
        assert list(t) == list(base_t[off:off + 30])


def test_layer_saving_formula():
    # Eq. 4 on hand-made logs
    assert ob.layer_saving(np.array([28, 22, 28, 22]), 28) == pytest.approx((1 - 25 / 28) * 100)
    assert ob.layer_saving(np.array([40] * 7), 40) == 0.0
    assert ob.layer_saving(np.array([10]), 40) == pytest.approx(75.0)
    # benchmark workloads: tiny (whole chunks) 37.5 %, Step shape 21.43 %, GLM shape 15 %
    for w, want in [(wl.TINY, 37.5), (wl.STEP_AUDIO_2_MINI, (1 - 22 / 28) * 100),
                    (wl.GLM_4_VOICE, 15.0)]:
        s = w.schedule
        n = 4 * s.period_k * (s.n_text + s.n_speech)
        depth, is_text = ob.schedule_run(w.shape, s, n)
        assert ob.layer_saving(depth[is_text == 0], w.shape.n_layers) == pytest.approx(want)


def test_refused_configs():
    bad = [dict(exit_layer=0), dict(exit_layer=5), dict(period_k=0), dict(phase=4), dict(phase=-1),
           dict(scope=2), dict(n_text=0, n_speech=0), dict(n_text=-1)]
    for kw in bad:
        s = wl.TINY.schedule.replace(**kw)
        assert ob.schedule_run(wl.TINY.shape, s, 8) is None, kw


# ---------------------------------------------------------------- the text ends before the speech

def brute_force_with_text_budget(L, e, K, phase, scope, nt, ns, n, off, budget):
    """Sec. IV-A: speech is most of a response because the text ends first.  Written out position
    by position from a list of what has been generated: a slot of the cycle is text while fewer
    than `budget` text tokens exist; a speech position's index is its place among all speech
    (stream) or the number of speech positions since the last text one (chunk: the chunk that runs
    when the text ends goes on)."""
    kinds, depth = [], []
    cyc = nt + ns
    for g in range(n):
        slot = (g + off) % cyc
        kind = "t" if slot < nt and kinds.count("t") < budget else "s"
        if kind == "t":
            full = True
        else:
            if scope == wl.SCOPE_STREAM:
                idx = kinds.count("s")
            elif "t" in kinds:
                idx = g - 1 - max(i for i, k in enumerate(kinds) if k == "t")
            else:           # no text yet: the sequence entered the cycle inside a speech chunk
                idx = g + (off % cyc) - nt if (off % cyc) >= nt else g
                # (entered on a text slot with a spent budget cannot happen: budget >= 1)
            full = e == L or K == 1 or idx % K == phase
        kinds.append(kind)
        depth.append(L if full else e)
    return np.array(depth), np.array([1 if k == "t" else 0 for k in kinds])


def test_text_budget_against_brute_force():
    rng = np.random.default_rng(17)
    L, checked, tails = 12, 0, 0
    for _ in range(300):
        e = int(rng.integers(1, L))
        K = int(rng.integers(1, 6))
        phase = int(rng.integers(0, K))
        nt, ns = int(rng.integers(1, 5)), int(rng.integers(1, 8))
        scope = int(rng.integers(0, 2))
        off = int(rng.integers(0, nt + ns))
        budget = int(rng.integers(1, 4 * nt + 2))
        n = 8 * (nt + ns)
        sched = wl.Schedule(e, K, phase, scope, nt, ns)
        res = ob.schedule_run(shape_with_layers(L), sched, n, off, text_budget=budget)
        if res is None:
            continue
        want_d, want_t = brute_force_with_text_budget(L, e, K, phase, scope, nt, ns, n, off, budget)
        assert list(res[1]) == list(want_t), (nt, ns, off, budget)
        assert list(res[0]) == list(want_d), (e, K, phase, scope, nt, ns, off, budget)
        assert res[1].sum() == min(budget, want_t.sum()) == budget      # exactly the budget, then none
        last_text = int(np.flatnonzero(res[1])[-1])
        assert not res[1][last_text + 1:].any()
        tails += int(n - last_text > nt + ns)
        checked += 1
    assert checked > 150 and tails > 100


def test_text_budget_reproduces_the_speech_share_of_the_paper():
    """Sec. IV-A: 79.5 % (Step-Audio-2, 1:2) and 81.2 % (GLM-4-Voice, 13:26) of the generated
    tokens are speech.  The budget that gives that share over a response, and the closed forms of
    the tail: one full-depth position every K in it, mean speech depth from the counts."""
    for (nt, ns, L, e, share, n) in [(1, 2, 28, 20, 0.795, 1024), (13, 26, 40, 32, 0.812, 1024)]:
        budget = round((1.0 - share) * n)
        K, phase = 4, 3
        for scope in (wl.SCOPE_STREAM, wl.SCOPE_CHUNK):
            sched = wl.Schedule(e, K, phase, scope, nt, ns)
            depth, is_text = ob.schedule_run(shape_with_layers(L), sched, n, 0, text_budget=budget)
            assert is_text.sum() == budget
            assert abs((1 - is_text.mean()) - share) < 0.5 / n + 1e-12
            speech = depth[is_text == 0]
            last_text = int(np.flatnonzero(is_text)[-1])
            tail = depth[last_text + 1:]
            full_at = np.flatnonzero(tail == L)
            assert len(full_at) >= 3 and np.all(np.diff(full_at) == K)      # periodic refresh goes on
            if scope == wl.SCOPE_STREAM:
                S = len(speech)
                n_full = (S - 1 - phase) // K + 1                             # j = phase, phase + K, ...
                assert (speech == L).sum() == n_full
                assert speech.mean() == pytest.approx((n_full * L + (S - n_full) * e) / S, abs=1e-12)
            else:
                assert full_at[0] == phase                                    # the tail's chunk index starts at 0
    # an unlimited budget is the plain cycle
    sched = wl.Schedule(20, 4, 3, wl.SCOPE_CHUNK, 1, 2)
    a = ob.schedule_run(shape_with_layers(28), sched, 60, 1)
    b = ob.schedule_run(shape_with_layers(28), sched, 60, 1, text_budget=0)
    c = ob.schedule_run(shape_with_layers(28), sched, 60, 1, text_budget=10 ** 6)
    assert list(a[0]) == list(b[0]) == list(c[0]) and list(a[1]) == list(c[1])


# ---------------------------------------------------------------- a phase that moves

def test_moved_phase_against_brute_force():
    """Table II: the phase is a free choice (Even / Odd / Triple).  A sequence's phase may be
    moved for its future speech positions; written out from lists: the rule with the phase that
    is in force at each position."""
    rng = np.random.default_rng(29)
    L, checked = 12, 0
    for _ in range(200):
        e = int(rng.integers(1, L))
        K = int(rng.integers(2, 6))
        nt, ns = int(rng.integers(1, 4)), int(rng.integers(1, 9))
        scope = int(rng.integers(0, 2))
        off = int(rng.integers(0, nt + ns))
        n = 7 * (nt + ns)
        steps = sorted(int(x) for x in rng.integers(0, n, size=int(rng.integers(1, 4))))
        moves = [(s, int(rng.integers(0, K))) for s in steps]
        sched = wl.Schedule(e, K, int(rng.integers(0, K)), scope, nt, ns)
        base = ob.schedule_run(shape_with_layers(L), sched, n, off)
        if base is None:
            continue
        got = ob.schedule_run_moves(shape_with_layers(L), sched, n, moves, off)
        speech_seen, phase = 0, sched.phase
        for g in range(n):
            for s, p in moves:
                if s <= g:
                    phase = p       # the last move at or before g wins (moves are ascending)
            slot = (g + off) % (nt + ns)
            if slot < nt:
                assert got[1][g] == 1 and got[0][g] == L
            else:
                idx = slot - nt if scope == wl.SCOPE_CHUNK else speech_seen
                assert got[1][g] == 0 and got[0][g] == (L if idx % K == phase else e), (g, moves)
                speech_seen += 1
        checked += 1
    assert checked > 100


def test_aligned_phases_make_full_depth_steps_coincide():
    """The alignment a batch scheduler wants: every sequence gets phase (j + K - 1) mod K, j its
    speech count so far.  From then on, sequences that generate speech only run full depth on the
    same steps, every K-th; the run of early exits joined by the move stays within 2K - 2."""
    L, e, K = 28, 20, 4
    sched = wl.Schedule(e, K, 3, wl.SCOPE_STREAM, 1, 2)
    n, at = 120, 50
    rows = []
    for off, budget in [(0, 5), (1, 9), (2, 3), (1, 12)]:
        d0, t0 = ob.schedule_run(shape_with_layers(L), sched, n, off, text_budget=budget)
        assert not t0[at - 6:].any()                       # every sequence is in its speech tail by then
        j = int((t0[:at] == 0).sum())                      # speech positions before step `at`
        d, t = ob.schedule_run_moves(shape_with_layers(L), sched, n, [(at, (j + K - 1) % K)], off, text_budget=budget)
        assert np.array_equal(d[:at], d0[:at]) and np.array_equal(t, t0)
        rows.append(d[at:])
        ee_runs = "".join("f" if x == L else "e" for x in d).split("f")
        assert max(len(r) for r in ee_runs) <= 2 * K - 2
    rows = np.array(rows)
    assert np.all(rows == rows[0])                          # the same steps for all four
    full = np.flatnonzero(rows[0] == L)
    assert full[0] == K - 1 and np.all(np.diff(full) == K)
