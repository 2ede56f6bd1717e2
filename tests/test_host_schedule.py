"""The library's own schedule function (the one its dispatch kernel evaluates, a closed form of
the sequence counters) run on the host through the C ABI, against the oracle's scheduler (a state
machine with explicit counters): Sec. IV-B.1 on both modalities, cycle offsets, per-chunk and
stream counters, and the text budget after which a sequence generates speech only (Sec. IV-A).
No GPU is touched."""
import numpy as np
import pytest

import workloads as wl
from oracle import binding as ob
from paper_2603_09215_amd import binding as sb


def test_library_schedule_equals_the_oracles_on_random_configurations():
    rng = np.random.default_rng(23)
    L = 12
    shape = wl.TINY.shape.replace(n_layers=L)
    compared = refused = with_tail = 0
    for _ in range(600):
        e = int(rng.integers(1, L + 1))
        K, kt = int(rng.integers(1, 7)), int(rng.integers(0, 5))
        phase, pt = int(rng.integers(0, K)), int(rng.integers(0, max(kt, 1)))
        nt, ns = int(rng.integers(0, 6)), int(rng.integers(0, 9))
        if nt + ns == 0:
            continue
        scope = int(rng.integers(0, 2))
        off = int(rng.integers(0, 2 * (nt + ns)))
        budget = int(rng.integers(0, 3 * nt + 2)) if nt > 0 and rng.integers(0, 2) else 0
        n = 7 * (nt + ns) + 5
        sched = wl.Schedule(e, K, phase, scope, nt, ns, text_period_k=kt, text_phase=pt)
        want = ob.schedule_run(shape, sched, n, off, text_budget=budget)
        got = sb.schedule_preview(shape, sched, n, off, text_budget=budget)
        assert (want is None) == (got is None), (e, K, phase, kt, pt, scope, nt, ns)
        if want is None:
            refused += 1
            continue
        assert list(got[1]) == list(want[1]), ("modality", e, K, phase, kt, pt, scope, nt, ns, off, budget)
        assert list(got[0]) == list(want[0]), ("depth", e, K, phase, kt, pt, scope, nt, ns, off, budget)
        compared += 1
        with_tail += int(budget > 0 and want[1].sum() == budget)
    assert compared > 400 and refused > 5 and with_tail > 60


@pytest.mark.parametrize("name", ["step_audio_2_mini", "glm_4_voice"])
def test_library_schedule_at_the_benchmark_settings(name):
    w = wl.WORKLOADS[name]
    n = w.decode_len
    for budget in (0, round(0.2 * n)):
        for off in (0, 1, w.schedule.n_text + 3):
            want = ob.schedule_run(w.shape, w.schedule, n, off, text_budget=budget)
            got = sb.schedule_preview(w.shape, w.schedule, n, off, text_budget=budget)
            assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])


def test_library_schedule_refuses_what_it_cannot_run():
    w = wl.TINY
    assert sb.schedule_preview(w.shape, w.schedule.replace(period_k=40, phase=0), 10) is None
    assert sb.schedule_preview(w.shape, w.schedule.replace(n_text=0, n_speech=4), 10, text_budget=2) is None
    assert sb.schedule_preview(w.shape, w.schedule, 10, cycle_offset=-1) is None
