"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code, CPU only): a driver
(oracle/sanitize_check.c) includes the oracle's source unchanged and walks every entry point on a
tiny model in six schedule configurations, for the fp32 build and its fp64 twin."""
import pytest

from oracle import build_oracle


@pytest.mark.parametrize("kind", ["f32", "f64"])
def test_oracle_runs_clean_under_sanitizers(kind):
    r = build_oracle.run_sanitized(kind)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "sanitize_check: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
