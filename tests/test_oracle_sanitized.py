"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code, no GPU):
oracle/sanitize_check.c drives every oracle function on heap blocks of exactly the contracted
sizes; a report of either sanitizer fails the run."""
import subprocess


def test_oracle_runs_clean_under_asan_and_ubsan():
    from oracle import build

    exe = build.build_sanitized()
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stderr[-2000:]
    assert "sanitize ok" in res.stdout
