"""CPU-only: the oracle rebuilt with the undefined-behaviour sanitizer passes all its pins without a
single report (signed overflow, misaligned or out-of-bounds access through its own indexing, bad shifts)."""
import os
import subprocess
import sys
import textwrap

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pins_under_ubsan(tmp_path):
    so = str(tmp_path / "liboracle_ubsan.so")
    script = textwrap.dedent(f"""
        import sys
        sys.path.insert(0, {ROOT!r}); sys.path.insert(0, {os.path.join(ROOT, 'tests')!r})
        import oracle, pins
        oracle.build(extra_flags=["-fsanitize=undefined", "-fsanitize=bounds-strict", "-g"], out_path={so!r})
        L = oracle.lib({so!r})
        for pin in pins.ALL_PINS:
            pin(oracle, L)
        print("pins ok")
    """)
    r = subprocess.run([sys.executable, "-c", script], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "pins ok" in r.stdout
    assert "runtime error" not in r.stderr, r.stderr[-2000:]
