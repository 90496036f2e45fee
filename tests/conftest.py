import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
for pth in (ROOT, os.path.join(ROOT, "oracle")):
    if pth not in sys.path:
        sys.path.insert(0, pth)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_terminal_summary(terminalreporter):
    """Code / header mismatch rates of every GPU stream that was compared with the oracle, and whether
    any comparison needed the summation envelope or a second code decision (none may, for calibrated plans)."""
    mod = sys.modules.get("test_gpu_parity")
    rates = getattr(mod, "RATES", None) if mod else None
    if not rates:
        return
    tr = terminalreporter
    tr.write_sep("-", "GPU vs oracle: mismatch rates")
    worst = {}
    for st in rates:
        key = st["label"].split("-job")[0]
        w = worst.setdefault(key, dict(n=0, code=0.0, hdr=0.0, env=False, red=False, bar=st["code_bar"], hbar=st["hdr_bar"]))
        w["n"] += 1
        w["code"] = max(w["code"], st["code_rate"])
        w["hdr"] = max(w["hdr"], st["hdr_rate"])
        w["env"] |= st["envelope"]
        w["red"] |= st["redecided"]
    for key, w in worst.items():
        tr.write_line(f"{key:34s} streams {w['n']:3d}  code max {w['code']:.2e} (bar {w['bar']:.1e})  "
                      f"header max {w['hdr']:.2e} (bar {w['hbar']:.1e})"
                      f"{'  REDECIDED' if w['red'] else ''}")
    tr.write_line(f"streams with a header that differs from the oracle's (each held to the fp32 summation envelope): "
                  f"{sum(s['envelope'] for s in rates)} of {len(rates)}; "
                  f"streams needing a second code decision: {sum(s['redecided'] for s in rates)}")
