import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.dirname(os.path.abspath(__file__))
for p_ in (ROOT, HERE):
    if p_ not in sys.path:
        sys.path.insert(0, p_)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_terminal_summary(terminalreporter):
    """One line per oracle-parity case of this run: worst relative error and the ReLU ties it needed."""
    try:
        import parity
    except ImportError:
        return
    if not parity.CASE_RECORDS:
        return
    tr = terminalreporter
    tr.write_line("")
    tr.write_line(f"oracle parity cases of this run ({len(parity.CASE_RECORDS)}; also in {parity.CASE_LOG}):")
    for r in parity.CASE_RECORDS:
        ties = "; ".join(f"it{t['iter']}:" + ",".join(f"{e['step']}{e['layer']}[{e['row']},{e['col']}]|T|/rms={e['abs_over_rms']:.1e}"
                                                      for e in t["entries"]) for t in r["ties"])
        tr.write_line(f"  {r['case']}: {r['iters']} iterations, worst rel err {r['worst']:.2e}, "
                      f"tie iterations {len(r['ties'])}" + (f" ({ties})" if ties else "") +
                      ("" if r["ok"] else "  FAILED"))
