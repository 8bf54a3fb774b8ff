import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_terminal_summary(terminalreporter):
    """After a GPU run: which comparisons needed the library's own projection decisions (and how
    far from a face the farthest of them was), and the worst error of every output in units of
    its tolerance."""
    try:
        from tests import gpu_util
    except Exception:
        return
    tr = terminalreporter
    if gpu_util.WORST:
        tr.write_sep("-", "parity: worst |err| / tolerance per output")
        for key in sorted(gpu_util.WORST):
            tr.write_line(f"  {key:32s} {gpu_util.WORST[key]:.3f}")
    if gpu_util.MASK_REPORT:
        tr.write_sep("-", "parity: comparisons that used the library's own projection decisions")
        for r in gpu_util.MASK_REPORT:
            tr.write_line(f"  {r['test']}: {r['differ']} of {r['decisions']} decisions differ, "
                          f"farthest {r['max_distance']:.2e} from a face")
    elif gpu_util.WORST:
        tr.write_line("parity: every projection decision agreed with the oracle's")
