import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def parse_golden(name):
    """tests/golden/<name>: '#' comments, then 'key: v v v ...' lines (ints or floats, a/b fractions allowed)."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, vals = line.split(":", 1)
            parsed = []
            for tok in vals.split():
                if "/" in tok:
                    a, b = tok.split("/")
                    parsed.append(float(a) / float(b))
                else:
                    parsed.append(float(tok))
            out[key.strip()] = parsed
    return out


@pytest.fixture(scope="session")
def golden5():
    return parse_golden("five_vertex.txt")


@pytest.fixture(scope="session")
def hgnn():
    """The GPU binding with the library loaded (built first only when nothing is built)."""
    import __graft_entry__ as ge
    ge.ensure_built()
    import paper_2411_01109_amd as mod
    mod.load()
    return mod


@pytest.fixture(scope="session")
def dev():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


def pytest_terminal_summary(terminalreporter):
    """One line per run: how often the norm rule's cancelling branch was taken (tests/parity.py)."""
    try:
        import parity
    except ImportError:
        return
    log = parity.CANCEL_LOG
    worst = max((t[1] for t in log), default=0.0)
    terminalreporter.write_line(f"[parity] cancelling branch of the norm rule taken {len(log)} time(s)"
                                + (f"; largest true rel-L2 it replaced {worst:.3e}" if log else ""))
