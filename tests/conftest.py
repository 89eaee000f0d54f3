import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    # a fresh checkout has no library yet: build it once (an existing one is used as it is)
    import __graft_entry__
    __graft_entry__.ensure_built()


def _gpu_present() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _gpu_present():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def read_golden(name):
    """Parse a tests/golden/*.txt fixture: '#' starts a comment, every other
    non-empty line is 'key: value'.  Returns a dict of raw strings."""
    path = os.path.join(ROOT, "tests", "golden", name)
    out = {}
    with open(path) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, val = line.split(":", 1)
            out[key.strip()] = val.strip()
    return out


def progress(msg: str) -> None:
    """A progress line for long GPU tests: goes to the real stderr (not
    captured by pytest) and, when the results folder of a remote run exists,
    to a log file in it, so that a long test is not mistaken for a hung one."""
    line = f"[progress] {msg}\n"
    try:
        sys.__stderr__.write(line)
        sys.__stderr__.flush()
    except Exception:
        pass
    folder = os.path.join(ROOT, "gpurun_out")
    if os.path.isdir(folder):
        try:
            with open(os.path.join(folder, "test_progress.log"), "a") as fh:
                fh.write(line)
        except Exception:
            pass
