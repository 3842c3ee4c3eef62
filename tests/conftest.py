import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _keep_freed_memory():
    """The fp64 oracle allocates and frees arrays of hundreds of megabytes per layer; by default
    glibc maps and unmaps each of them, and touching fresh pages costs more than the arithmetic.
    Keep freed blocks in the heap instead (M_MMAP_THRESHOLD, M_TRIM_THRESHOLD)."""
    try:
        import ctypes
        libc = ctypes.CDLL("libc.so.6")
        libc.mallopt(-3, 2 ** 31 - 1)
        libc.mallopt(-1, 2 ** 31 - 1)
    except Exception:
        pass


_keep_freed_memory()


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def read_golden(name):
    """key = value lines of a fixture under tests/golden/ ('#' starts a comment)."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = line.split("=", 1)
            out[k.strip()] = v.strip()
    return out
