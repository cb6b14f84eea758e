import os
import sys
import time

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    """The CPU checker (compiled on first use)."""
    from oracle import oracle as orc
    orc.build(force=False)
    return orc


@pytest.fixture(scope="session")
def full_checker(request, oracle):
    """full_checker(idx) -> (workload idx at full size, the CPU checker's results for
    every one of its instances).  Computed once per session on all host threads (a
    minute or two for the largest workload) and shared by the full-size tests of
    every form of the solve; progress lines go to the terminal, past the capture."""
    from paper_2407_14843_amd import workloads as wl
    cache = {}
    capman = request.config.pluginmanager.getplugin("capturemanager")

    def say(text):
        if capman is not None:
            with capman.global_and_fixture_disabled():
                print(text, flush=True)
        else:
            print(text, flush=True)

    def get(idx):
        if idx not in cache:
            w = wl.workload(idx)
            threads = min(os.cpu_count() or 1, 16)
            parts, t0, chunk = [], time.time(), 8192
            for lo in range(0, w.n_inst, chunk):
                hi = min(lo + chunk, w.n_inst)
                parts.append(oracle.solve(w.take(np.arange(lo, hi)), threads=threads))
                say(f"[checker] {w.name}: {hi}/{w.n_inst} instances, {time.time() - t0:.0f} s, "
                    f"{threads} threads")
            cache[idx] = (w, tuple(np.concatenate(x) for x in zip(*parts)))
        return cache[idx]

    return get
