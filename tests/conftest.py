import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_lib():
    import oracle
    return oracle.default()


_workloads = {}
_sims = {}


def get_workload(name, tokens=None):
    """Session cache of generated workloads (the big ones take seconds)."""
    from paper_2602_07616_amd import workloads
    key = (name, tokens)
    if key not in _workloads:
        _workloads[key] = workloads.make_workload(name, tokens=tokens)
    return _workloads[key]


def get_similarity(name):
    """Oracle-computed expert-similarity matrix (fp32) of a named layer."""
    import oracle
    from paper_2602_07616_amd import workloads
    spec = workloads.SPECS[name]
    key = (spec.weight_seed, spec.hidden_seed, spec.experts, spec.hidden, spec.inter,
           spec.calib_batches, spec.calib_tokens, spec.clusters)
    if key not in _sims:
        wl = get_workload(name)
        sim = oracle.similarity_frobenius(wl.calib, wl.w_gate_up, wl.w_down, spec.dtype)
        _sims[key] = sim.astype(np.float32)
    return _sims[key]
