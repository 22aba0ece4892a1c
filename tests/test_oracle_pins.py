"""CPU-only: the oracle against what the paper and mathematics fix."""
import numpy as np
import pytest

from . import pins
from .conftest import get_similarity, get_workload


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda p: p.__name__)
def test_pin(oracle_lib, pin):
    pin(oracle_lib)


def test_tiny_config_end_to_end(oracle_lib):
    """BASELINE config 1: invariants of the re-routing on the real tiny layer,
    and the planted twins (experts 8-15 ~ experts 0-7) dominate the similarity."""
    o = oracle_lib
    wl = get_workload("tiny")
    sp = wl.spec
    sim = get_similarity("tiny")
    for i in range(8):
        assert np.argsort(-sim[i])[1] == i + 8 and sim[i, i + 8] > 0.8
    off = sim[~np.eye(16, dtype=bool)].reshape(16, 15)
    assert np.sort(off, axis=1)[:, :-1].max() < 0.2
    for S, rho in sp.grid:
        r = o.layer(wl.hidden, wl.router_w, wl.w_gate_up, wl.w_down, None, None, sp.dtype,
                    sp.top_k, sim, S, rho)
        assert r.min_gap > 1e-9
        assert np.array_equal(r.rerouted_ids, o.reroute_per_slot(r.topk_ids, sim, S, rho))
        pins.check_reroute_invariants(r.topk_ids, r.rerouted_ids, sim, S, rho, r.primary_mask,
                                      r.final_set, r.count_before, r.count_after)
        assert r.n_active_after <= r.n_active_before


@pytest.mark.parametrize("name", ["qwen3_b32", "dsv2lite_b64"])
def test_routing_invariants_full_size(oracle_lib, name):
    """Routing half of the full-size bf16 layers (no expert FFN: fast)."""
    o = oracle_lib
    wl = get_workload(name)
    sp = wl.spec
    sim = pins.rand_sim(sp.weight_seed, sp.experts)
    for S, rho in sp.grid + ((sp.top_k, 0.0),):
        r = o.route(wl.hidden, wl.router_w, sp.dtype, sp.top_k, sim, S, rho)
        assert r.min_gap > 1e-9
        assert np.array_equal(r.rerouted_ids, o.reroute_per_slot(r.topk_ids, sim, S, rho))
        pins.check_reroute_invariants(r.topk_ids, r.rerouted_ids, sim, S, rho, r.primary_mask,
                                      r.final_set, r.count_before, r.count_after)
