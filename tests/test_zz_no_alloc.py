"""sere_moe_decode_static (the entry point that allocates nothing: its intermediate buffers live
in a device array inside the library) against sere_moe_decode on the same inputs, through the C
ABI: two calls in a row on one GPU, the second on a smaller batch of a smaller layer, so that the
second call finds the first one's leftovers in the shared scratch array."""
import numpy as np
import pytest

from paper_2602_07616_amd import workloads as wk
from . import pins

pytestmark = pytest.mark.gpu

CASES = [
    # dtype, T, d_h, M, K, d_m, shared, S, rho  -- first the larger call, then the smaller one
    (wk.BF16, 96, 1024, 48, 6, 512, 1, 2, 0.0),
    (wk.BF16, 7, 256, 12, 3, 192, 0, 1, 0.3),
]


def test_static_scratch_entry_point_matches_workspace_entry_point():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2602_07616_amd import binding as B, device
    B.load()
    layers = []
    for i, (dtype, T, dh, M, K, dm, n_sh, S, rho) in enumerate(CASES):
        spec = wk.custom_spec(f"static{i}", dtype, dh, M, K, dm, n_sh, T, 4400 + i, clusters=4,
                              calib_batches=1, calib_tokens=4)
        wl = wk.make_workload(spec)
        layer = device.DeviceLayer.from_workload(wl, pins.rand_sim(4400 + i, M), S, rho)
        assert B.sere_workspace_bytes(layer.cfg) <= B.SERE_STATIC_SCRATCH_BYTES
        # the existing entry point, with its caller-owned workspace
        layer.run_decode()
        want_out = layer.out.clone()
        want_route = layer.routing_to_host()
        layers.append((layer, want_out, want_route))
    # two calls in a row through the entry point without a workspace; nothing else in between
    got = []
    for layer, _, _ in layers:
        layer.out.fill_(5.0)
        for name, _ in B.sere_route_out._fields_:
            getattr(layer.route, name).fill_(-3)
        print(f"sere_moe_decode_static T={layer.cfg.num_tokens} M={layer.cfg.num_experts}", flush=True)
        B.sere_moe_decode_static(layer.cfg, layer.hidden, layer.router_w, layer.w_gate_up, layer.w_down,
                                 layer.shared_gate_up, layer.shared_down, layer.sim, layer.out, layer.route)
    torch.cuda.synchronize()
    for layer, want_out, want_route in layers:
        got_route = layer.routing_to_host()
        for k in want_route:
            assert np.array_equal(got_route[k], want_route[k]), k
        # the same kernels on the same inputs: the outputs agree bit for bit, which is inside
        # the output tolerance of the parity tests
        assert (layer.out == want_out).all()
    # a second round in the opposite order (small, then large) gives the same again
    for layer, want_out, _ in reversed(layers):
        layer.out.zero_()
        B.sere_moe_decode_static(layer.cfg, layer.hidden, layer.router_w, layer.w_gate_up, layer.w_down,
                                 layer.shared_gate_up, layer.shared_down, layer.sim, layer.out, None)
        torch.cuda.synchronize()
        assert (layer.out == want_out).all()


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    from paper_2602_07616_amd import binding as B
    B.load()
    cfg = B.make_config(4096, 2048, 128, 8, 768, 0, B.SERE_BF16, 2, 0.0)      # needs far more than 32 MiB
    assert B.sere_workspace_bytes(cfg) > B.SERE_STATIC_SCRATCH_BYTES
    x = torch.zeros(64, device="cuda")
    with pytest.raises(B.SereError) as err:
        B.sere_moe_decode_static(cfg, x, x, x, x, None, None, x, x, None)
    assert err.value.status == B.SERE_ERR_SCRATCH_TOO_SMALL
