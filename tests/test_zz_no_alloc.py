"""The allocation-free routing entry point (built-in device scratch instead of a
caller workspace) against moe_gate_route, through the C ABI: two calls in a
row, the second on a smaller input, every output bit-equal; an input beyond the
built-in scratch is refused on the host."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2109_10465_amd import binding as B
from paper_2109_10465_amd import inputs as I

pytestmark = pytest.mark.gpu

NAMES = ["probs", "expert_idx", "gate_w", "slot", "expert_count", "expert_demand", "slot_src"]


def route_both(T, E, k, C, seed, use_keys=True):
    rng = np.random.default_rng(seed)
    logits = torch.from_numpy((rng.standard_normal((T, E)) * 2.0).astype(np.float32)).cuda()
    keys = torch.from_numpy(rng.random(T, dtype=np.float32)).cuda() if use_keys else None
    s = B.make_shape(T, 64, 64, E, k, C, I.F32, I.RELU)
    i32, f32 = torch.int32, torch.float32

    def outputs():
        # filled with a pattern first: an output the call did not write would show
        mk = lambda shape, dt: torch.full(shape, -7, dtype=dt, device="cuda")
        return dict(probs=mk((T, E), f32), expert_idx=mk((T, k), i32), gate_w=mk((T, k), f32), slot=mk((T, k), i32),
                    expert_count=mk((E,), i32), expert_demand=mk((E,), i32), slot_src=mk((E, C), i32))

    a, b = outputs(), outputs()
    ws = torch.empty(B.moe_workspace_bytes(s), dtype=torch.uint8, device="cuda")
    print(f"[gpu] moe_gate_route_static vs moe_gate_route: T={T} E={E} k={k} C={C} keys={use_keys}", flush=True)
    B.moe_gate_route(s, logits, keys, *[a[n] for n in NAMES], ws)
    B.moe_gate_route_static(s, logits, keys, *[b[n] for n in NAMES])
    torch.cuda.synchronize()
    for n in NAMES:
        assert torch.equal(a[n], b[n]), n
    assert int(b["expert_demand"].sum()) == T * k
    return b


def test_static_scratch_routing_equals_workspace_routing_twice_second_smaller():
    B.lib()
    assert B.moe_gate_route_static_max_bytes() == 5 << 20
    big = route_both(20000, 24, 2, 900, seed=1)             # skewless top-2, drops on most experts, ragged last chunk
    assert (big["slot"] < 0).any()
    small = route_both(777, 5, 1, 100, seed=2)              # smaller: reuses the front of the same scratch
    assert (small["slot"] < 0).any()
    route_both(4096, 128, 2, 70, seed=3, use_keys=False)    # position priority, many experts


def test_static_scratch_refuses_what_does_not_fit():
    B.lib()
    s = B.make_shape(1 << 21, 64, 64, 256, 2, 16384, I.F32, I.RELU)      # needs far more scratch than the array holds
    assert B.moe_workspace_bytes(s) > B.moe_gate_route_static_max_bytes()
    rc = B.lib().moe_gate_route_static(ctypes.byref(s), *([None] * 10))
    assert rc == -4 and "workspace" in B.moe_status_string(rc)
