"""The C-ABI library loads without a GPU, exports every symbol the header
declares, and its host-only entry points behave as documented.  No kernel is
launched here."""
import ctypes
import os
import re

import pytest

from oracle import moe_oracle as O
from paper_2109_10465_amd import binding as B
from paper_2109_10465_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    """Every function declared in include/*.h (the layer's ABI and the measurement aid's header)."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, fn)).read(), flags=re.S)
            names |= set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_symbols()
    assert len(names) >= 14
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names
    for n in names:
        assert callable(getattr(B, n))


def test_capacity_rule_matches_oracle_and_workloads():
    for w in I.WORKLOADS.values():
        assert B.moe_capacity(w.T, w.E, w.k, w.capacity_factor) == w.capacity
    for T, E, k, cf in [(10, 4, 1, 1.0), (1, 64, 1, 1.0), (100, 8, 2, 2.0), (4096, 8, 2, 1.25),
                        (777, 5, 2, 1.1), (33, 7, 1, 0.5)]:
        assert B.moe_capacity(T, E, k, cf) == O.capacity(T, E, k, cf)
    assert B.moe_capacity(0, 4, 1, 1.0) == -1
    assert B.moe_capacity(16, 4, 3, 1.0) == -1
    assert B.moe_capacity(16, 4, 1, -1.0) == -1


def test_workspace_query_and_shape_validation():
    for w in I.WORKLOADS.values():
        s = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act)
        n = B.moe_workspace_bytes(s)
        assert n > 0 and n % 256 == 0
        # at least the backward's dz buffer
        assert n >= w.E * w.capacity * w.d_ff * (2 if w.dtype == I.BF16 else 4)
    bad = [
        B.make_shape(64, 12, 16, 4, 1, 16, 0, 0),     # d_model % 8
        B.make_shape(64, 16, 16, 4, 3, 16, 0, 0),     # k
        B.make_shape(64, 16, 16, 1, 2, 16, 0, 0),     # E < k
        B.make_shape(64, 16, 16, 300, 1, 16, 0, 0),   # E > 256
        B.make_shape(0, 16, 16, 4, 1, 16, 0, 0),      # T
        B.make_shape(64, 16, 16, 4, 1, 0, 0, 0),      # capacity
        B.make_shape(64, 16, 16, 4, 1, 16, 5, 0),     # dtype
        B.make_shape(64, 16, 16, 4, 1, 16, 0, 9),     # act
    ]
    for s in bad:
        assert B.moe_workspace_bytes(s) == 0


def test_argument_errors_are_reported_before_any_launch():
    # invalid shapes / NULL pointers return an error code on the host; nothing
    # touches a device, so this runs without one
    L = B.lib()
    bad = B.make_shape(64, 12, 16, 4, 1, 16, 0, 0)
    assert L.moe_gate_logits(ctypes.byref(bad), None, None, None, None, None) == -2
    ok = B.make_shape(64, 16, 16, 4, 1, 16, 0, 0)
    assert L.moe_gate_logits(ctypes.byref(ok), None, None, None, None, None) == -1
    assert L.moe_dispatch(ctypes.byref(ok), None, None, None, None, None) == -1
    assert L.moe_gate_bwd(None, None, None, None, None, None, None) == -1
    baddt = B.make_shape(64, 16, 16, 4, 1, 16, 7, 0)
    assert L.moe_combine_fwd(ctypes.byref(baddt), None, None, None, None, None, None) == -3
    assert B.moe_status_string(0) == "ok"
    assert "workspace" in B.moe_status_string(-4)
    with pytest.raises(B.MoeError):
        B._check(-2, "x")


def test_build_rejects_scratch_in_kernels_with_hand_issued_loads():
    """A kernel that issues loads through inline asm and waits for them by hand must not spill: the build reads the
    compiler's resource-usage remarks and fails if such a kernel reports scratch memory."""
    from paper_2109_10465_amd import build as bld
    remark = ("gate.hip:1:1: remark: Function Name: _Z22gate_logits_lds_kernelILi4EEviiiPKtPKfS3_Pf [-Rpass-analysis]\n"
              "gate.hip:1:1: remark:     VGPRs: 168 [-Rpass-analysis]\n"
              "gate.hip:1:1: remark:     ScratchSize [bytes/lane]: {n} [-Rpass-analysis]\n")
    bld.check_no_scratch("gate.hip", remark.format(n=0))
    with pytest.raises(RuntimeError):
        bld.check_no_scratch("gate.hip", remark.format(n=28))
    # other kernels of the same file may spill
    bld.check_no_scratch("gate.hip", remark.format(n=28).replace("gate_logits_lds_kernel", "gate_dx_kernel"))


def test_static_routing_scratch_holds_the_shape_the_header_names():
    """moe_hip.h promises that the built-in scratch of moe_gate_route_static is enough for T = 65536, k = 2 with any
    E <= 256.  With tiny d_model, d_ff and capacity the routing workspace is the largest one, so the general
    workspace size is the routing workspace size (host-only calls)."""
    B.lib()
    cap = B.moe_gate_route_static_max_bytes()
    for E in (2, 32, 64, 65, 128, 129, 256):
        s = B.make_shape(65536, 8, 8, E, 2, 1, 0, 0)
        assert 0 < B.moe_workspace_bytes(s) <= cap, E
    assert B.moe_workspace_bytes(B.make_shape(1 << 21, 8, 8, 256, 2, 1, 0, 0)) > cap
