"""Helpers shared by the GPU parity tests: upload seeded inputs, run the HIP
layer through the C ABI, download results, compare against the CPU oracle."""
import numpy as np
import torch

from oracle import moe_oracle as O
from paper_2109_10465_amd import binding as B
from paper_2109_10465_amd import inputs as I
from paper_2109_10465_amd.layer import MoELayer

TOL = {I.F32: 1e-5, I.BF16: 2e-2}     # rel-L2 bounds on outputs and gradients
INT_NAMES = ["expert_idx", "slot", "expert_count", "expert_demand", "slot_src"]


def to_dev(a, dtype):
    """fp32 numpy array -> device tensor in the activation dtype (values are
    already bf16-representable for bf16 workloads, so this is exact)."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if dtype == I.BF16 else t


def host(t):
    return t.detach().float().cpu().numpy() if t.dtype.is_floating_point else t.detach().cpu().numpy()


def rel_l2(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    den = np.linalg.norm(want)
    num = np.linalg.norm(got - want)
    return num / den if den > 0 else num


def run_layer(w, d, use_keys=True):
    """One forward+backward of workload w on the GPU; returns (layer, dict of
    host arrays) with the same names the oracle uses."""
    layer = MoELayer(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act)
    x, dy = to_dev(d["x"], w.dtype), to_dev(d["dy"], w.dtype)
    W1, W2 = to_dev(d["W1"], w.dtype), to_dev(d["W2"], w.dtype)
    Wg = to_dev(d["Wg"], I.F32)
    bias = to_dev(d["bias"], I.F32)
    keys = to_dev(d["rts_keys"], I.F32) if use_keys else None
    print(f"[gpu] {w.name}: T={w.T} d={w.d_model} f={w.d_ff} E={w.E} k={w.k} C={w.capacity} "
          f"dtype={w.dtype} keys={use_keys}", flush=True)
    layer.step(x, Wg, bias, W1, W2, keys, dy)
    torch.cuda.synchronize()
    names = ["logits", "probs", "expert_idx", "gate_w", "slot", "expert_count", "expert_demand",
             "slot_src", "xd", "z", "h", "yd", "y", "dyd", "dgate_w", "dxd", "dW1", "dW2",
             "dlogits", "dWg", "dx"]
    out = {n: host(getattr(layer, n)) for n in names}
    return layer, out


def row_mask(count, C):
    """[E,C] mask of the rows in use."""
    return np.arange(C)[None, :] < np.asarray(count)[:, None]


def check_full(w, d, got, use_keys=True):
    """Element-by-element parity of every output against the oracle.  Routing
    is checked bit-exactly given the GPU's own fp32 logits; floats by rel-L2."""
    tol = TOL[w.dtype]
    keys = d["rts_keys"] if use_keys else None
    ref_logits = O.gate_logits(d["x"], d["Wg"], d["bias"])
    assert rel_l2(got["logits"], ref_logits) <= 1e-5
    ref = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], keys, d["dy"], w.k, w.capacity,
                      w.act, logits=got["logits"])
    for n in INT_NAMES:
        assert np.array_equal(got[n], ref[n]), n
    errs = {}
    for n in ["probs", "gate_w"]:
        errs[n] = rel_l2(got[n], ref[n])
        assert errs[n] <= 1e-5, (n, errs[n])
    m = row_mask(ref["expert_count"], w.capacity)
    pairs = [("xd", "Xd"), ("z", "Z"), ("h", "H"), ("yd", "Yd"), ("dyd", "dYd"), ("dxd", "dXd")]
    for g, r in pairs:
        errs[g] = rel_l2(got[g][m], ref[r][m])
        assert errs[g] <= tol, (g, errs[g])
    assert np.array_equal(got["xd"][m], d["x"][ref["slot_src"][m] // w.k])     # bit copies
    for n in ["y", "dgate_w", "dW1", "dW2", "dlogits", "dWg", "dx"]:
        errs[n] = rel_l2(got[n], ref[n])
        assert errs[n] <= tol, (n, errs[n])
    dropped = np.all(ref["slot"] < 0, axis=1)
    assert not got["y"][dropped].any()
    assert not got["dlogits"][dropped].any() and not got["dx"][dropped].any()
    return ref, errs
