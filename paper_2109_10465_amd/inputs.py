"""Seeded synthetic inputs for the MoE-layer workloads.

This module only produces input arrays (numpy, host memory).  It holds none of
the layer's arithmetic and is the one module that both the CPU oracle's tests
and the HIP path's tests/benchmark draw from, so both sides see the same
numbers.  It never touches the GPU library.

The five workloads mirror the shapes the paper trains with (Sec. 4.2: d_model
1024 / d_ff 4096; Table of model sizes: 8..128 experts; Sec. 5.1: top-1 or
top-2, capacity factor 1.0 / 2.0; Sec. 2.3: hidden 2048 with ~8192 tokens per
expert).  They stand in for token streams routed by a trained gate, which are
not available; routing skew is synthesised through a per-expert logit bias.

Random numbers: numpy's counter-based Philox generator, one independent stream
per (seed, tensor name).  Normal draws are fp32; for bf16 workloads activations
and expert weights are rounded to bf16 (nearest-even) and returned widened to
fp32, so both implementations start from identical, bf16-representable values.
"""
import math
import zlib
from dataclasses import dataclass

import numpy as np
from scipy.special import ndtr

RELU, GELU = 0, 1
F32, BF16 = 0, 1


@dataclass(frozen=True)
class Workload:
    name: str
    T: int
    d_model: int
    d_ff: int
    E: int
    k: int
    capacity_factor: float
    capacity: int          # slots per expert, = ceil(k * cf * T / E)
    dtype: int             # F32 or BF16 activations / expert weights
    act: int               # RELU or GELU
    w_std: float           # std of gate and expert weights
    skew: str              # "none" | "hot0" | "zipf"
    skew_param: float      # hot0: top-1 share of expert 0; zipf: exponent


WORKLOADS = {
    "cfg1": Workload("cfg1", 256, 64, 256, 4, 1, 1.0, 64, F32, RELU, 0.02, "none", 0.0),
    "cfg2": Workload("cfg2", 4096, 512, 2048, 8, 2, 1.25, 1280, F32, GELU, 0.02, "hot0", 0.30),
    "cfg3": Workload("cfg3", 16384, 1024, 4096, 32, 2, 1.0, 1024, BF16, GELU, 0.02, "none", 0.0),
    "cfg4": Workload("cfg4", 32768, 1024, 4096, 128, 1, 1.0, 256, BF16, GELU, 0.02, "zipf", 1.1),
    "cfg5": Workload("cfg5", 65536, 2048, 8192, 16, 2, 2.0, 16384, BF16, GELU, 0.01, "none", 0.0),
}


def small(name, T, d_model, d_ff, E, k, capacity, dtype=F32, act=GELU, w_std=0.02,
          skew="none", skew_param=0.0, capacity_factor=float("nan")):
    """An ad-hoc workload for tests (ragged sizes, edge cases)."""
    return Workload(name, T, d_model, d_ff, E, k, capacity_factor, capacity, dtype, act,
                    w_std, skew, skew_param)


def _rng(seed, tensor):
    return np.random.Generator(np.random.Philox(key=[seed, zlib.crc32(tensor.encode())]))


def round_to_bf16(a):
    """fp32 array -> nearest-even bf16 value, returned as fp32 (finite inputs)."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    u = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def _normal(seed, tensor, shape, std, bf16):
    a = _rng(seed, tensor).standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return round_to_bf16(a) if bf16 else a


# ---- routing skew: a per-expert additive logit bias ------------------------
def _norm_cdf(z):
    return ndtr(z)


def _top1_share(bias, sigma, e):
    """P(argmax_e' (n_e' + bias_e') = e) for iid n ~ N(0, sigma^2): the integral
    of phi(z) * prod_{e' != e} Phi(z + (bias_e - bias_e') / sigma) over z."""
    z = np.linspace(-9.0, 9.0, 3601)
    w = np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)
    prod = np.ones_like(z)
    for e2 in range(len(bias)):
        if e2 != e:
            prod *= _norm_cdf(z + (bias[e] - bias[e2]) / sigma)
    return float(np.sum(w * prod) * (z[1] - z[0]))


def _bisect(fn, target, lo, hi):
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if fn(mid) < target:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def gate_bias(w, seed=0):
    """Per-expert logit bias realising the workload's skew, or None.

    hot0: bias = beta * onehot(0), beta chosen so that expert 0 is the top-1
    choice of `skew_param` of the tokens when the unbiased logits are iid
    N(0, sigma^2), sigma = w_std * sqrt(d_model).
    zipf: bias_e = tau * ln q_e with q_e ~ rank_e^-a over a seeded permutation
    of the experts, tau chosen so that the most popular expert's top-1 share
    equals its Zipf mass q_max.
    """
    if w.skew == "none":
        return None
    sigma = w.w_std * math.sqrt(w.d_model)
    if w.skew == "hot0":
        one = np.zeros(w.E)
        one[0] = 1.0
        beta = _bisect(lambda b: _top1_share(b * one, sigma, 0), w.skew_param, 0.0, 20.0 * sigma)
        return (beta * one).astype(np.float32)
    if w.skew == "zipf":
        q = np.arange(1, w.E + 1, dtype=np.float64) ** (-w.skew_param)
        q /= q.sum()
        perm = _rng(seed, "zipf_perm").permutation(w.E)
        lnq = np.empty(w.E)
        lnq[perm] = np.log(q)
        top = int(perm[0])
        tau = _bisect(lambda t: _top1_share(t * lnq, sigma, top), q[0], 0.0, 4.0)
        return (tau * lnq).astype(np.float32)
    raise ValueError(w.skew)


def make_inputs(w, seed=0, with_weights=True):
    """All input arrays of one layer step, as fp32 numpy arrays:
    x[T,d], dy[T,d] ~ N(0,1); Wg[d,E], W1[E,d,f], W2[E,f,d] ~ N(0, w_std);
    rts_keys[T] ~ U[0,1) (fp32); bias[E] or None."""
    bf = w.dtype == BF16
    out = {
        "x": _normal(seed, "x", (w.T, w.d_model), 1.0, bf),
        "dy": _normal(seed, "dy", (w.T, w.d_model), 1.0, bf),
        "Wg": _normal(seed, "Wg", (w.d_model, w.E), w.w_std, False),
        "rts_keys": _rng(seed, "rts_keys").random(w.T, dtype=np.float32),
        "bias": gate_bias(w, seed),
    }
    if with_weights:
        out["W1"] = _normal(seed, "W1", (w.E, w.d_model, w.d_ff), w.w_std, bf)
        out["W2"] = _normal(seed, "W2", (w.E, w.d_ff, w.d_model), w.w_std, bf)
    return out
