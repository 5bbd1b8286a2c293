"""ctypes binding of libmoe_hip.so: same names as the C ABI (include/moe_hip.h).

Argument marshalling only.  Tensors are torch CUDA tensors used as device
memory; every call enqueues on torch's current stream unless `stream` is given.
There is no fallback: if the library has not been built, importing a symbol
raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_hip.so")

F32, BF16 = 0, 1
RELU, GELU = 0, 1

EXPORTS = [
    "moe_status_string", "moe_capacity", "moe_workspace_bytes", "moe_gate_logits", "moe_gate_route",
    "moe_dispatch", "moe_expert_ffn_fwd", "moe_combine_fwd", "moe_combine_bwd", "moe_expert_ffn_bwd",
    "moe_gate_bwd", "moe_gate_logits_bwd", "moe_aux_loss", "moe_gate_bwd_aux",
    "moe_utilisation_accumulate", "moe_gate_route_grouped",
    "moe_gate_logits_jitter", "moe_gate_logits_bwd_jitter", "moe_expert_ffn_fwd_dropout",
    "moe_dispatch_gate_logits_bwd", "moe_microbench_mfma_bf16",
    "moe_gate_route_static", "moe_gate_route_static_max_bytes", "moe_dispatch_tokens",
]


class MoeShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("T", "d_model", "d_ff", "E", "k", "capacity", "dtype", "act")]


class MoeError(RuntimeError):
    pass


_lib = None


def lib():
    """The loaded library; built with `python -m paper_2109_10465_amd.build`."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MoeError(f"{LIB_PATH} is missing: build it with `python -m paper_2109_10465_amd.build`")
        # torch first: the process must hold ONE HIP runtime, the one torch's streams
        # and allocations belong to; the library then binds to that same runtime
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
        shp = ctypes.POINTER(MoeShape)
        L.moe_status_string.restype = ctypes.c_char_p
        L.moe_status_string.argtypes = [ctypes.c_int]
        L.moe_capacity.restype = i32
        L.moe_capacity.argtypes = [i32, i32, i32, ctypes.c_double]
        L.moe_workspace_bytes.restype = sz
        L.moe_workspace_bytes.argtypes = [shp]
        L.moe_gate_route_static_max_bytes.restype = sz
        L.moe_gate_route_static_max_bytes.argtypes = []
        sigs = {
            "moe_gate_route_static": [shp] + [vp] * 10,
            "moe_gate_logits": [shp] + [vp] * 5,
            "moe_gate_route": [shp] + [vp] * 10 + [sz, vp],
            "moe_dispatch": [shp] + [vp] * 5,
            "moe_dispatch_tokens": [shp] + [vp] * 5,
            "moe_expert_ffn_fwd": [shp] + [vp] * 8,
            "moe_combine_fwd": [shp] + [vp] * 6,
            "moe_combine_bwd": [shp] + [vp] * 8,
            "moe_expert_ffn_bwd": [shp] + [vp] * 11 + [sz, vp],
            "moe_gate_bwd": [shp] + [vp] * 6,
            "moe_gate_logits_bwd": [shp] + [vp] * 6 + [sz, vp],
            "moe_aux_loss": [shp] + [vp] * 6 + [sz, vp],
            "moe_gate_bwd_aux": [shp] + [vp] * 5 + [ctypes.c_float, vp, vp],
            "moe_utilisation_accumulate": [shp, vp, vp, vp],
            "moe_gate_route_grouped": [shp, i32] + [vp] * 10 + [sz, vp],
            "moe_gate_logits_jitter": [shp, vp, vp, vp, ctypes.c_float, ctypes.c_uint64, vp, vp],
            "moe_gate_logits_bwd_jitter": [shp, vp, vp, vp, ctypes.c_float, ctypes.c_uint64, vp, vp, vp, sz, vp],
            "moe_expert_ffn_fwd_dropout": [shp] + [vp] * 4 + [ctypes.c_float, ctypes.c_uint64] + [vp] * 4,
            "moe_dispatch_gate_logits_bwd": [shp] + [vp] * 6 + [ctypes.c_float, ctypes.c_uint64, vp, vp, vp, sz, vp],
            "moe_microbench_mfma_bf16": [i32, i32, i32, vp, vp],
        }
        for name, args in sigs.items():
            fn = getattr(L, name)
            fn.restype = ctypes.c_int
            fn.argtypes = args
        _lib = L
    return _lib


def make_shape(T, d_model, d_ff, E, k, capacity, dtype, act):
    return MoeShape(T, d_model, d_ff, E, k, capacity, dtype, act)


def _p(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(rc, what):
    if rc != 0:
        raise MoeError(f"{what}: {lib().moe_status_string(rc).decode()} ({rc})")


def moe_status_string(status):
    return lib().moe_status_string(status).decode()


def moe_capacity(T, E, k, capacity_factor):
    return lib().moe_capacity(T, E, k, capacity_factor)


def moe_workspace_bytes(shape):
    return lib().moe_workspace_bytes(ctypes.byref(shape))


def moe_gate_logits(shape, x, Wg, bias, logits, stream=None):
    _check(lib().moe_gate_logits(ctypes.byref(shape), _p(x), _p(Wg), _p(bias), _p(logits),
                                 _stream(stream)), "moe_gate_logits")


def moe_gate_route(shape, logits, rts_keys, probs, expert_idx, gate_w, slot, expert_count,
                   expert_demand, slot_src, ws, stream=None):
    _check(lib().moe_gate_route(ctypes.byref(shape), _p(logits), _p(rts_keys), _p(probs),
                                _p(expert_idx), _p(gate_w), _p(slot), _p(expert_count),
                                _p(expert_demand), _p(slot_src), _p(ws),
                                0 if ws is None else ws.numel() * ws.element_size(),
                                _stream(stream)), "moe_gate_route")


def moe_gate_route_static_max_bytes():
    return lib().moe_gate_route_static_max_bytes()


def moe_gate_route_static(shape, logits, rts_keys, probs, expert_idx, gate_w, slot, expert_count,
                          expert_demand, slot_src, stream=None):
    _check(lib().moe_gate_route_static(ctypes.byref(shape), _p(logits), _p(rts_keys), _p(probs),
                                       _p(expert_idx), _p(gate_w), _p(slot), _p(expert_count),
                                       _p(expert_demand), _p(slot_src), _stream(stream)), "moe_gate_route_static")


def moe_gate_route_grouped(shape, n_groups, logits, rts_keys, probs, expert_idx, gate_w, slot, expert_count,
                           expert_demand, slot_src, ws, stream=None):
    _check(lib().moe_gate_route_grouped(ctypes.byref(shape), int(n_groups), _p(logits), _p(rts_keys), _p(probs),
                                        _p(expert_idx), _p(gate_w), _p(slot), _p(expert_count),
                                        _p(expert_demand), _p(slot_src), _p(ws),
                                        0 if ws is None else ws.numel() * ws.element_size(),
                                        _stream(stream)), "moe_gate_route_grouped")


def moe_dispatch(shape, x, slot_src, expert_count, xd, stream=None):
    _check(lib().moe_dispatch(ctypes.byref(shape), _p(x), _p(slot_src), _p(expert_count), _p(xd),
                              _stream(stream)), "moe_dispatch")


def moe_dispatch_tokens(shape, x, expert_idx, slot, xd, stream=None):
    _check(lib().moe_dispatch_tokens(ctypes.byref(shape), _p(x), _p(expert_idx), _p(slot), _p(xd),
                                     _stream(stream)), "moe_dispatch_tokens")


def moe_expert_ffn_fwd(shape, xd, expert_count, W1, W2, h_saved, dact_saved, yd, stream=None):
    _check(lib().moe_expert_ffn_fwd(ctypes.byref(shape), _p(xd), _p(expert_count), _p(W1), _p(W2),
                                    _p(h_saved), _p(dact_saved), _p(yd), _stream(stream)),
           "moe_expert_ffn_fwd")


def moe_combine_fwd(shape, yd, expert_idx, slot, gate_w, y, stream=None):
    _check(lib().moe_combine_fwd(ctypes.byref(shape), _p(yd), _p(expert_idx), _p(slot), _p(gate_w),
                                 _p(y), _stream(stream)), "moe_combine_fwd")


def moe_combine_bwd(shape, dy, yd, expert_idx, slot, gate_w, dyd, dgate_w, stream=None):
    _check(lib().moe_combine_bwd(ctypes.byref(shape), _p(dy), _p(yd), _p(expert_idx), _p(slot),
                                 _p(gate_w), _p(dyd), _p(dgate_w), _stream(stream)),
           "moe_combine_bwd")


def moe_expert_ffn_bwd(shape, dyd, xd, h_saved, dact_saved, expert_count, W1, W2, dxd, dW1, dW2, ws,
                       stream=None):
    _check(lib().moe_expert_ffn_bwd(ctypes.byref(shape), _p(dyd), _p(xd), _p(h_saved), _p(dact_saved),
                                    _p(expert_count), _p(W1), _p(W2), _p(dxd), _p(dW1), _p(dW2),
                                    _p(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                    _stream(stream)), "moe_expert_ffn_bwd")


def moe_gate_bwd(shape, dgate_w, probs, expert_idx, slot, dlogits, stream=None):
    _check(lib().moe_gate_bwd(ctypes.byref(shape), _p(dgate_w), _p(probs), _p(expert_idx), _p(slot),
                              _p(dlogits), _stream(stream)), "moe_gate_bwd")


def moe_aux_loss(shape, probs, expert_idx, first_frac, mean_prob, loss, ws, stream=None):
    _check(lib().moe_aux_loss(ctypes.byref(shape), _p(probs), _p(expert_idx), _p(first_frac), _p(mean_prob),
                              _p(loss), _p(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                              _stream(stream)), "moe_aux_loss")


def moe_gate_bwd_aux(shape, dgate_w, probs, expert_idx, slot, first_frac, aux_coef, dlogits, stream=None):
    _check(lib().moe_gate_bwd_aux(ctypes.byref(shape), _p(dgate_w), _p(probs), _p(expert_idx), _p(slot),
                                  _p(first_frac), float(aux_coef), _p(dlogits), _stream(stream)),
           "moe_gate_bwd_aux")


def moe_gate_logits_jitter(shape, x, Wg, bias, jitter_eps, seed, logits, stream=None):
    _check(lib().moe_gate_logits_jitter(ctypes.byref(shape), _p(x), _p(Wg), _p(bias), float(jitter_eps), int(seed),
                                        _p(logits), _stream(stream)), "moe_gate_logits_jitter")


def moe_gate_logits_bwd_jitter(shape, x, Wg, dlogits, jitter_eps, seed, dWg, dx_accum, ws, stream=None):
    _check(lib().moe_gate_logits_bwd_jitter(ctypes.byref(shape), _p(x), _p(Wg), _p(dlogits), float(jitter_eps),
                                            int(seed), _p(dWg), _p(dx_accum), _p(ws),
                                            0 if ws is None else ws.numel() * ws.element_size(),
                                            _stream(stream)), "moe_gate_logits_bwd_jitter")


def moe_dispatch_gate_logits_bwd(shape, x, Wg, dlogits, dxd, expert_idx, slot, jitter_eps, seed, dWg, dx, ws,
                                 stream=None):
    _check(lib().moe_dispatch_gate_logits_bwd(ctypes.byref(shape), _p(x), _p(Wg), _p(dlogits), _p(dxd),
                                              _p(expert_idx), _p(slot),
                                              float(jitter_eps), int(seed), _p(dWg), _p(dx), _p(ws),
                                              0 if ws is None else ws.numel() * ws.element_size(),
                                              _stream(stream)), "moe_dispatch_gate_logits_bwd")


def moe_microbench_mfma_bf16(n_workgroups, iters, random_operands, out, stream=None):
    _check(lib().moe_microbench_mfma_bf16(int(n_workgroups), int(iters), int(bool(random_operands)), _p(out),
                                          _stream(stream)), "moe_microbench_mfma_bf16")


def moe_expert_ffn_fwd_dropout(shape, xd, expert_count, W1, W2, drop_p, seed, h_saved, dact_saved, yd,
                               stream=None):
    _check(lib().moe_expert_ffn_fwd_dropout(ctypes.byref(shape), _p(xd), _p(expert_count), _p(W1), _p(W2),
                                            float(drop_p), int(seed), _p(h_saved), _p(dact_saved), _p(yd),
                                            _stream(stream)), "moe_expert_ffn_fwd_dropout")


def moe_utilisation_accumulate(shape, counts, accum, stream=None):
    _check(lib().moe_utilisation_accumulate(ctypes.byref(shape), _p(counts), _p(accum), _stream(stream)),
           "moe_utilisation_accumulate")


def moe_gate_logits_bwd(shape, x, Wg, dlogits, dWg, dx_accum, ws, stream=None):
    _check(lib().moe_gate_logits_bwd(ctypes.byref(shape), _p(x), _p(Wg), _p(dlogits), _p(dWg),
                                     _p(dx_accum), _p(ws),
                                     0 if ws is None else ws.numel() * ws.element_size(),
                                     _stream(stream)), "moe_gate_logits_bwd")
