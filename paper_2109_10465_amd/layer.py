"""Buffer owner and call sequence for one MoE layer step on one GPU.

Holds the device buffers (torch tensors used as raw memory) and issues the
C-ABI calls in the order gate -> capacity/RTS -> dispatch -> experts -> combine
(forward) and its reverse (backward).  No arithmetic happens here.
"""
import torch

from . import binding as B

_TORCH_DT = {B.F32: torch.float32, B.BF16: torch.bfloat16}


class MoELayer:
    def __init__(self, T, d_model, d_ff, E, k, capacity, dtype, act, device="cuda:0", aux_coef=0.0,
                 forward_only=False, groups=1, jitter_eps=0.0, drop_p=0.0):
        if not torch.cuda.is_available():
            raise B.MoeError("MoELayer needs a GPU; there is no CPU fallback")
        B.lib()
        self.shape = B.make_shape(T, d_model, d_ff, E, k, capacity, dtype, act)
        self.T, self.d, self.f, self.E, self.k, self.C = T, d_model, d_ff, E, k, capacity
        self.device = torch.device(device)
        self.aux_coef = float(aux_coef)     # weight of the balancing loss in the objective (0 = off)
        self.jitter_eps = float(jitter_eps)  # gate jitter (training); the seed is given per step
        self.drop_p = float(drop_p)          # expert dropout on the hidden activation (training)
        self.seed = 0
        self.groups = int(groups)           # > 1: token selection inside groups of T/groups consecutive tokens
        self.forward_only = bool(forward_only)   # evaluation: no saved derivative, no backward buffers
        adt = _TORCH_DT[dtype]
        dev = self.device

        def buf(shape, dt):
            return torch.empty(shape, dtype=dt, device=dev)

        i32, f32 = torch.int32, torch.float32
        self.logits = buf((T, E), f32)
        self.probs = buf((T, E), f32)
        self.expert_idx = buf((T, k), i32)
        self.gate_w = buf((T, k), f32)
        self.slot = buf((T, k), i32)
        self.expert_count = buf((E,), i32)
        self.expert_demand = buf((E,), i32)
        self.slot_src = buf((E, capacity), i32)
        self.first_frac = buf((E,), f32)     # balancing loss: first-choice share, mean probability, value
        self.mean_prob = buf((E,), f32)
        self.aux_loss = buf((1,), f32)
        self.xd = buf((E, capacity, d_model), adt)
        self.h = buf((E, capacity, d_ff), adt)       # act(z)
        self.dact = None if forward_only else buf((E, capacity, d_ff), adt)    # act'(z)
        self.yd = buf((E, capacity, d_model), adt)
        self.y = buf((T, d_model), adt)
        self.utilisation = torch.zeros((E,), dtype=torch.int64, device=dev)   # tokens routed to each expert so far
        nbytes = B.moe_workspace_bytes(self.shape)
        if nbytes == 0:
            raise B.MoeError("unsupported shape")
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        if forward_only:
            return
        # backward
        self.dyd = buf((E, capacity, d_model), adt)
        self.dgate_w = buf((T, k), f32)
        self.dxd = buf((E, capacity, d_model), adt)
        self.dW1 = buf((E, d_model, d_ff), f32)
        self.dW2 = buf((E, d_ff, d_model), f32)
        self.dlogits = buf((T, E), f32)
        self.dWg = buf((d_model, E), f32)
        self.dx = buf((T, d_model), adt)

    def forward(self, x, Wg, bias, W1, W2, rts_keys, logits=None, seed=0):
        """logits: optional precomputed [T,E] fp32 gate logits; the projection call is
        then skipped and routing runs on exactly these values."""
        s = self.shape
        self._saved = (x, Wg, W1, W2)
        self.seed = int(seed)     # of this step's jitter and dropout draws
        if logits is None:
            B.moe_gate_logits_jitter(s, x, Wg, bias, self.jitter_eps, self.seed, self.logits)
        else:
            self.logits.copy_(logits)
        if self.groups > 1:
            B.moe_gate_route_grouped(s, self.groups, self.logits, rts_keys, self.probs, self.expert_idx,
                                     self.gate_w, self.slot, self.expert_count, self.expert_demand,
                                     self.slot_src, self.ws)
        else:
            B.moe_gate_route(s, self.logits, rts_keys, self.probs, self.expert_idx, self.gate_w,
                             self.slot, self.expert_count, self.expert_demand, self.slot_src, self.ws)
        if self.forward_only:
            B.moe_utilisation_accumulate(s, self.expert_demand, self.utilisation)
        if self.aux_coef != 0.0:
            B.moe_aux_loss(s, self.probs, self.expert_idx, self.first_frac, self.mean_prob, self.aux_loss,
                           self.ws)
        B.moe_dispatch_tokens(s, x, self.expert_idx, self.slot, self.xd)    # reads every token row once
        if self.drop_p > 0.0:
            B.moe_expert_ffn_fwd_dropout(s, self.xd, self.expert_count, W1, W2, self.drop_p, self.seed, self.h,
                                         self.dact, self.yd)
        else:
            B.moe_expert_ffn_fwd(s, self.xd, self.expert_count, W1, W2, self.h, self.dact, self.yd)
        B.moe_combine_fwd(s, self.yd, self.expert_idx, self.slot, self.gate_w, self.y)
        return self.y

    def backward(self, dy):
        if self.forward_only:
            raise B.MoeError("this layer was built forward-only")
        s = self.shape
        x, Wg, W1, W2 = self._saved
        B.moe_combine_bwd(s, dy, self.yd, self.expert_idx, self.slot, self.gate_w, self.dyd,
                          self.dgate_w)
        B.moe_expert_ffn_bwd(s, self.dyd, self.xd, self.h, self.dact, self.expert_count, W1, W2,
                             self.dxd, self.dW1, self.dW2, self.ws)
        if self.aux_coef != 0.0:
            B.moe_gate_bwd_aux(s, self.dgate_w, self.probs, self.expert_idx, self.slot, self.first_frac,
                               self.aux_coef, self.dlogits)
        else:
            B.moe_gate_bwd(s, self.dgate_w, self.probs, self.expert_idx, self.slot, self.dlogits)
        # dispatch's backward (combine with unit weights) and the gate projection's backward in one call
        B.moe_dispatch_gate_logits_bwd(s, x, Wg, self.dlogits, self.dxd, self.expert_idx, self.slot,
                                       self.jitter_eps, self.seed,
                                       self.dWg, self.dx, self.ws)
        return self.dx, self.dWg, self.dW1, self.dW2

    def step(self, x, Wg, bias, W1, W2, rts_keys, dy, logits=None, seed=0):
        self.forward(x, Wg, bias, W1, W2, rts_keys, logits, seed)
        return self.backward(dy)

    def capture_step(self, x, Wg, bias, W1, W2, rts_keys, dy, seed=0):
        """Records one forward+backward step into a HIP graph and returns it (`.replay()` runs the step again on
        the same tensors: refill x, dy, the weights and the keys in place between replays).  The library
        allocates nothing and clears nothing with memset, so every call of the step is a plain kernel node.
        Replay takes the host out of the loop; the device time is the same as eager (measured: the chain of
        dependent kernels, not their launch, sets the time of a step even for a 256-token layer).
        The seed of the step's noise draws is a host value and is recorded with the graph."""
        if self.forward_only:
            raise B.MoeError("this layer was built forward-only")
        self.step(x, Wg, bias, W1, W2, rts_keys, dy, seed=seed)       # first use of every kernel happens eagerly
        torch.cuda.synchronize(self.device)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step(x, Wg, bias, W1, W2, rts_keys, dy, seed=seed)
        return graph
