"""CPU oracle for one GPU's Mixture-of-Experts layer, forward and backward.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, fp64 statement of
what the MoE layer computes.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product path (the HIP library
and its Python binding) never does, and it shares no code with that path.

Every function is written from the definition of the operation, in fp64, with
no blocking, fusion or reordering; numpy's matmul is the only library step.
Paper passages followed (arXiv 2109.10465):

  * Sec. 3.1 (Random Token Selection): each expert has a limited capacity; an
    expert chosen by more tokens than its capacity drops the ones "at the end"
    of the flattened [batch*seq] token tensor; RTS replaces position priority
    by a random per-token priority.
  * Sec. 5.1, "MoE setting": top-1 gating (Switch) or top-2 gating (GShard),
    capacity factor 1.0 (train) / 2.0 (eval).
  * Sec. 4.2 (model details): an expert is the transformer feed-forward block,
    d_model -> d_ff -> d_model; pre-LayerNorm residual blocks, so a token that
    is dropped by every chosen expert gets a zero MoE output and is carried by
    the residual connection outside this layer.
  * Sec. 3.2: the gate is one matrix with a column per expert.
  * Sec. 2.3: the compute that matters is the per-expert matmul, whose size is
    hidden size x tokens per expert.

The paper prints no formula for the gate, the capacity or the combine.  The
readings taken here (all listed in the design notes of the repository):

  softmax over the E gate logits; the k experts with the largest *logits*
  (ties -> smaller expert id); k=1 weight = probability of the chosen expert;
  k=2 weights = the two probabilities renormalised to sum to one, before and
  independently of capacity drops; capacity C = max(1, ceil(k*cf*T/E));
  candidates of an expert are ordered by (choice index, RTS key descending,
  token index ascending) and the first C keep their rank as slot; a dropped
  choice contributes nothing forward and receives no gradient; selection and
  slots are constants for differentiation.

Parity pins: every function below is pinned by tests/test_oracle_*.py against
closed forms, brute force on tiny inputs, finite differences, independent
library routines (scipy softmax, torch autograd in fp64) or invariants; none is
"parity unpinned".
"""
import math

import numpy as np
from scipy.special import erf as _erf

RELU = 0
GELU = 1

_F = np.float64


# --------------------------------------------------------------------------
# seeded noise: gate jitter (Sec. 5.1) and expert dropout (Sec. 5.4)
# --------------------------------------------------------------------------
# Both sides of a parity test must draw the same random numbers, so they come
# from a counter-based generator that each implements for itself: Philox4x32
# with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
# as 1, 2, 3", SC 2011).  Element i of a tensor uses word i % 4 of the block with
# counter (i // 4 low word, i // 4 high word, stream, 0) and key (seed low word,
# seed high word); stream 1 = gate jitter, stream 2 = expert dropout.
_PHILOX_M0, _PHILOX_M1 = 0xD2511F53, 0xCD9E8D57
_PHILOX_W0, _PHILOX_W1 = 0x9E3779B9, 0xBB67AE85
STREAM_JITTER, STREAM_DROPOUT = 1, 2


def philox4x32(c0, c1, c2, c3, k0, k1, rounds=10):
    """One Philox4x32 block per counter (arrays of 32-bit words held in uint64);
    returns the four 32-bit output words."""
    m32 = np.uint64(0xFFFFFFFF)
    c0, c1, c2, c3 = (np.asarray(v, np.uint64) & m32 for v in (c0, c1, c2, c3))
    k0, k1 = np.uint64(k0) & m32, np.uint64(k1) & m32
    for _ in range(rounds):
        p0 = np.uint64(_PHILOX_M0) * c0             # 32 x 32 -> 64 bit products
        p1 = np.uint64(_PHILOX_M1) * c2
        c0, c1, c2, c3 = ((p1 >> np.uint64(32)) ^ c1 ^ k0) & m32, p1 & m32, \
                         ((p0 >> np.uint64(32)) ^ c3 ^ k1) & m32, p0 & m32
        k0 = (k0 + np.uint64(_PHILOX_W0)) & m32
        k1 = (k1 + np.uint64(_PHILOX_W1)) & m32
    return c0, c1, c2, c3


def random_words(n, seed, stream):
    """The 32-bit word of elements 0..n-1 (as uint64 array) under the layout above."""
    blocks = np.arange((n + 3) // 4, dtype=np.uint64)
    w = philox4x32(blocks & np.uint64(0xFFFFFFFF), blocks >> np.uint64(32), stream, 0,
                   int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF)
    return np.stack(w, axis=1).reshape(-1)[:n]


def jitter_noise(T, d, eps, seed):
    """Multiplicative jitter on the gate's input (Sec. 5.1: jittering noise on the
    gating input, as in the Switch Transformer): factor 1 + eps (2u - 1) per
    element of x, u = word / 2^32 uniform in [0,1).  Only the gate sees x * noise;
    the experts receive x itself."""
    u = random_words(T * d, seed, STREAM_JITTER).astype(_F) / 4294967296.0
    return (1.0 + eps * (2.0 * u - 1.0)).reshape(T, d)


def dropout_scale(E, C, f, p, seed):
    """Expert dropout (Sec. 5.4: expert dropout of 0.4 in fine-tuning, as in the
    Switch Transformer): dropout on the expert's hidden activation.  Element
    (e, s, c) of the [E, C, f] buffer is dropped when its word < floor(p 2^32);
    kept elements are scaled by 1 / (1 - p).  Returns the scale tensor."""
    w = random_words(E * C * f, seed, STREAM_DROPOUT)
    keep = w >= np.uint64(int(math.floor(p * 4294967296.0)))
    return (keep.astype(_F) / (1.0 - p)).reshape(E, C, f)


# --------------------------------------------------------------------------
# gate: projection, softmax, top-k, weights          (Sec. 3.2, Sec. 5.1)
# --------------------------------------------------------------------------
def gate_logits(x, Wg, bias=None):
    """logits[t,e] = sum_i x[t,i] * Wg[i,e] (+ bias[e]).  Gate matrix with one
    column per expert (Sec. 3.2).  The bias only exists to build skewed
    synthetic gates; the paper's gate has none."""
    l = np.asarray(x, _F) @ np.asarray(Wg, _F)
    if bias is not None:
        l = l + np.asarray(bias, _F)[None, :]
    return l


def softmax(logits):
    """p[t,e] = exp(l[t,e] - max_e l[t,:]) / sum_e exp(l[t,e] - max_e l[t,:])."""
    l = np.asarray(logits, _F)
    z = np.exp(l - l.max(axis=1, keepdims=True))
    return z / z.sum(axis=1, keepdims=True)


def top_k(logits, k):
    """expert_idx[t,0] = argmax_e logits[t,e]; expert_idx[t,1] = argmax over the
    remaining experts.  Equal logits: the smaller expert id wins (numpy's argmax
    returns the first maximum).  The comparison is on the logits exactly as
    given (widening fp32 to fp64 changes neither order nor equality)."""
    l = np.array(logits, _F, copy=True)
    T, E = l.shape
    assert 1 <= k <= 2 and k <= E
    idx = np.empty((T, k), np.int32)
    rows = np.arange(T)
    for j in range(k):
        idx[:, j] = np.argmax(l, axis=1)
        l[rows, idx[:, j]] = -np.inf
    return idx


def gate_weights(p, expert_idx):
    """k=1: g0 = p[t,e0].  k=2: g_j = p[t,e_j] / (p[t,e0] + p[t,e1])."""
    p = np.asarray(p, _F)
    T, k = expert_idx.shape
    sel = np.take_along_axis(p, expert_idx.astype(np.int64), axis=1)
    if k == 1:
        return sel
    return sel / sel.sum(axis=1, keepdims=True)


def capacity(T, E, k, capacity_factor):
    """Slots per expert: max(1, ceil(k * cf * T / E)) (Sec. 5.1 capacity factor;
    Sec. 2.3: tokens per expert depend on batch, experts and top-1 vs top-2)."""
    return max(1, int(math.ceil(float(k) * float(capacity_factor) * T / E)))


# --------------------------------------------------------------------------
# capacity assignment with Random Token Selection            (Sec. 3.1)
# --------------------------------------------------------------------------
def route(expert_idx, rts_keys, E, C):
    """Slot assignment by the counting definition.

    Candidate (t,j) of expert e = expert_idx[t,j] has priority tuple
    (j, -r[t], t); rank(t,j) = number of candidates (t',j') of the same expert
    whose tuple is lexicographically smaller.  slot = rank if rank < C else -1.
    rts_keys None = all keys equal = position priority ("drop the tokens at
    the end", Sec. 3.1); otherwise a larger key means a higher priority.

    Returns slot[T,k], expert_count[E], expert_demand[E], slot_src[E,C]
    (slot_src[e,s] = t*k+j of the candidate holding slot s, -1 if unused).
    """
    expert_idx = np.asarray(expert_idx)
    T, k = expert_idx.shape
    r = np.zeros(T, _F) if rts_keys is None else np.asarray(rts_keys, _F)
    assert r.shape == (T,) and np.all(np.isfinite(r))
    slot = np.full((T, k), -1, np.int32)
    count = np.zeros(E, np.int32)
    demand = np.zeros(E, np.int32)
    slot_src = np.full((E, C), -1, np.int32)
    for e in range(E):
        t_c, j_c = np.nonzero(expert_idx == e)          # candidates of e
        n = t_c.size
        demand[e] = n
        count[e] = min(C, n)
        if n == 0:
            continue
        r_c = r[t_c]
        rank = np.zeros(n, np.int64)
        step = max(1, (1 << 24) // n)                   # bound the n x n table
        for a in range(0, n, step):
            b = min(n, a + step)
            jj, rr, tt = j_c[a:b, None], r_c[a:b, None], t_c[a:b, None]
            before = (j_c[None, :] < jj) | (
                (j_c[None, :] == jj) & ((r_c[None, :] > rr) | (
                    (r_c[None, :] == rr) & (t_c[None, :] < tt))))
            rank[a:b] = before.sum(axis=1)
        keep = rank < C
        slot[t_c[keep], j_c[keep]] = rank[keep]
        slot_src[e, rank[keep]] = t_c[keep] * k + j_c[keep]
    return slot, count, demand, slot_src


def route_grouped(expert_idx, rts_keys, E, C, G):
    """Grouped token selection (Sec. 3.1: a group dimension batches consecutive
    sentences, and the selection happens inside each group; Sec. 5.5 compares
    plain, grouped and RTS selection).

    The T tokens form G groups of T/G consecutive tokens.  Each group routes on
    its own with the rule of route() and C/G slots per expert, so the bias
    towards early positions is confined to a group.  An expert's kept rows of
    group 0 come first in its buffer, then those of group 1, and so on, with no
    gaps: slot = (rows kept for this expert in earlier groups) + rank in group.

    Returns slot[T,k], expert_count[E], expert_demand[E], slot_src[E,C]."""
    expert_idx = np.asarray(expert_idx)
    T, k = expert_idx.shape
    assert T % G == 0 and C % G == 0
    Tg, Cg = T // G, C // G
    slot = np.full((T, k), -1, np.int32)
    count = np.zeros(E, np.int32)
    demand = np.zeros(E, np.int32)
    slot_src = np.full((E, C), -1, np.int32)
    for g in range(G):
        a, b = g * Tg, (g + 1) * Tg
        keys_g = None if rts_keys is None else np.asarray(rts_keys)[a:b]
        s_g, c_g, d_g, src_g = route(expert_idx[a:b], keys_g, E, Cg)
        for e in range(E):
            n = int(c_g[e])
            slot_src[e, count[e]:count[e] + n] = src_g[e, :n] + a * k    # group-local t*k+j -> global
        kept = s_g >= 0
        slot[a:b][kept] = (s_g + count[expert_idx[a:b]])[kept]
        count += c_g
        demand += d_g
    return slot, count, demand, slot_src


# --------------------------------------------------------------------------
# dispatch / combine                                      (Sec. 3.1, Sec. 4.2)
# --------------------------------------------------------------------------
def dispatch(x, slot_src, k):
    """Xd[e,s,:] = x[t,:] where slot_src[e,s] = t*k+j; unused slots hold zeros
    (fixed-shape per-expert buffers, Sec. 3.1)."""
    x = np.asarray(x, _F)
    E, C = slot_src.shape
    Xd = np.zeros((E, C, x.shape[1]), _F)
    e, s = np.nonzero(slot_src >= 0)
    Xd[e, s, :] = x[slot_src[e, s] // k, :]
    return Xd


def combine_fwd(Yd, expert_idx, slot, gate_w=None):
    """y[t,:] = sum over kept choices j of g_j[t] * Yd[e_j[t], slot[t,j], :];
    a token with every choice dropped gets a zero row.  gate_w None = unit
    weights (that is the backward of dispatch)."""
    Yd = np.asarray(Yd, _F)
    T, k = expert_idx.shape
    y = np.zeros((T, Yd.shape[2]), _F)
    for j in range(k):
        kept = np.nonzero(slot[:, j] >= 0)[0]
        rows = Yd[expert_idx[kept, j], slot[kept, j], :]
        if gate_w is not None:
            rows = rows * np.asarray(gate_w, _F)[kept, j][:, None]
        y[kept, :] += rows
    return y


def combine_bwd(dy, Yd, expert_idx, slot, gate_w):
    """dYd[e,s,:] = g_j[t] * dy[t,:] and dg_j[t] = <dy[t,:], Yd[e,s,:]> for kept
    (t,j); zero for dropped choices and unused slots."""
    dy = np.asarray(dy, _F)
    Yd = np.asarray(Yd, _F)
    g = np.asarray(gate_w, _F)
    T, k = expert_idx.shape
    dYd = np.zeros_like(Yd)
    dg = np.zeros((T, k), _F)
    for j in range(k):
        kept = np.nonzero(slot[:, j] >= 0)[0]
        e, s = expert_idx[kept, j], slot[kept, j]
        dYd[e, s, :] = g[kept, j][:, None] * dy[kept, :]
        dg[kept, j] = np.einsum("td,td->t", dy[kept, :], Yd[e, s, :])
    return dYd, dg


# --------------------------------------------------------------------------
# expert feed-forward block                               (Sec. 4.2, Sec. 2.3)
# --------------------------------------------------------------------------
def act(z, kind):
    """relu(z) = max(z,0);  gelu(z) = z/2 * (1 + erf(z / sqrt 2))."""
    z = np.asarray(z, _F)
    if kind == RELU:
        return np.maximum(z, 0.0)
    if kind == GELU:
        return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))
    raise ValueError(kind)


def act_grad(z, kind):
    """relu'(z) = [z > 0];  gelu'(z) = Phi(z) + z * phi(z) (standard normal cdf
    and density)."""
    z = np.asarray(z, _F)
    if kind == RELU:
        return (z > 0).astype(_F)
    if kind == GELU:
        Phi = 0.5 * (1.0 + _erf(z / math.sqrt(2.0)))
        phi = np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)
        return Phi + z * phi
    raise ValueError(kind)


def expert_ffn_fwd(Xd, expert_count, W1, W2, kind, scale=None):
    """Per expert e, on its first n_e = expert_count[e] rows only:
    Z = Xd_e W1_e, H = act(Z), Yd_e = H W2_e.  No biases.  Other rows stay 0.
    scale[E,C,f] (expert dropout, see dropout_scale): H = act(Z) * scale."""
    Xd = np.asarray(Xd, _F)
    E, C, d = Xd.shape
    f = W1.shape[2]
    Z = np.zeros((E, C, f), _F)
    H = np.zeros((E, C, f), _F)
    Yd = np.zeros((E, C, d), _F)
    for e in range(E):
        n = int(expert_count[e])
        if n == 0:
            continue
        Z[e, :n] = Xd[e, :n] @ np.asarray(W1[e], _F)
        H[e, :n] = act(Z[e, :n], kind)
        if scale is not None:
            H[e, :n] *= scale[e, :n]
        Yd[e, :n] = H[e, :n] @ np.asarray(W2[e], _F)
    return Z, H, Yd


def expert_ffn_bwd(dYd, Xd, Z, expert_count, W1, W2, kind, scale=None):
    """dH = dYd W2^T, dZ = dH * act'(Z), dW2 = H^T dYd, dXd = dZ W1^T,
    dW1 = Xd^T dZ, each over the first n_e rows of expert e; an empty expert
    gets zero weight gradients.  With expert dropout (scale, a constant of the
    step) H = act(Z) * scale and dZ = dH * scale * act'(Z)."""
    dYd = np.asarray(dYd, _F)
    Xd = np.asarray(Xd, _F)
    Z = np.asarray(Z, _F)
    E, C, d = Xd.shape
    f = W1.shape[2]
    dXd = np.zeros((E, C, d), _F)
    dW1 = np.zeros((E, d, f), _F)
    dW2 = np.zeros((E, f, d), _F)
    for e in range(E):
        n = int(expert_count[e])
        if n == 0:
            continue
        w1, w2 = np.asarray(W1[e], _F), np.asarray(W2[e], _F)
        H = act(Z[e, :n], kind)
        dH = dYd[e, :n] @ w2.T
        dZ = dH * act_grad(Z[e, :n], kind)
        if scale is not None:
            H = H * scale[e, :n]
            dZ = dZ * scale[e, :n]
        dW2[e] = H.T @ dYd[e, :n]
        dXd[e, :n] = dZ @ w1.T
        dW1[e] = Xd[e, :n].T @ dZ
    return dXd, dW1, dW2


# --------------------------------------------------------------------------
# gate backward                                     (derivative of the gate)
# --------------------------------------------------------------------------
def gate_bwd(dgate_w, p, expert_idx, slot):
    """dgate_w -> dp -> dlogits with the selection and the slots held constant.

    A dropped choice has dg = 0.  k=1: dp[t,e0] = dg0.  k=2, with
    S = p[t,e0] + p[t,e1]: dp[t,e0] = p[t,e1] (dg0 - dg1) / S^2 and
    dp[t,e1] = p[t,e0] (dg1 - dg0) / S^2.  All other dp are zero.
    Softmax: dl[t,e] = p[t,e] (dp[t,e] - sum_e' p[t,e'] dp[t,e'])."""
    p = np.asarray(p, _F)
    T, E = p.shape
    k = expert_idx.shape[1]
    dg = np.where(slot >= 0, np.asarray(dgate_w, _F), 0.0)
    dp = np.zeros((T, E), _F)
    rows = np.arange(T)
    e0 = expert_idx[:, 0].astype(np.int64)
    if k == 1:
        dp[rows, e0] = dg[:, 0]
    else:
        e1 = expert_idx[:, 1].astype(np.int64)
        p0, p1 = p[rows, e0], p[rows, e1]
        S2 = (p0 + p1) ** 2
        dp[rows, e0] = p1 * (dg[:, 0] - dg[:, 1]) / S2
        dp[rows, e1] = p0 * (dg[:, 1] - dg[:, 0]) / S2
    return p * (dp - (p * dp).sum(axis=1, keepdims=True))


# --------------------------------------------------------------------------
# balancing auxiliary loss                          (Sec. 5.1, "MoE setting")
# --------------------------------------------------------------------------
def aux_loss(p, expert_idx):
    """Balancing loss of the gate (Sec. 5.1: an additional balancing loss, times
    0.01, is added to the training loss; the paper points to the Switch /
    GShard form and prints no formula).  Reading taken:

        f[e] = (number of tokens whose FIRST choice is e) / T     (before drops)
        P[e] = mean over tokens of p[t,e]
        L    = E * sum_e f[e] * P[e]

    L = 1 for a perfectly uniform gate.  Returns (L, f, P)."""
    p = np.asarray(p, _F)
    T, E = p.shape
    f = np.zeros(E, _F)
    for t in range(T):
        f[int(expert_idx[t, 0])] += 1.0
    f /= T
    P = p.sum(axis=0) / T
    return float(E * np.dot(f, P)), f, P


def aux_loss_bwd(p, f, coef):
    """Gradient of coef * L with respect to the logits, f held constant (the
    first-choice fractions are counts and carry no gradient):
        dp[t,e] = coef * E * f[e] / T        for every token, dropped or not
        dl[t,e] = p[t,e] (dp[t,e] - sum_e' p[t,e'] dp[t,e'])."""
    p = np.asarray(p, _F)
    T, E = p.shape
    dp = np.broadcast_to(coef * E * np.asarray(f, _F) / T, (T, E))
    return p * (dp - (p * dp).sum(axis=1, keepdims=True))


def utilisation(expert_idx_batches, E):
    """Pruning statistic (Sec. 3.3): the number of times a token is routed to
    each expert over a set of batches, counted on the gate's choices (every
    routed candidate, first and second choices alike, dropped or not)."""
    u = np.zeros(E, np.int64)
    for eidx in expert_idx_batches:
        for e in np.asarray(eidx).ravel():
            u[int(e)] += 1
    return u


def gate_logits_bwd(x, Wg, dlogits):
    """dWg = x^T dlogits;  dx_gate = dlogits Wg^T."""
    x = np.asarray(x, _F)
    dl = np.asarray(dlogits, _F)
    return x.T @ dl, dl @ np.asarray(Wg, _F).T


# --------------------------------------------------------------------------
# the whole layer, forward and backward
# --------------------------------------------------------------------------
def moe_layer(x, Wg, bias, W1, W2, rts_keys, dy, k, C, kind, logits=None, aux_coef=0.0, groups=1,
              jitter_eps=0.0, drop_p=0.0, seed=0):
    """One MoE layer forward and backward in the order gate -> capacity/RTS ->
    dispatch -> experts -> combine, then the reverse.  `logits`, when given,
    replaces the gate projection as the routing input (used to route on the
    fp32 logits another implementation produced); the gate projection's
    backward still uses x and Wg.  aux_coef > 0 adds aux_coef * (balancing loss)
    to the objective: its value is returned and its gradient joins dlogits.
    groups > 1 selects tokens inside groups of T/groups consecutive tokens.
    jitter_eps > 0 multiplies the gate's input by jitter_noise(seed); drop_p > 0
    applies expert dropout with dropout_scale(seed).
    Returns a dict of every intermediate."""
    E = W1.shape[0]
    xg = np.asarray(x, _F)                       # what the gate sees
    if jitter_eps != 0.0:
        xg = xg * jitter_noise(xg.shape[0], xg.shape[1], jitter_eps, seed)
    scale = dropout_scale(E, C, W1.shape[2], drop_p, seed) if drop_p != 0.0 else None
    lg = gate_logits(xg, Wg, bias) if logits is None else np.asarray(logits, _F)
    p = softmax(lg)
    eidx = top_k(lg, k)
    g = gate_weights(p, eidx)
    if groups == 1:
        slot, count, demand, slot_src = route(eidx, rts_keys, E, C)
    else:
        slot, count, demand, slot_src = route_grouped(eidx, rts_keys, E, C, groups)
    Xd = dispatch(x, slot_src, k)
    Z, H, Yd = expert_ffn_fwd(Xd, count, W1, W2, kind, scale)
    y = combine_fwd(Yd, eidx, slot, g)
    out = dict(logits=lg, probs=p, expert_idx=eidx, gate_w=g, slot=slot,
               expert_count=count, expert_demand=demand, slot_src=slot_src,
               Xd=Xd, Z=Z, H=H, Yd=Yd, y=y)
    L, f, P = aux_loss(p, eidx)
    out.update(aux_loss=L, first_frac=f, mean_prob=P)
    if dy is None:
        return out
    dYd, dg = combine_bwd(dy, Yd, eidx, slot, g)
    dXd, dW1, dW2 = expert_ffn_bwd(dYd, Xd, Z, count, W1, W2, kind, scale)
    dx_disp = combine_fwd(dXd, eidx, slot, None)
    dl = gate_bwd(dg, p, eidx, slot)
    if aux_coef != 0.0:
        dl = dl + aux_loss_bwd(p, f, aux_coef)
    dWg, dx_gate = gate_logits_bwd(xg, Wg, dl)   # dWg = (x * noise)^T dl
    if jitter_eps != 0.0:
        dx_gate = dx_gate * jitter_noise(xg.shape[0], xg.shape[1], jitter_eps, seed)
    out.update(dYd=dYd, dgate_w=dg, dXd=dXd, dW1=dW1, dW2=dW2, dx_disp=dx_disp,
               dlogits=dl, dWg=dWg, dx=dx_disp + dx_gate)
    return out
