"""CPU oracle for one Mixture-of-Diverse-Size-Experts (MoDSE) FFN layer.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 numpy statement
of what the layer computes, written from the paper (arXiv 2409.12210).  Only
tests, the smoke check and the benchmark's cpu_baseline leg may import it; the
GPU library never does, and nothing here imports the GPU library.

What it follows:
  * layer output       y = sum_i G_i(x) E_i(x)            (Sec. 2 Eq. 1; Sec. 3.1,
                                                           the diverse-size form)
  * gate               G(x) = Softmax(KeepTopK(H(x), k))   (Sec. 2 Eq. 2)
  * KeepTopK           keeps the k largest entries, -inf elsewhere (Sec. 2 Eq. 3)
  * router logits      H(x)_i = (x W_g)_i  [+ caller bias]  (first term of the
                       unnumbered H(x) equation of Sec. 2; the noise term is
                       switched off, see readings below)
  * experts            E_i has its own hidden width h_i     (Sec. 3.1)
  * pair constraint    h_{i1} + h_{i2} = 2h per pair        (Sec. 3.1)

Readings where the paper is silent or garbled (all listed in the design notes):
  * W_g is d_model x N (the paper prints h_input x h; a gate needs one logit
    per expert).
  * An expert is the Llama-2 FFN the paper says it starts from (Sec. 4.1):
    E(x) = W2 (silu(W1 x) * (W3 x)), no biases.
  * Top-k ties go to the lower expert index; slot 0 holds the largest logit.
  * No capacity limit: every (token, slot) is computed.
  * Rows of one expert keep ascending token order in the permuted layout.
  * The gate weight multiplies the expert OUTPUT (Eq. 1), in full precision.
  * Backward is the chain rule through the above; KeepTopK is piecewise
    constant, so logits that were not kept get zero gradient.

Every function works in float64 on whatever values it is given (bf16 configs
pass bf16-representable numbers, which fp64 holds exactly); there is no
intermediate rounding.

Pins: tests/test_oracle_*.py check this file against closed forms, brute
force, invariants, special cases that reduce to a dense SwiGLU FFN or to a
uniform top-2 MoE written with library routines, finite differences and
autograd.  No function here is unpinned.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# configuration identities
# --------------------------------------------------------------------------
def pair_sums(d_ff: Sequence[int]) -> List[int]:
    """Hidden-width sum of each expert pair (2p, 2p+1)  (Sec. 3.1, pair list)."""
    if len(d_ff) % 2:
        raise ValueError("experts must come in pairs")
    return [int(d_ff[2 * p]) + int(d_ff[2 * p + 1]) for p in range(len(d_ff) // 2)]


def satisfies_pair_constraint(d_ff: Sequence[int], h: int) -> bool:
    """True when every pair's widths sum to 2h  (Sec. 3.1, pair constraint)."""
    return all(s == 2 * int(h) for s in pair_sums(d_ff))


def expert_offsets(d_ff: Sequence[int]) -> List[int]:
    off = [0]
    for f in d_ff:
        off.append(off[-1] + int(f))
    return off


def expert_weights(W1, W3, W2, d_ff, d_model, e):
    """Slices of the packed weights that belong to expert e, as float64.
    W1, W3: [F, d] row blocks; W2: flat, expert e at d*foff[e], shape [d, f_e]."""
    foff = expert_offsets(d_ff)
    lo, hi = foff[e], foff[e + 1]
    w1 = np.asarray(W1[lo:hi], dtype=F64)
    w3 = np.asarray(W3[lo:hi], dtype=F64)
    w2 = np.asarray(W2).reshape(-1)[d_model * lo:d_model * hi].reshape(d_model, hi - lo).astype(F64)
    return w1, w3, w2


# --------------------------------------------------------------------------
# router and gate  (Sec. 2 Eq. 2, Eq. 3)
# --------------------------------------------------------------------------
def router_logits(x, W_gate, logit_bias=None):
    """H(x) = x W_g (+ bias)."""
    l = np.asarray(x, dtype=F64) @ np.asarray(W_gate, dtype=F64)
    if logit_bias is not None:
        l = l + np.asarray(logit_bias, dtype=F64)[None, :]
    return l


def top_k_indices(logits, k):
    """Indices of the k largest logits per row, largest first; ties -> lower
    index (np.argmax returns the first maximum)."""
    work = np.array(logits, dtype=F64, copy=True)
    T = work.shape[0]
    idx = np.empty((T, k), dtype=np.int32)
    rows = np.arange(T)
    for j in range(k):
        i = np.argmax(work, axis=1)
        idx[:, j] = i
        work[rows, i] = -np.inf
    return idx


def gate_dense(logits, idx):
    """G(x) as a dense [T, N] matrix: softmax of the logits with everything
    outside the kept set replaced by -inf (Eq. 2 with Eq. 3)."""
    logits = np.asarray(logits, dtype=F64)
    T, N = logits.shape
    kept = np.full((T, N), -np.inf)
    rows = np.arange(T)[:, None]
    kept[rows, idx] = logits[rows, idx]
    m = kept.max(axis=1, keepdims=True)
    e = np.exp(kept - m)          # exp(-inf) == 0 exactly
    return e / e.sum(axis=1, keepdims=True)


def gate_weights(logits, idx):
    """The k non-zero gate values per token, in slot order: [T, k]."""
    G = gate_dense(logits, idx)
    return G[np.arange(G.shape[0])[:, None], idx]


def near_tie_mask(logits, k, tol=1e-6):
    """Tokens whose routing decision is within `tol` of flipping: the gap
    between the k-th and (k+1)-th logit (set membership) or between two kept
    logits (slot order) is below tol."""
    s = -np.sort(-np.asarray(logits, dtype=F64), axis=1)
    N = s.shape[1]
    upto = min(k, N - 1)
    gaps = s[:, :upto] - s[:, 1:upto + 1]
    return (gaps < tol).any(axis=1)


# --------------------------------------------------------------------------
# canonical permutation (ascending expert, then ascending token)
# --------------------------------------------------------------------------
@dataclass
class Routing:
    topk_idx: np.ndarray    # [T, k] int32
    topk_w: np.ndarray      # [T, k] float64
    counts: np.ndarray      # [N] int32
    offsets: np.ndarray     # [N+1] int32
    row_of: np.ndarray      # [T, k] int32: (token, slot) -> permuted row
    src_of: np.ndarray      # [T*k] int32: permuted row -> token*k + slot
    logits: np.ndarray      # [T, N] float64


def permutation_from_indices(idx, n_experts):
    """counts, offsets, row_of, src_of for given top-k indices.  A stable sort
    of the flattened (token, slot) list by expert id keeps ascending token
    order inside each expert."""
    idx = np.asarray(idx, dtype=np.int32)
    T, k = idx.shape
    flat = idx.reshape(-1)
    counts = np.bincount(flat, minlength=n_experts).astype(np.int32)
    offsets = np.zeros(n_experts + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    src_of = np.argsort(flat, kind="stable").astype(np.int32)
    row_of = np.empty(T * k, dtype=np.int32)
    row_of[src_of] = np.arange(T * k, dtype=np.int32)
    return counts, offsets, row_of.reshape(T, k), src_of


def route(x, W_gate, n_experts, top_k, logit_bias=None) -> Routing:
    logits = router_logits(x, W_gate, logit_bias)
    assert logits.shape[1] == n_experts
    idx = top_k_indices(logits, top_k)
    w = gate_weights(logits, idx)
    counts, offsets, row_of, src_of = permutation_from_indices(idx, n_experts)
    return Routing(idx, w, counts, offsets, row_of, src_of, logits)


# --------------------------------------------------------------------------
# experts and the layer  (Sec. 2 Eq. 1; Sec. 3.1)
# --------------------------------------------------------------------------
def silu(a):
    return a / (1.0 + np.exp(-a))


def expert_ffn(x, w1, w3, w2):
    """E(x) = W2 (silu(W1 x) * (W3 x)) for rows of x.  w1,w3: [f,d]; w2: [d,f]."""
    a = x @ w1.T
    b = x @ w3.T
    return (silu(a) * b) @ w2.T


def layer_fwd_dense(x, W_gate, W1, W3, W2, d_ff, top_k, logit_bias=None):
    """The definition as printed: every expert is evaluated for every token and
    weighted by its gate value, zeros included.  For small inputs."""
    x = np.asarray(x, dtype=F64)
    T, d = x.shape
    N = len(d_ff)
    logits = router_logits(x, W_gate, logit_bias)
    idx = top_k_indices(logits, top_k)
    G = gate_dense(logits, idx)
    y = np.zeros((T, d))
    for i in range(N):
        w1, w3, w2 = expert_weights(W1, W3, W2, d_ff, d, i)
        y += G[:, i:i + 1] * expert_ffn(x, w1, w3, w2)
    return y


def layer_fwd(x, W_gate, W1, W3, W2, d_ff, top_k, logit_bias=None, routing: Optional[Routing] = None,
              topk_idx=None):
    """Same sum restricted to its non-zero terms: expert i is evaluated only on
    the tokens that kept it.  `topk_idx` (optional) overrides the selection,
    for staged parity checks; gate weights are then computed from the oracle's
    own logits on that selection."""
    x = np.asarray(x, dtype=F64)
    T, d = x.shape
    N = len(d_ff)
    if routing is None:
        logits = router_logits(x, W_gate, logit_bias)
        idx = top_k_indices(logits, top_k) if topk_idx is None else np.asarray(topk_idx)
        w = gate_weights(logits, idx)
    else:
        idx, w = routing.topk_idx, routing.topk_w
    y = np.zeros((T, d))
    for i in range(N):
        t, j = np.nonzero(idx == i)
        if t.size == 0:
            continue
        w1, w3, w2 = expert_weights(W1, W3, W2, d_ff, d, i)
        y[t] += w[t, j][:, None] * expert_ffn(x[t], w1, w3, w2)
    return y


# --------------------------------------------------------------------------
# backward (chain rule through Eq. 1-3; loss gradient dY = d loss / d y)
# --------------------------------------------------------------------------
@dataclass
class Grads:
    dX: np.ndarray        # [T, d]
    dW_gate: np.ndarray   # [d, N]
    dW1: np.ndarray       # [F, d]
    dW3: np.ndarray       # [F, d]
    dW2: np.ndarray       # [d*F] flat, packed like W2
    dlogits: np.ndarray   # [T, N]


def gate_backward(w, dg):
    """Gradient of the k kept logits given gradients of the k gate values.
    Softmax Jacobian on the kept set: dl_j = g_j (dg_j - sum_m g_m dg_m)."""
    return w * (dg - (w * dg).sum(axis=1, keepdims=True))


def layer_bwd(x, W_gate, W1, W3, W2, d_ff, top_k, dY, logit_bias=None, topk_idx=None,
              need_weight_grads=True) -> Grads:
    x = np.asarray(x, dtype=F64)
    dY = np.asarray(dY, dtype=F64)
    Wg = np.asarray(W_gate, dtype=F64)
    T, d = x.shape
    N = len(d_ff)
    foff = expert_offsets(d_ff)
    F = foff[-1]
    logits = router_logits(x, Wg, logit_bias)
    idx = top_k_indices(logits, top_k) if topk_idx is None else np.asarray(topk_idx)
    w = gate_weights(logits, idx)

    dX = np.zeros((T, d))
    dg = np.zeros((T, top_k))
    dW1 = np.zeros((F, d)) if need_weight_grads else None
    dW3 = np.zeros((F, d)) if need_weight_grads else None
    dW2 = np.zeros(d * F) if need_weight_grads else None
    for i in range(N):
        t, j = np.nonzero(idx == i)
        if t.size == 0:
            continue
        w1, w3, w2 = expert_weights(W1, W3, W2, d_ff, d, i)
        xe = x[t]
        a = xe @ w1.T
        b = xe @ w3.T
        sig = 1.0 / (1.0 + np.exp(-a))
        h = a * sig * b
        o = h @ w2.T
        dg[t, j] = (dY[t] * o).sum(axis=1)              # y depends on g_j through g_j * o
        do = w[t, j][:, None] * dY[t]
        dh = do @ w2
        da = dh * b * sig * (1.0 + a * (1.0 - sig))     # d silu(a)/da = sig (1 + a (1 - sig))
        db = dh * a * sig
        dX[t] += da @ w1 + db @ w3                      # tokens are distinct within one expert
        if need_weight_grads:
            dW2[d * foff[i]:d * foff[i + 1]] = (do.T @ h).reshape(-1)
            dW1[foff[i]:foff[i + 1]] = da.T @ xe
            dW3[foff[i]:foff[i + 1]] = db.T @ xe
    dl = gate_backward(w, dg)
    dlogits = np.zeros((T, N))
    dlogits[np.arange(T)[:, None], idx] = dl
    dW_gate = x.T @ dlogits
    dX += dlogits @ Wg.T
    return Grads(dX, dW_gate, dW1, dW3, dW2, dlogits)


def wgrad_columns(x, W_gate, W1, W3, W2, d_ff, top_k, dY, e, cols, logit_bias=None, topk_idx=None):
    """Exact slices of expert e's weight gradients for hidden units `cols`:
    dW1_e[cols, :], dW3_e[cols, :], dW2_e[:, cols].  Each hidden unit's
    gradient needs all of the expert's tokens but only that unit's weights, so
    a slice is computed exactly without the rest.  For full-size parity."""
    x = np.asarray(x, dtype=F64)
    dY = np.asarray(dY, dtype=F64)
    T, d = x.shape
    logits = router_logits(x, W_gate, logit_bias)
    idx = top_k_indices(logits, top_k) if topk_idx is None else np.asarray(topk_idx)
    w = gate_weights(logits, idx)
    t, j = np.nonzero(idx == e)
    cols = np.asarray(cols)
    w1, w3, w2 = expert_weights(W1, W3, W2, d_ff, d, e)
    w1c, w3c, w2c = w1[cols], w3[cols], w2[:, cols]
    xe = x[t]
    a = xe @ w1c.T
    b = xe @ w3c.T
    sig = 1.0 / (1.0 + np.exp(-a))
    h = a * sig * b
    do = w[t, j][:, None] * dY[t]
    dh = do @ w2c
    da = dh * b * sig * (1.0 + a * (1.0 - sig))
    db = dh * a * sig
    return da.T @ xe, db.T @ xe, do.T @ h


# --------------------------------------------------------------------------
# helpers for parity tests
# --------------------------------------------------------------------------
def unpermute_combine(O, row_of, w):
    """y[t] = sum_j w[t,j] * O[row_of[t,j]] - the gate-weighted sum of Eq. 1
    written on permuted expert outputs."""
    O = np.asarray(O, dtype=F64)
    y = np.zeros((row_of.shape[0], O.shape[1]))
    for j in range(row_of.shape[1]):
        y += np.asarray(w, dtype=F64)[:, j:j + 1] * O[row_of[:, j]]
    return y


def permute_rows(x, src_of, top_k):
    return np.asarray(x)[np.asarray(src_of) // top_k]


def calibrate_logit_bias(x, W_gate, n_experts, top_k, target_shares, rounds=200, tol=0.002):
    """Find an additive logit bias so that each expert's share of the T*k
    assignments approaches `target_shares` (skewed-routing stress input).
    Damped fixed point bias_e += 0.5 ln(target_e / realised_e).  Returns (bias,
    realised shares).  This prepares an INPUT; it is not part of the method."""
    base = router_logits(x, W_gate)
    bias = np.zeros(n_experts)
    tgt = np.asarray(target_shares, dtype=F64)
    best = None
    for _ in range(rounds):
        idx = top_k_indices(base + bias[None, :], top_k)
        share = np.bincount(idx.reshape(-1), minlength=n_experts) / idx.size
        err = np.abs(share - tgt).max()
        if best is None or err < best[0]:
            best = (err, bias.copy(), share.copy())
        if err < tol:
            break
        bias = bias + 0.5 * np.log(tgt / np.maximum(share, 1e-9))
        bias -= bias.mean()
    return best[1], best[2]
