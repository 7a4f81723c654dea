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
  * noise term         RMSNorm(Softplus(x W_n)) added to the logits (second
                       term of H(x), Sec. 2 Eq. 4-5) -- optional, see readings
  * auxiliary loss     L_a = alpha N sum_i f_i P_i          (Sec. 3.2 Eq. 9-12)
  * routing statistics per-slot token counts per expert, their max/min ratio
                       (Appendix A tables) and the average hidden width of the
                       chosen experts (Sec. 4.3, workload measure)

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
  * Noise term (off unless asked for): the text says it is added to the expert
    outputs, the formula adds it to the logits; the formula is followed.  It
    carries no random factor, so it is a deterministic function of x.  RMSNorm
    runs over the N per-expert values of one token (n = N), gamma is one
    scalar, epsilon is a parameter (1e-6 in the tests).
  * Auxiliary loss: p(x) is the softmax of H(x) over ALL N experts (the gate of
    Eq. 2 is a softmax over the kept ones only); "routed to expert i" in f_i
    means argmax p(x) = i, the first choice, ties to the lower index; f_i is a
    constant in the backward pass (it is piecewise constant in the logits).

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
def softplus(u):
    """log(1 + exp(u))  (Sec. 2 Eq. 5)."""
    return np.logaddexp(0.0, np.asarray(u, dtype=F64))


@dataclass
class Noise:
    """Parameters of the second term of H(x): W_n [d, N], the RMSNorm gain gamma and epsilon (Sec. 2)."""
    W_noise: np.ndarray
    gamma: float
    eps: float = 1e-6


def noise_term(x, noise: "Noise"):
    """RMSNorm(Softplus(x W_n)) per token, the norm taken over the N per-expert values  (Sec. 2, second term
    of the H(x) equation with Eq. 4 and Eq. 5).  Returns (z, u, s, r): the term, x W_n, its softplus and the
    root-mean-square with epsilon."""
    u = np.asarray(x, dtype=F64) @ np.asarray(noise.W_noise, dtype=F64)
    s = softplus(u)
    r = np.sqrt((s * s).mean(axis=1, keepdims=True) + noise.eps)
    return noise.gamma * s / r, u, s, r


def router_logits(x, W_gate, logit_bias=None, noise: Optional["Noise"] = None):
    """H(x) = x W_g (+ bias) (+ the noise term when asked for)."""
    l = np.asarray(x, dtype=F64) @ np.asarray(W_gate, dtype=F64)
    if logit_bias is not None:
        l = l + np.asarray(logit_bias, dtype=F64)[None, :]
    if noise is not None:
        l = l + noise_term(x, noise)[0]
    return l


def top_k_indices(logits, k):
    """Positions of the k largest logits per row, largest first (KeepTopK, Eq. 3,
    keeps k distinct positions of the vector); ties -> lower index.  Written
    as the definition: a stable sort by descending value, first k positions.
    Logits of -inf (experts masked out by a bias) sort last like any other
    value, so the picks stay distinct even when fewer than k logits are finite."""
    work = np.asarray(logits, dtype=F64)
    order = np.argsort(-work, axis=1, kind="stable")
    return np.ascontiguousarray(order[:, :k]).astype(np.int32)


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


def route(x, W_gate, n_experts, top_k, logit_bias=None, noise=None) -> Routing:
    logits = router_logits(x, W_gate, logit_bias, noise)
    assert logits.shape[1] == n_experts
    idx = top_k_indices(logits, top_k)
    w = gate_weights(logits, idx)
    counts, offsets, row_of, src_of = permutation_from_indices(idx, n_experts)
    return Routing(idx, w, counts, offsets, row_of, src_of, logits)


# --------------------------------------------------------------------------
# auxiliary load-balance loss  (Sec. 3.2 Eq. 9-12)
# --------------------------------------------------------------------------
def router_probs(logits):
    """p(x): softmax of the router logits over all N experts (Eq. 11)."""
    l = np.asarray(logits, dtype=F64)
    e = np.exp(l - l.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def aux_loss(logits, alpha):
    """L_a = alpha N sum_i f_i P_i (Eq. 9) with f_i the fraction of tokens whose largest probability is
    expert i (Eq. 10) and P_i the mean probability of expert i (Eq. 12).  Returns (L_a, f, P, p)."""
    p = router_probs(logits)
    T, N = p.shape
    first = np.argmax(np.asarray(logits, dtype=F64), axis=1)   # argmax p = argmax logits; ties -> lower index
    f = np.bincount(first, minlength=N).astype(F64) / T
    P = p.mean(axis=0)
    return float(alpha) * N * float((f * P).sum()), f, P, p


def aux_loss_dlogits(logits, alpha):
    """d L_a / d logits with f held constant: L_a = sum_t <c, p_t>, c_i = alpha N f_i / T, and the softmax
    Jacobian gives dl_t = p_t * (c - <c, p_t>)."""
    _, f, _, p = aux_loss(logits, alpha)
    T, N = p.shape
    c = float(alpha) * N * f / T
    return p * (c[None, :] - (p * c[None, :]).sum(axis=1, keepdims=True))


# --------------------------------------------------------------------------
# routing statistics  (Appendix A tables; Sec. 4.3 workload measure)
# --------------------------------------------------------------------------
@dataclass
class RoutingStats:
    slot_counts: np.ndarray   # [k, N] int64: tokens whose j-th choice is expert i
    slot_ratio: np.ndarray    # [k] max/min of each row (inf when an expert got none)
    total_ratio: float        # max/min of the column sums
    avg_hidden: float         # sum_i n_i h_i / sum_i n_i over all (token, slot) choices


def slot_count_stats(slot_counts, d_ff) -> RoutingStats:
    c = np.asarray(slot_counts, dtype=np.int64)
    with np.errstate(divide="ignore"):
        slot_ratio = c.max(axis=1) / c.min(axis=1).astype(F64)
        tot = c.sum(axis=0)
        total_ratio = float(tot.max() / F64(tot.min()))
    avg = float((tot * np.asarray(d_ff, dtype=F64)).sum() / tot.sum()) if tot.sum() else 0.0
    return RoutingStats(c, slot_ratio, total_ratio, avg)


def routing_stats(topk_idx, d_ff) -> RoutingStats:
    idx = np.asarray(topk_idx)
    N = len(d_ff)
    c = np.stack([np.bincount(idx[:, j], minlength=N) for j in range(idx.shape[1])])
    return slot_count_stats(c, d_ff)


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
              topk_idx=None, noise=None):
    """Same sum restricted to its non-zero terms: expert i is evaluated only on
    the tokens that kept it.  `topk_idx` (optional) overrides the selection,
    for staged parity checks; gate weights are then computed from the oracle's
    own logits on that selection."""
    x = np.asarray(x, dtype=F64)
    T, d = x.shape
    N = len(d_ff)
    if routing is None:
        logits = router_logits(x, W_gate, logit_bias, noise)
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
    dW_noise: Optional[np.ndarray] = None   # [d, N] when the noise term is on
    dgamma: Optional[float] = None


def gate_backward(w, dg):
    """Gradient of the k kept logits given gradients of the k gate values.
    Softmax Jacobian on the kept set: dl_j = g_j (dg_j - sum_m g_m dg_m)."""
    return w * (dg - (w * dg).sum(axis=1, keepdims=True))


def noise_backward(x, noise: "Noise", dlogits):
    """Gradients of the noise term z = gamma s / r, s = softplus(u), u = x W_n, r = sqrt(mean_i s_i^2 + eps)
    given d loss / d z = dlogits.  Returns (dX contribution, dW_noise, dgamma)."""
    x = np.asarray(x, dtype=F64)
    Wn = np.asarray(noise.W_noise, dtype=F64)
    _, u, s, r = noise_term(x, noise)
    N = s.shape[1]
    dgamma = float((dlogits * s / r).sum())
    # z_i = gamma s_i / r(s):  dz_i/ds_j = gamma (delta_ij / r - s_i s_j / (N r^3))
    ds = noise.gamma * (dlogits / r - s * (dlogits * s).sum(axis=1, keepdims=True) / (N * r ** 3))
    du = ds / (1.0 + np.exp(-u))           # d softplus(u)/du = sigmoid(u)
    return du @ Wn.T, x.T @ du, dgamma


def layer_bwd(x, W_gate, W1, W3, W2, d_ff, top_k, dY, logit_bias=None, topk_idx=None,
              need_weight_grads=True, noise=None, aux_alpha=None, aux_grad=1.0) -> Grads:
    """Gradients of  loss = <dY, y> + aux_grad * L_a  (the second term only when aux_alpha is given)."""
    x = np.asarray(x, dtype=F64)
    dY = np.asarray(dY, dtype=F64)
    Wg = np.asarray(W_gate, dtype=F64)
    T, d = x.shape
    N = len(d_ff)
    foff = expert_offsets(d_ff)
    F = foff[-1]
    logits = router_logits(x, Wg, logit_bias, noise)
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
    if aux_alpha is not None:
        dlogits += float(aux_grad) * aux_loss_dlogits(logits, aux_alpha)
    dW_gate = x.T @ dlogits
    dX += dlogits @ Wg.T
    dW_noise = dgamma = None
    if noise is not None:
        dx_n, dW_noise, dgamma = noise_backward(x, noise, dlogits)
        dX += dx_n
    return Grads(dX, dW_gate, dW1, dW3, dW2, dlogits, dW_noise, dgamma)


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
