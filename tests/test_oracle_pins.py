"""Pins for the CPU oracle: every check here compares oracle/modse_oracle.py
with something other than itself - a closed form, brute force over tiny inputs,
an invariant, a special case that reduces to a dense SwiGLU FFN or to a uniform
top-2 MoE written with torch library routines, finite differences, autograd, or
a number the paper prints."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import workloads as wl
from oracle import modse_oracle as orc

RTOL = 1e-11


def rel_err(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = max(np.abs(b).max(), 1e-300)
    return np.abs(a - b).max() / den


def tiny_layer(seed, T=24, d=16, d_ff=(8, 24, 16, 16), scale_w=0.5, scale_g=1.0):
    g = np.random.default_rng(seed)
    F = sum(d_ff)
    x = g.standard_normal((T, d))
    Wg = g.standard_normal((d, len(d_ff))) * scale_g
    W1 = g.standard_normal((F, d)) * scale_w
    W3 = g.standard_normal((F, d)) * scale_w
    W2 = g.standard_normal(d * F) * scale_w
    dY = g.standard_normal((T, d))
    return x, Wg, W1, W3, W2, dY


# ---------------------------------------------------------------- paper-printed numbers
def test_pair_constraint_on_paper_table2(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "table2_expert_pairs.txt")) if not l.startswith("#")]
    assert len(rows) == 2
    for r in rows:
        h = int(r[1])
        d_ff = [int(v) for v in r[2:]]
        assert len(d_ff) == 8
        assert orc.pair_sums(d_ff) == [2 * h] * 4
        assert orc.satisfies_pair_constraint(d_ff, h)
        # total hidden width equals the uniform model's N*h (parameter conservation)
        assert sum(d_ff) == 8 * h
        bad = list(d_ff)
        bad[0] += 32
        assert not orc.satisfies_pair_constraint(bad, h)


def test_benchmark_configs_satisfy_pair_constraint():
    for name, h in (("C0", 256), ("C1", 5632), ("C3", 14336), ("C4", 5632), ("P700", 5120)):
        assert orc.satisfies_pair_constraint(wl.CONFIGS[name].d_ff, h), name
    assert orc.satisfies_pair_constraint(wl.CONFIGS["C1U"].d_ff, 5632)


def test_each_slot_routes_every_token_once(golden_dir):
    # the paper's routing tables: the two slot rows of one layer sum to the same token total
    rows = [l.split() for l in open(os.path.join(golden_dir, "appendixA_epoch7_layer0.txt")) if not l.startswith("#")]
    tot = {r[0]: sum(int(v) for v in r[1:]) for r in rows}
    assert abs(tot["top0"] - tot["top1"]) <= 1000 and abs(tot["top0"] - 195657650) <= 1000
    # same structure in the oracle: per-slot histograms each sum to T, combined to T*k
    x, Wg, *_ = tiny_layer(0, T=200, d_ff=(8,) * 8)
    r = orc.route(x, Wg, 8, 2)
    for j in range(2):
        assert np.bincount(r.topk_idx[:, j], minlength=8).sum() == 200
    assert r.counts.sum() == 400 and r.offsets[-1] == 400


# ---------------------------------------------------------------- gate
def test_gate_closed_form_k2():
    g = np.random.default_rng(1)
    logits = g.standard_normal((500, 8)) * 3
    idx = orc.top_k_indices(logits, 2)
    w = orc.gate_weights(logits, idx)
    l1 = logits[np.arange(500), idx[:, 0]]
    l2 = logits[np.arange(500), idx[:, 1]]
    g1 = 1.0 / (1.0 + np.exp(l2 - l1))           # two-way softmax is a logistic function of the gap
    assert np.abs(w[:, 0] - g1).max() < 1e-15
    assert np.abs(w[:, 1] - (1 - g1)).max() < 1e-15
    assert (w[:, 0] >= w[:, 1]).all()
    G = orc.gate_dense(logits, idx)
    assert np.abs(G.sum(1) - 1).max() < 1e-15
    assert ((G != 0).sum(1) == 2).all()           # experts that were not kept get exactly 0
    # one hand-worked value: logits (ln 3, 0, -5): g = (3/4, 1/4, 0)
    G1 = orc.gate_dense(np.array([[math.log(3.0), 0.0, -5.0]]), np.array([[0, 1]]))
    assert np.allclose(G1, [[0.75, 0.25, 0.0]], atol=1e-15)


def test_gate_k1_and_full_k():
    g = np.random.default_rng(2)
    logits = g.standard_normal((50, 6))
    idx = orc.top_k_indices(logits, 1)
    assert (idx[:, 0] == logits.argmax(1)).all()
    assert (orc.gate_weights(logits, idx) == 1.0).all()
    # k = N: keeping everything is the plain softmax (library routine)
    idx = orc.top_k_indices(logits, 6)
    G = orc.gate_dense(logits, idx)
    ref = torch.softmax(torch.from_numpy(logits), dim=1).numpy()
    assert np.abs(G - ref).max() < 1e-15


def test_gate_equals_renormalised_full_softmax():
    # softmax over the kept logits == full softmax, top-k, renormalise
    g = np.random.default_rng(3)
    logits = g.standard_normal((300, 8)) * 2
    p = torch.softmax(torch.from_numpy(logits), dim=1)
    v, i = torch.topk(p, 2, dim=1)
    ref = (v / v.sum(1, keepdim=True)).numpy()
    idx = orc.top_k_indices(logits, 2)
    assert (idx == i.numpy()).all()
    assert np.abs(orc.gate_weights(logits, idx) - ref).max() < 1e-14


def test_topk_brute_force_with_ties():
    g = np.random.default_rng(4)
    logits = np.round(g.standard_normal((400, 8)) * 2) / 2      # coarse grid: many exact ties
    logits[0] = 0.0                                             # all equal -> experts 0, 1
    logits[1] = [1, 5, 5, 5, 0, 0, 0, 0]                        # tie for first -> 1 then 2
    logits[2] = [3, 1, 1, 0, 0, 0, 0, 1]                        # tie for second -> 1
    for k in (1, 2, 3):
        idx = orc.top_k_indices(logits, k)
        for t in range(logits.shape[0]):
            want = sorted(range(8), key=lambda i: (-logits[t, i], i))[:k]
            assert list(idx[t]) == want
    assert list(orc.top_k_indices(logits, 2)[0]) == [0, 1]
    assert list(orc.top_k_indices(logits, 2)[1]) == [1, 2]
    assert list(orc.top_k_indices(logits, 2)[2]) == [0, 1]


def test_topk_picks_are_distinct_when_experts_are_masked_out():
    # Eq. 3 keeps k distinct positions.  With all but one logit at -inf (experts masked by a bias) the second
    # pick is the lowest other index and its gate weight is exactly 0.  Checked against hand values and against
    # a loop that removes each winner from the candidate set.
    ninf = -np.inf
    logits = np.array([[0.3, ninf, ninf, ninf, ninf, ninf, ninf, ninf],
                       [ninf, ninf, ninf, ninf, ninf, 1.5, ninf, ninf],
                       [ninf] * 8,
                       [ninf, ninf, 2.0, ninf, 2.0, ninf, ninf, ninf],
                       [ninf, -1.0, ninf, ninf, ninf, ninf, ninf, 7.0]])
    want = [[0, 1], [5, 0], [0, 1], [2, 4], [7, 1]]
    idx = orc.top_k_indices(logits, 2)
    assert idx.tolist() == want
    for t in range(logits.shape[0]):
        left = list(range(8))
        for j in range(3):
            best = left[0]
            for i in left[1:]:
                if logits[t, i] > logits[t, best]:
                    best = i
            assert orc.top_k_indices(logits, 3)[t, j] == best
            left.remove(best)
    w = orc.gate_weights(logits[[0, 1, 4]], idx[[0, 1, 4]])
    assert w[:2].tolist() == [[1.0, 0.0], [1.0, 0.0]]
    assert abs(w[2, 0] - 1 / (1 + np.exp(-8.0))) < 1e-15 and abs(w[2].sum() - 1) < 1e-15


def test_near_tie_mask():
    logits = np.array([[1.0, 0.5, 0.5 - 5e-7, -3.0],     # 2nd/3rd gap below tol
                       [1.0, 1.0 - 5e-7, 0.0, -3.0],     # 1st/2nd gap below tol
                       [1.0, 0.5, 0.0, -3.0]])
    assert list(orc.near_tie_mask(logits, 2)) == [True, True, False]
    assert list(orc.near_tie_mask(logits, 1)) == [False, True, False]


# ---------------------------------------------------------------- permutation
def test_permutation_brute_force_and_invariants():
    g = np.random.default_rng(5)
    T, N, k = 97, 8, 2
    x = g.standard_normal((T, 16))
    Wg = g.standard_normal((16, N))
    r = orc.route(x, Wg, N, k)
    # brute force: walk experts in order, tokens in order
    rows = []
    for e in range(N):
        for t in range(T):
            for j in range(k):
                if r.topk_idx[t, j] == e:
                    rows.append(t * k + j)
    assert list(r.src_of) == rows
    for t in range(T):
        for j in range(k):
            assert r.src_of[r.row_of[t, j]] == t * k + j
    counts = [sum(1 for v in r.topk_idx.reshape(-1) if v == e) for e in range(N)]
    assert list(r.counts) == counts
    assert r.offsets[0] == 0 and list(np.diff(r.offsets)) == counts and r.offsets[-1] == T * k
    # each token appears exactly k times; tokens strictly increase inside a segment
    assert sorted(r.src_of // k) == sorted(list(range(T)) * k)
    for e in range(N):
        seg = r.src_of[r.offsets[e]:r.offsets[e + 1]] // k
        assert (np.diff(seg) > 0).all()
        assert (r.topk_idx.reshape(-1)[r.src_of[r.offsets[e]:r.offsets[e + 1]]] == e).all()


def test_unpermute_of_permute_is_identity():
    g = np.random.default_rng(6)
    T, N, k = 64, 8, 2
    x = g.standard_normal((T, 16)).astype(np.float32)
    r = orc.route(x, g.standard_normal((16, N)), N, k)
    xp = orc.permute_rows(x, r.src_of, k)
    y = orc.unpermute_combine(xp, r.row_of, np.full((T, k), 1.0 / k))
    assert (y == x).all()        # 0.5 x + 0.5 x is exact


def test_empty_expert_and_single_token():
    g = np.random.default_rng(7)
    x = g.standard_normal((5, 8))
    Wg = g.standard_normal((8, 4))
    Wg[:, 3] = 0
    bias = np.array([0, 0, 0, -100.0])           # expert 3 never chosen
    r = orc.route(x, Wg, 4, 2, bias)
    assert r.counts[3] == 0 and r.offsets[3] == r.offsets[4] == 10
    r1 = orc.route(x[:1], Wg, 4, 2)
    assert r1.counts.sum() == 2 and sorted(r1.row_of.reshape(-1)) == [0, 1]


# ---------------------------------------------------------------- layer forward
def torch_uniform_top2_moe(x, Wg, W1s, W3s, W2s, k):
    """Standard top-k MoE with equal-size experts from torch library routines.
    W1s, W3s: [N, f, d]; W2s: [N, d, f]."""
    logits = x @ Wg
    v, i = torch.topk(logits, k, dim=-1)
    g = torch.softmax(v, dim=-1)
    G = torch.zeros_like(logits).scatter(1, i, g)
    a = torch.einsum("td,nfd->tnf", x, W1s)
    b = torch.einsum("td,nfd->tnf", x, W3s)
    o = torch.einsum("tnf,ndf->tnd", TF.silu(a) * b, W2s)
    return (G[:, :, None] * o).sum(1)


def stack_padded(W1, W3, W2, d_ff, d):
    """Zero-pad every expert to the widest one -> stacked uniform tensors."""
    N, fm = len(d_ff), max(d_ff)
    W1s = np.zeros((N, fm, d))
    W3s = np.zeros((N, fm, d))
    W2s = np.zeros((N, d, fm))
    for e in range(N):
        w1, w3, w2 = orc.expert_weights(W1, W3, W2, d_ff, d, e)
        W1s[e, :d_ff[e]] = w1
        W3s[e, :d_ff[e]] = w3
        W2s[e, :, :d_ff[e]] = w2
    return W1s, W3s, W2s


def test_dense_definition_equals_sparse_evaluation():
    x, Wg, W1, W3, W2, _ = tiny_layer(10, T=40, d=16, d_ff=(8, 40, 16, 32, 24, 24))
    yd = orc.layer_fwd_dense(x, Wg, W1, W3, W2, (8, 40, 16, 32, 24, 24), 2)
    ys = orc.layer_fwd(x, Wg, W1, W3, W2, (8, 40, 16, 32, 24, 24), 2)
    assert rel_err(ys, yd) < 1e-14


def test_equal_size_experts_reproduce_standard_top2_moe():
    d_ff = (24,) * 8
    x, Wg, W1, W3, W2, _ = tiny_layer(11, T=60, d=16, d_ff=d_ff)
    W1s, W3s, W2s = stack_padded(W1, W3, W2, d_ff, 16)
    ref = torch_uniform_top2_moe(*(torch.from_numpy(a) for a in (x, Wg, W1s, W3s, W2s)), 2).numpy()
    assert rel_err(orc.layer_fwd(x, Wg, W1, W3, W2, d_ff, 2), ref) < RTOL
    assert rel_err(orc.layer_fwd_dense(x, Wg, W1, W3, W2, d_ff, 2), ref) < RTOL


@pytest.mark.parametrize("k", [1, 2])
def test_zero_padding_reduces_diverse_sizes_to_uniform_moe(k):
    # silu(0)*0 = 0: padding narrow experts with zero units changes nothing
    d_ff = (8, 56, 16, 48, 24, 40, 32, 32)
    x, Wg, W1, W3, W2, _ = tiny_layer(12, T=80, d=16, d_ff=d_ff)
    W1s, W3s, W2s = stack_padded(W1, W3, W2, d_ff, 16)
    ref = torch_uniform_top2_moe(*(torch.from_numpy(a) for a in (x, Wg, W1s, W3s, W2s)), k).numpy()
    assert rel_err(orc.layer_fwd(x, Wg, W1, W3, W2, d_ff, k), ref) < RTOL


def test_split_invariance_against_dense_swiglu_ffn():
    # N=2, k=2, W_g=0: both experts chosen with weight 1/2, so the layer is half of a dense
    # SwiGLU FFN over the concatenated hidden units, wherever the split falls.
    g = np.random.default_rng(13)
    T, d, H2 = 20, 12, 40
    x = g.standard_normal((T, d))
    W1 = g.standard_normal((H2, d)) * 0.4
    W3 = g.standard_normal((H2, d)) * 0.4
    W2cat = g.standard_normal((d, H2)) * 0.4
    xt, w1t, w3t, w2t = (torch.from_numpy(a) for a in (x, W1, W3, W2cat))
    ref = 0.5 * TF.linear(TF.silu(TF.linear(xt, w1t)) * TF.linear(xt, w3t), w2t).numpy()
    for s in range(4, H2, 4):
        d_ff = (s, H2 - s)
        W2 = np.concatenate([W2cat[:, :s].reshape(-1), W2cat[:, s:].reshape(-1)])
        y = orc.layer_fwd(x, np.zeros((d, 2)), W1, W3, W2, d_ff, 2)
        assert rel_err(y, ref) < RTOL, s
        r = orc.route(x, np.zeros((d, 2)), 2, 2)
        assert (r.topk_idx == [0, 1]).all() and (r.topk_w == 0.5).all()


def test_linearity_in_w2():
    d_ff = (8, 24, 16, 16)
    x, Wg, W1, W3, W2, _ = tiny_layer(14, d_ff=d_ff)
    y = orc.layer_fwd(x, Wg, W1, W3, W2, d_ff, 2)
    assert rel_err(orc.layer_fwd(x, Wg, W1, W3, 4.0 * W2, d_ff, 2), 4.0 * y) < 1e-15


def test_logit_bias_moves_routing_only():
    d_ff = (8, 24, 16, 16)
    x, Wg, W1, W3, W2, _ = tiny_layer(15, d_ff=d_ff)
    bias = np.array([0.0, 0.0, 50.0, 0.0])
    r = orc.route(x, Wg, 4, 2, bias)
    assert (r.topk_idx[:, 0] == 2).all()
    # a constant shift of all logits changes nothing
    y0 = orc.layer_fwd(x, Wg, W1, W3, W2, d_ff, 2)
    y1 = orc.layer_fwd(x, Wg, W1, W3, W2, d_ff, 2, logit_bias=np.full(4, 3.25))
    assert rel_err(y1, y0) < 1e-13


# ---------------------------------------------------------------- backward
def loss_of(x, Wg, W1, W3, W2, d_ff, dY, idx):
    return float((orc.layer_fwd(x, Wg, W1, W3, W2, d_ff, 2, topk_idx=idx) * dY).sum())


def test_backward_central_finite_differences():
    d_ff = (4, 12, 8, 8)
    x, Wg, W1, W3, W2, dY = tiny_layer(20, T=6, d=5, d_ff=d_ff, scale_w=0.7)
    gr = orc.layer_bwd(x, Wg, W1, W3, W2, d_ff, 2, dY)
    logits = orc.router_logits(x, Wg)
    assert not orc.near_tie_mask(logits, 2, tol=1e-3).any()     # away from routing flips
    idx = orc.top_k_indices(logits, 2)
    eps = 1e-6
    tensors = {"x": (x, gr.dX), "Wg": (Wg, gr.dW_gate), "W1": (W1, gr.dW1), "W3": (W3, gr.dW3), "W2": (W2, gr.dW2)}
    rng = np.random.default_rng(0)
    for name, (arr, grad) in tensors.items():
        flat = arr.reshape(-1)
        gflat = np.asarray(grad).reshape(-1)
        picks = range(flat.size) if flat.size <= 60 else rng.choice(flat.size, 60, replace=False)
        scale = np.abs(gflat).max()
        for p in picks:
            old = flat[p]
            flat[p] = old + eps
            lp = loss_of(x, Wg, W1, W3, W2, d_ff, dY, None)
            flat[p] = old - eps
            lm = loss_of(x, Wg, W1, W3, W2, d_ff, dY, None)
            flat[p] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - gflat[p]) <= 2e-7 * scale + 1e-9, (name, p, fd, gflat[p])
    assert (orc.top_k_indices(orc.router_logits(x, Wg), 2) == idx).all()


def torch_grads(x, Wg, W1, W3, W2, d_ff, d, dY, k):
    W1s, W3s, W2s = stack_padded(W1, W3, W2, d_ff, d)
    ts = [torch.from_numpy(np.array(a)).requires_grad_(True) for a in (x, Wg, W1s, W3s, W2s)]
    y = torch_uniform_top2_moe(*ts, k)
    y.backward(torch.from_numpy(dY))
    return [t.grad.numpy() for t in ts]


@pytest.mark.parametrize("k", [1, 2])
def test_backward_matches_autograd_of_padded_uniform_moe(k):
    d_ff = (8, 56, 16, 48, 24, 40, 32, 32)
    d = 16
    x, Wg, W1, W3, W2, dY = tiny_layer(21, T=70, d=d, d_ff=d_ff)
    gx, gWg, gW1s, gW3s, gW2s = torch_grads(x, Wg, W1, W3, W2, d_ff, d, dY, k)
    gr = orc.layer_bwd(x, Wg, W1, W3, W2, d_ff, k, dY)
    assert rel_err(gr.dX, gx) < RTOL
    assert rel_err(gr.dW_gate, gWg) < RTOL
    foff = orc.expert_offsets(d_ff)
    for e, f in enumerate(d_ff):
        assert rel_err(gr.dW1[foff[e]:foff[e + 1]], gW1s[e, :f]) < RTOL
        assert rel_err(gr.dW3[foff[e]:foff[e + 1]], gW3s[e, :f]) < RTOL
        assert rel_err(gr.dW2[d * foff[e]:d * foff[e + 1]].reshape(d, f), gW2s[e, :, :f]) < RTOL


def test_backward_identities():
    d_ff = (8, 24, 16, 16, 8, 8)
    x, Wg, W1, W3, W2, dY = tiny_layer(22, T=50, d=16, d_ff=d_ff)
    bias = np.array([0, 0, 0, 0, -100.0, 0])      # expert 4 never selected
    gr = orc.layer_bwd(x, Wg, W1, W3, W2, d_ff, 2, dY, logit_bias=bias)
    assert np.abs(gr.dlogits.sum(1)).max() < 1e-13          # softmax gradient sums to zero
    assert ((gr.dlogits != 0).sum(1) <= 2).all()
    assert (gr.dW_gate[:, 4] == 0).all()
    foff = orc.expert_offsets(d_ff)
    assert (gr.dW1[foff[4]:foff[5]] == 0).all() and (gr.dW3[foff[4]:foff[5]] == 0).all()
    assert (gr.dW2[16 * foff[4]:16 * foff[5]] == 0).all()
    # k=2 collapses to dl_1 = -dl_2
    r = orc.route(x, Wg, 6, 2, bias)
    dl = gr.dlogits[np.arange(50)[:, None], r.topk_idx]
    assert np.abs(dl[:, 0] + dl[:, 1]).max() < 1e-13
    # linear in dY
    gr2 = orc.layer_bwd(x, Wg, W1, W3, W2, d_ff, 2, -2.0 * dY, logit_bias=bias)
    assert rel_err(gr2.dX, -2.0 * gr.dX) < 1e-14 and rel_err(gr2.dW1, -2.0 * gr.dW1) < 1e-14


def test_wgrad_columns_equal_slices_of_full_backward():
    d_ff = (8, 24, 16, 16)
    d = 16
    x, Wg, W1, W3, W2, dY = tiny_layer(23, T=40, d=d, d_ff=d_ff)
    gr = orc.layer_bwd(x, Wg, W1, W3, W2, d_ff, 2, dY)
    foff = orc.expert_offsets(d_ff)
    for e in range(4):
        cols = np.array([0, d_ff[e] // 2, d_ff[e] - 1])
        g1, g3, g2 = orc.wgrad_columns(x, Wg, W1, W3, W2, d_ff, 2, dY, e, cols)
        assert rel_err(g1, gr.dW1[foff[e]:foff[e + 1]][cols]) < 1e-13
        assert rel_err(g3, gr.dW3[foff[e]:foff[e + 1]][cols]) < 1e-13
        full2 = gr.dW2[d * foff[e]:d * foff[e + 1]].reshape(d, d_ff[e])
        assert rel_err(g2, full2[:, cols]) < 1e-13


def test_token_rows_are_independent():
    # y and dX of a token depend on that token only: a subset run equals the slice
    d_ff = (8, 24, 16, 16)
    x, Wg, W1, W3, W2, dY = tiny_layer(24, T=30, d_ff=d_ff)
    sel = np.array([1, 7, 8, 22])
    y = orc.layer_fwd(x, Wg, W1, W3, W2, d_ff, 2)
    ys = orc.layer_fwd(x[sel], Wg, W1, W3, W2, d_ff, 2)
    assert rel_err(ys, y[sel]) < 1e-14
    gr = orc.layer_bwd(x, Wg, W1, W3, W2, d_ff, 2, dY)
    grs = orc.layer_bwd(x[sel], Wg, W1, W3, W2, d_ff, 2, dY[sel], need_weight_grads=False)
    assert rel_err(grs.dX, gr.dX[sel]) < 1e-14


# ---------------------------------------------------------------- input recipe
def test_bf16_rounding_is_rne_and_matches_torch():
    g = np.random.default_rng(30)
    a = (g.standard_normal(10000) * 3).astype(np.float32)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert (wl.round_to_bf16(a) == ref).all()
    bits = wl.bf16_bits(wl.round_to_bf16(a))
    assert (wl.bf16_bits_to_f32(bits) == ref).all()


def test_inputs_are_seeded_and_independent_of_other_tensors():
    c = wl.with_tokens(wl.CONFIGS["C0"], 32)
    a = wl.make_inputs(c, need_dy=True)
    b = wl.make_inputs(wl.with_tokens(wl.CONFIGS["C0"], 64), need_dy=True)
    assert (a.W1 == b.W1).all() and (a.W_gate == b.W_gate).all()
    assert a.x.shape == (32, 256) and a.W2.shape == (256 * 2048,)
    assert abs(a.W1.std() - 0.02) < 1e-3 and abs(b.x.std() - 1.0) < 2e-2
    sh = wl.zipf_target_shares(wl.CONFIGS["C1"].d_ff, 1.2)
    assert abs(sh.sum() - 1) < 1e-12 and sh.argmax() == 1 and sh.max() < 0.5
