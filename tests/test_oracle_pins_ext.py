"""Pins for the oracle's gate extensions: the noise term of H(x) (Sec. 2 Eq. 4-5), the auxiliary
load-balance loss (Sec. 3.2 Eq. 9-12) and the routing statistics (Appendix A, Sec. 4.3).  Each check compares
oracle/modse_oracle.py with something other than itself: closed forms, torch library routines, autograd,
finite differences, invariants, numbers the paper prints."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import modse_oracle as orc


def rel_err(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


def tiny(seed, T=20, d=12, d_ff=(8, 24, 16, 16)):
    g = np.random.default_rng(seed)
    F = sum(d_ff)
    N = len(d_ff)
    return dict(x=g.standard_normal((T, d)), Wg=g.standard_normal((d, N)), Wn=g.standard_normal((d, N)) * 0.7,
                W1=g.standard_normal((F, d)) * 0.5, W3=g.standard_normal((F, d)) * 0.5,
                W2=g.standard_normal(d * F) * 0.5, dY=g.standard_normal((T, d)), d_ff=list(d_ff))


# ---------------------------------------------------------------- noise term
def test_noise_term_matches_torch_softplus_and_rms_norm():
    v = tiny(1)
    gamma, eps = 0.8, 1e-6
    z, u, s, r = orc.noise_term(v["x"], orc.Noise(v["Wn"], gamma, eps))
    ut = torch.from_numpy(v["x"]) @ torch.from_numpy(v["Wn"])
    N = ut.shape[1]
    ref = TF.rms_norm(TF.softplus(ut), (N,), weight=torch.full((N,), gamma, dtype=torch.float64), eps=eps)
    assert rel_err(z, ref.numpy()) < 1e-12
    assert rel_err(s, TF.softplus(ut).numpy()) < 1e-12


def test_noise_term_closed_forms():
    v = tiny(2)
    gamma = 1.3
    # epsilon = 0: the normalised vector has mean square gamma^2 exactly
    z = orc.noise_term(v["x"], orc.Noise(v["Wn"], gamma, 0.0))[0]
    assert np.allclose((z * z).mean(axis=1), gamma * gamma, rtol=1e-13)
    # W_n = 0: softplus(0) = ln 2 for every expert, so the term is the same constant for all experts ...
    eps = 1e-6
    z0 = orc.noise_term(v["x"], orc.Noise(np.zeros_like(v["Wn"]), gamma, eps))[0]
    c = gamma * np.log(2.0) / np.sqrt(np.log(2.0) ** 2 + eps)
    assert np.allclose(z0, c, rtol=1e-14)
    # ... and a constant added to all logits changes neither the selection nor the gate
    base = orc.route(v["x"], v["Wg"], 4, 2)
    with_n = orc.route(v["x"], v["Wg"], 4, 2, noise=orc.Noise(np.zeros_like(v["Wn"]), gamma, eps))
    assert (base.topk_idx == with_n.topk_idx).all()
    assert np.allclose(base.topk_w, with_n.topk_w, rtol=1e-12)
    # softplus is positive and above its argument; large arguments pass through
    u = np.array([-800.0, -1.0, 0.0, 1.0, 800.0])
    sp = orc.softplus(u)
    assert sp[0] == 0.0 and sp[4] == 800.0 and abs(sp[2] - np.log(2.0)) < 1e-16
    assert (sp >= np.maximum(u, 0.0)).all()


def test_noise_term_enters_the_logits():
    v = tiny(3)
    n = orc.Noise(v["Wn"], 0.9, 1e-6)
    l0 = orc.router_logits(v["x"], v["Wg"])
    l1 = orc.router_logits(v["x"], v["Wg"], None, n)
    assert rel_err(l1 - l0, orc.noise_term(v["x"], n)[0]) < 1e-13
    # and through the layer: same output as feeding the term in as a per-token bias of the logits
    y = orc.layer_fwd(v["x"], v["Wg"], v["W1"], v["W3"], v["W2"], v["d_ff"], 2, noise=n)
    idx = orc.top_k_indices(l1, 2)
    r = orc.Routing(idx, orc.gate_weights(l1, idx), *orc.permutation_from_indices(idx, 4), l1)
    y2 = orc.layer_fwd(v["x"], v["Wg"], v["W1"], v["W3"], v["W2"], v["d_ff"], 2, routing=r)
    assert rel_err(y, y2) < 1e-13


def _torch_layer_loss(v, k, noise=None, alpha=None, aux_grad=1.0, idx=None):
    """<dY, y> (+ aux_grad L_a) of the layer written with torch routines on a FIXED selection idx."""
    t = {n: torch.tensor(v[n], dtype=torch.float64, requires_grad=n in ("x", "Wg", "Wn", "W1", "W3", "W2"))
         for n in ("x", "Wg", "Wn", "W1", "W3", "W2", "dY")}
    gamma = torch.tensor(noise[0] if noise else 0.0, dtype=torch.float64, requires_grad=True)
    logits = t["x"] @ t["Wg"]
    N = logits.shape[1]
    if noise:
        logits = logits + TF.rms_norm(TF.softplus(t["x"] @ t["Wn"]), (N,), weight=gamma.expand(N), eps=noise[1])
    idx_t = torch.tensor(idx, dtype=torch.int64)
    g = torch.softmax(torch.gather(logits, 1, idx_t), dim=1)
    d = t["x"].shape[1]
    foff = np.concatenate([[0], np.cumsum(v["d_ff"])])
    y = torch.zeros_like(t["x"])
    for e in range(N):
        w1, w3 = t["W1"][foff[e]:foff[e + 1]], t["W3"][foff[e]:foff[e + 1]]
        w2 = t["W2"][d * foff[e]:d * foff[e + 1]].reshape(d, -1)
        o = TF.linear(TF.silu(TF.linear(t["x"], w1)) * TF.linear(t["x"], w3), w2)
        ge = (g * (idx_t == e)).sum(dim=1, keepdim=True)
        y = y + ge * o
    loss = (t["dY"] * y).sum()
    if alpha is not None:
        p = torch.softmax(logits, dim=1)
        f = TF.one_hot(torch.argmax(logits, dim=1), N).to(torch.float64).mean(dim=0).detach()
        loss = loss + aux_grad * alpha * N * (f * p.mean(dim=0)).sum()
    loss.backward()
    return t, gamma


@pytest.mark.parametrize("k", [1, 2])
def test_backward_with_noise_and_aux_matches_autograd(k):
    v = tiny(4 + k)
    gamma, eps, alpha, ag = 0.6, 1e-6, 0.05, 3.0
    n = orc.Noise(v["Wn"], gamma, eps)
    idx = orc.top_k_indices(orc.router_logits(v["x"], v["Wg"], None, n), k)
    G = orc.layer_bwd(v["x"], v["Wg"], v["W1"], v["W3"], v["W2"], v["d_ff"], k, v["dY"], noise=n, aux_alpha=alpha,
                      aux_grad=ag)
    t, g_t = _torch_layer_loss(v, k, noise=(gamma, eps), alpha=alpha, aux_grad=ag, idx=idx)
    assert rel_err(G.dX, t["x"].grad.numpy()) < 1e-10
    assert rel_err(G.dW_gate, t["Wg"].grad.numpy()) < 1e-10
    assert rel_err(G.dW_noise, t["Wn"].grad.numpy()) < 1e-10
    assert abs(G.dgamma - g_t.grad.item()) < 1e-10 * max(1.0, abs(g_t.grad.item()))
    assert rel_err(G.dW1, t["W1"].grad.numpy()) < 1e-10
    assert rel_err(G.dW2, t["W2"].grad.numpy()) < 1e-10


def test_noise_backward_central_finite_differences():
    v = tiny(7, T=6, d=5, d_ff=(8, 8, 8))
    gamma, eps = 0.9, 1e-6
    n = orc.Noise(v["Wn"], gamma, eps)
    dl = np.random.default_rng(0).standard_normal((6, 3))
    dx, dWn, dgam = orc.noise_backward(v["x"], n, dl)
    loss = lambda x, Wn, g: float((orc.noise_term(x, orc.Noise(Wn, g, eps))[0] * dl).sum())
    h = 1e-6
    for (i, j) in [(0, 0), (3, 2), (5, 4)]:
        xp, xm = v["x"].copy(), v["x"].copy()
        xp[i, j] += h
        xm[i, j] -= h
        assert abs((loss(xp, v["Wn"], gamma) - loss(xm, v["Wn"], gamma)) / (2 * h) - dx[i, j]) < 1e-7
    for (i, j) in [(0, 0), (2, 1), (4, 2)]:
        wp, wm = v["Wn"].copy(), v["Wn"].copy()
        wp[i, j] += h
        wm[i, j] -= h
        assert abs((loss(v["x"], wp, gamma) - loss(v["x"], wm, gamma)) / (2 * h) - dWn[i, j]) < 1e-7
    assert abs((loss(v["x"], v["Wn"], gamma + h) - loss(v["x"], v["Wn"], gamma - h)) / (2 * h) - dgam) < 1e-7


# ---------------------------------------------------------------- auxiliary loss
def test_aux_loss_closed_forms():
    alpha, N, T = 0.01, 8, 64
    # equal logits: p is uniform, so L_a = alpha N sum_i f_i / N = alpha whatever f is; ties send every token to 0
    L, f, P, p = orc.aux_loss(np.zeros((T, N)), alpha)
    assert abs(L - alpha) < 1e-15 and f[0] == 1.0 and f[1:].sum() == 0.0 and np.allclose(P, 1.0 / N)
    # sharp and perfectly spread: token t prefers expert t mod N with probability ~1: f = P = 1/N, L_a = alpha
    lg = np.full((T, N), -50.0)
    lg[np.arange(T), np.arange(T) % N] = 50.0
    L, f, P, _ = orc.aux_loss(lg, alpha)
    assert np.allclose(f, 1.0 / N) and abs(L - alpha) < 1e-12
    # collapsed: everything on expert 3: f = P = e_3, L_a = alpha N (the maximum)
    lg = np.full((T, N), -50.0)
    lg[:, 3] = 50.0
    L, f, P, _ = orc.aux_loss(lg, alpha)
    assert f[3] == 1.0 and abs(L - alpha * N) < 1e-12
    # hand-worked: T = 2, N = 2, logits (ln 3, 0) and (0, 0): p = (3/4, 1/4), (1/2, 1/2); both argmax = 0
    L, f, P, p = orc.aux_loss(np.array([[np.log(3.0), 0.0], [0.0, 0.0]]), 1.0)
    assert np.allclose(p, [[0.75, 0.25], [0.5, 0.5]]) and np.allclose(f, [1.0, 0.0]) and np.allclose(P, [0.625, 0.375])
    assert abs(L - 2 * 0.625) < 1e-15


def test_aux_loss_matches_torch_and_autograd():
    g = np.random.default_rng(11)
    T, N, alpha = 40, 8, 0.02
    lg = g.standard_normal((T, N)) * 2.0
    L, f, P, p = orc.aux_loss(lg, alpha)
    lt = torch.tensor(lg, requires_grad=True)
    pt = torch.softmax(lt, dim=1)
    ft = TF.one_hot(torch.argmax(pt, dim=1), N).to(torch.float64).mean(dim=0)
    Lt = alpha * N * (ft.detach() * pt.mean(dim=0)).sum()
    Lt.backward()
    assert abs(L - Lt.item()) < 1e-14
    assert np.allclose(f, ft.numpy()) and np.allclose(P, pt.mean(dim=0).detach().numpy(), rtol=1e-13)
    dl = orc.aux_loss_dlogits(lg, alpha)
    assert rel_err(dl, lt.grad.numpy()) < 1e-12
    assert np.abs(dl.sum(axis=1)).max() < 1e-16       # softmax Jacobian: rows of dlogits sum to zero
    # finite differences away from argmax ties
    h = 1e-6
    for (i, j) in [(0, 0), (7, 3), (39, 7)]:
        a, b = lg.copy(), lg.copy()
        a[i, j] += h
        b[i, j] -= h
        assert abs((orc.aux_loss(a, alpha)[0] - orc.aux_loss(b, alpha)[0]) / (2 * h) - dl[i, j]) < 1e-9


def test_aux_first_choice_is_slot0_of_the_gate():
    v = tiny(12, T=50)
    lg = orc.router_logits(v["x"], v["Wg"])
    _, f, _, _ = orc.aux_loss(lg, 0.01)
    idx = orc.top_k_indices(lg, 2)
    assert np.allclose(f, np.bincount(idx[:, 0], minlength=4) / 50.0)


# ---------------------------------------------------------------- routing statistics
def test_stats_reproduce_the_papers_max_min_columns(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "appendixA_epoch7_ratios.txt")) if not l.startswith("#")]
    assert len(rows) == 4
    sizes = [4.5, 4, 3, 2.5, 2.5, 2, 1, 0.5]
    for r in rows:
        c = np.array([int(q) for q in r[1:9]])
        st = orc.slot_count_stats(c[None, :], sizes)
        assert c.max() == int(r[9]) and c.min() == int(r[10])
        assert f"{st.slot_ratio[0]:.2f}" == r[11], r[0]
    # top0 and top1 of a layer together: the per-expert totals are far more even than either slot
    both = np.array([[int(q) for q in rows[0][1:9]], [int(q) for q in rows[1][1:9]]])
    st = orc.slot_count_stats(both, sizes)
    assert st.total_ratio < 1.07 < st.slot_ratio.min()


def test_stats_brute_force_and_average_hidden_size():
    g = np.random.default_rng(5)
    N, T, k = 8, 300, 2
    idx = np.stack([g.permutation(N)[:k] for _ in range(T)])
    d_ff = [2816, 8448, 4224, 7040, 4928, 6336, 5632, 5632]
    st = orc.routing_stats(idx, d_ff)
    brute = np.zeros((k, N), dtype=np.int64)
    tot_h = 0
    for t in range(T):
        for j in range(k):
            brute[j, idx[t, j]] += 1
            tot_h += d_ff[idx[t, j]]
    assert (st.slot_counts == brute).all()
    assert abs(st.avg_hidden - tot_h / (T * k)) < 1e-9
    # equal widths: the average chosen width is that width whatever the routing (the paper's baseline
    # figure, 3840 = 2.5 x 1536, Sec. 4.3) ...
    assert orc.routing_stats(idx, [3840] * N).avg_hidden == 3840.0
    # ... and with every expert chosen equally often it is the mean width h of the pair constraint
    even = np.stack([np.arange(T * k) % N]).reshape(T, k)
    assert abs(orc.routing_stats(even, d_ff).avg_hidden - 5632.0) < 1e-9
    # an expert nobody chose: infinite max/min
    assert np.isinf(orc.slot_count_stats([[3, 0, 1]], [8, 8, 8]).slot_ratio[0])
