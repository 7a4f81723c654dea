"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py times.
Routing is compared in full (it is cheap for the oracle); floating-point outputs are compared on what the
fp64 oracle can compute exactly in seconds: y on a seeded sample of tokens (token rows are independent),
weight-gradient slices for sampled hidden units of every expert (each unit needs all of the expert's
tokens but only its own weights), dX and dW_gate in full."""
import os

import numpy as np
import pytest

import workloads as wl
from oracle import modse_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def max_rel(a, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(a, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-300))


def run_config(name, need_bwd=False, bias=None):
    from paper_2409_12210_amd.harness import LayerRunner
    cfg = wl.CONFIGS[name]
    inp = wl.make_inputs(cfg, need_dy=need_bwd, logit_bias=bias)
    r = LayerRunner.from_inputs(inp, need_bwd=need_bwd)
    r.fwd()
    if need_bwd:
        r.bwd()
    return cfg, inp, r


def check_routing_full(cfg, inp, got):
    T, k, N = cfg.n_tokens, cfg.top_k, cfg.n_experts
    ref = orc.route(inp.x, inp.W_gate, N, k, inp.logit_bias)
    near = orc.near_tie_mask(ref.logits, k)
    idx = got["topk_idx"]
    assert (idx[~near] == ref.topk_idx[~near]).all()
    assert np.abs(got["topk_w"][~near] - ref.topk_w[~near]).max() < 2e-7
    assert abs(int(got["near_tie_count"][0]) - int(near.sum())) <= 2
    counts, offsets, row_of, src_of = orc.permutation_from_indices(idx, N)
    assert (got["counts"] == counts).all() and (got["offsets"] == offsets).all()
    assert (got["row_of"] == row_of).all() and (got["src_of"] == src_of).all()
    # invariants that hold at any size
    assert counts.sum() == T * k
    assert np.abs(got["topk_w"].sum(1) - 1).max() < 1e-6
    assert (np.bincount(src_of // k, minlength=T) == k).all()
    return idx, int(near.sum())


def check_y_sample(cfg, inp, r, idx, n=512):
    from paper_2409_12210_amd.harness import to_host
    sel = wl.sample_tokens(cfg.n_tokens, n)
    y_ref = orc.layer_fwd(inp.x[sel], inp.W_gate, inp.W1, inp.W3, inp.W2, cfg.d_ff, cfg.top_k, inp.logit_bias,
                          topk_idx=idx[sel])
    import torch
    y = to_host(r.y[torch.from_numpy(sel).to(r.y.device)])
    err = max_rel(y, y_ref)
    assert err <= TOL[cfg.dtype], err
    return err


@pytest.mark.parametrize("name", ["C1", "C1U"])
def test_c1_forward_full_size(name):
    cfg, inp, r = run_config(name)
    idx, _ = check_routing_full(cfg, inp, r.routing_host())
    check_y_sample(cfg, inp, r, idx)


def test_c2_skewed_routing_full_size():
    bias = wl.load_bias_fixture(os.path.join(ROOT, "tests", "golden", "zipf_bias_C2.txt"))
    cfg, inp, r = run_config("C2", bias=bias)
    got = r.routing_host()
    idx, _ = check_routing_full(cfg, inp, got)
    share = got["counts"] / got["counts"].sum()
    assert np.abs(share - wl.zipf_target_shares(cfg.d_ff, cfg.zipf_s)).max() < 0.005
    check_y_sample(cfg, inp, r, idx)


def test_c3_decode_shape_all_tokens():
    from paper_2409_12210_amd.harness import to_host
    cfg, inp, r = run_config("C3")
    idx, _ = check_routing_full(cfg, inp, r.routing_host())
    y_ref = orc.layer_fwd(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, cfg.d_ff, cfg.top_k, topk_idx=idx)
    assert max_rel(to_host(r.y), y_ref) <= TOL["bf16"]


def check_training_step(cfg, inp, r):
    """Forward + backward at full size: routing in full, y on a token sample, dX and dW_gate in full, and of the
    expert weight gradients one hidden unit out of every 256 (the weight-gradient GEMMs tile the hidden units
    in blocks of 256, so every tile of every expert is touched), plus each expert's first and last unit."""
    from paper_2409_12210_amd.harness import to_host
    idx, _ = check_routing_full(cfg, inp, r.routing_host())
    check_y_sample(cfg, inp, r, idx)
    tol = TOL["bf16"]
    # dX and dW_gate in full (needs the forward of every token in fp64: a few tens of seconds of BLAS)
    g = orc.layer_bwd(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, cfg.d_ff, cfg.top_k, inp.dY, inp.logit_bias,
                      topk_idx=idx, need_weight_grads=False)
    assert max_rel(to_host(r.dX), g.dX) <= tol
    assert max_rel(to_host(r.dW_gate), g.dW_gate) <= tol
    # exact slices of the expert weight gradients; tolerance relative to the largest entry seen
    foff = orc.expert_offsets(cfg.d_ff)
    d = cfg.d_model
    dW1, dW3, dW2 = to_host(r.dW1), to_host(r.dW3), to_host(r.dW2)
    rng = np.random.Generator(np.random.Philox(key=99))
    worst = {"dW1": 0.0, "dW3": 0.0, "dW2": 0.0}
    for e, f in enumerate(cfg.d_ff):
        cols = np.array([rng.integers(lo, min(lo + 256, f)) for lo in range(0, f, 256)] + [0, f - 1])
        cols = np.unique(cols)
        g1, g3, g2 = orc.wgrad_columns(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, cfg.d_ff, cfg.top_k, inp.dY, e, cols,
                                       inp.logit_bias, topk_idx=idx)
        worst["dW1"] = max(worst["dW1"], max_rel(dW1[foff[e]:foff[e + 1]][cols], g1))
        worst["dW3"] = max(worst["dW3"], max_rel(dW3[foff[e]:foff[e + 1]][cols], g3))
        worst["dW2"] = max(worst["dW2"], max_rel(dW2[d * foff[e]:d * foff[e + 1]].reshape(d, f)[:, cols], g2))
    for name, err in worst.items():
        assert err <= tol, (name, err)


def test_c4_training_step_full_size():
    cfg, inp, r = run_config("C4", need_bwd=True)
    check_training_step(cfg, inp, r)


def test_c2_training_step_full_size():
    """Backward under skewed routing: the weight-gradient GEMMs' K (tokens per expert) then ranges over more
    than a factor of ten between experts."""
    bias = wl.load_bias_fixture(os.path.join(ROOT, "tests", "golden", "zipf_bias_C2.txt"))
    cfg, inp, r = run_config("C2", need_bwd=True, bias=bias)
    counts = r.routing_host()["counts"]
    assert counts.max() > 8 * counts.min()
    check_training_step(cfg, inp, r)


def test_p700_forward_full_size():
    """The 9:1 width pairs of the paper's 700M model (Table 2) at 16384 tokens."""
    cfg, inp, r = run_config("P700")
    idx, _ = check_routing_full(cfg, inp, r.routing_host())
    check_y_sample(cfg, inp, r, idx)


def test_c1_gate_extensions_and_statistics_full_size():
    """Router with the noise term and the auxiliary loss at the 16K-token configuration, and the routing
    statistics of the plain router: all cheap enough for the oracle to do in full."""
    import torch
    from paper_2409_12210_amd.harness import LayerRunner, to_host
    cfg = wl.CONFIGS["C1"]
    inp = wl.make_inputs(cfg)
    T, k, N = cfg.n_tokens, cfg.top_k, cfg.n_experts
    Wn = wl.make_noise_weights(cfg)
    gamma, eps, alpha = 0.5, 1e-6, 0.01
    r = LayerRunner.from_inputs(inp)
    r.enable_ext(W_noise=Wn, gamma=gamma, eps=eps, aux_alpha=alpha)
    r.route()
    got = r.routing_host()
    on = orc.Noise(Wn, gamma, eps)
    ref = orc.route(inp.x, inp.W_gate, N, k, None, on)
    near = orc.near_tie_mask(ref.logits, k)
    assert (got["topk_idx"][~near] == ref.topk_idx[~near]).all()
    assert np.abs(got["topk_w"][~near] - ref.topk_w[~near]).max() < 2e-7
    counts, offsets, row_of, src_of = orc.permutation_from_indices(got["topk_idx"], N)
    assert (got["counts"] == counts).all() and (got["row_of"] == row_of).all()
    L, f, P, p = orc.aux_loss(ref.logits, alpha)
    assert max_rel(to_host(r.ext.probs), p) < 1e-5
    assert max_rel(to_host(r.ext.noise_pre), orc.noise_term(inp.x, on)[1]) < 1e-5
    assert np.abs(to_host(r.ext.aux_f) - np.bincount(got["topk_idx"][:, 0], minlength=N) / T).max() < 1e-7
    assert max_rel(to_host(r.ext.aux_P), P) < 1e-5
    assert abs(float(to_host(r.ext.aux_loss)[0]) - L) < 1e-4 * L
    # statistics of this routing
    sc, sm = r.stats()
    torch.cuda.synchronize()
    st = orc.routing_stats(got["topk_idx"], cfg.d_ff)
    assert (to_host(sc) == st.slot_counts).all()
    sm = to_host(sm)
    assert np.allclose(sm[:k], st.slot_ratio, rtol=1e-5)
    assert abs(sm[k] - st.total_ratio) < 1e-5 * st.total_ratio and abs(sm[k + 1] - st.avg_hidden) < 1e-5 * st.avg_hidden
