"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element, on
seeded synthetic inputs small enough for the oracle to finish in seconds yet spanning several tiles and
ragged tails.  Integer outputs must match bit for bit; floating-point outputs must satisfy
max|out - ref| <= tol * max|ref| with tol = 1e-4 (fp32) or 2e-2 (bf16 inputs, fp32 accumulation)."""
import numpy as np
import pytest

import workloads as wl
from oracle import modse_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _runner(inp, need_bwd=False):
    from paper_2409_12210_amd.harness import LayerRunner
    return LayerRunner.from_inputs(inp, need_bwd=need_bwd)


def max_rel(a, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(a, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-300))


def make(name, d, d_ff, T, dtype, k=2, seed=3, need_dy=False, bias=None):
    cfg = wl.LayerConfig(name, d, tuple(d_ff), k, T, dtype, seed=seed, dy_seed=seed + 1)
    return wl.make_inputs(cfg, need_dy=need_dy, logit_bias=bias)


def check_routing(inp, got):
    """Stage-wise integer parity: (i) top-k indices on tokens that are not near-ties, (ii) the
    permutation against the canonical order computed from the GPU's own indices, (iii) invariants."""
    c = inp.cfg
    T, k, N = c.n_tokens, c.top_k, c.n_experts
    ref = orc.route(inp.x, inp.W_gate, N, k, inp.logit_bias)
    near = orc.near_tie_mask(ref.logits, k)
    idx = got["topk_idx"][:T]
    assert (idx[~near] == ref.topk_idx[~near]).all()
    assert np.abs(got["topk_w"][:T][~near] - ref.topk_w[~near]).max() < 2e-7
    # gaps within a hair of the 1e-6 threshold may be counted either way
    lo = int(orc.near_tie_mask(ref.logits, k, tol=0.99e-6).sum())
    hi = int(orc.near_tie_mask(ref.logits, k, tol=1.01e-6).sum())
    assert lo <= int(got["near_tie_count"][0]) <= hi
    counts, offsets, row_of, src_of = orc.permutation_from_indices(idx, N)
    assert (got["counts"] == counts).all()
    assert (got["offsets"] == offsets).all()
    assert (got["row_of"][:T] == row_of).all()
    assert (got["src_of"][:T * k] == src_of).all()
    assert np.abs(got["topk_w"][:T].sum(1) - 1).max() < 1e-6
    return idx, int(near.sum())


ROUTE_CASES = [
    ("c0", 256, (128, 384, 192, 320, 224, 288, 256, 256), 512, "f32", 2),
    ("ragged_T", 256, (128, 384, 192, 320, 224, 288, 256, 256), 501, "f32", 2),
    ("one_token", 64, (32, 96), 1, "f32", 2),
    ("bf16_mid", 512, (96, 416, 160, 352, 224, 288, 256, 256), 1000, "bf16", 2),
    ("top1", 256, (128, 384, 192, 320), 300, "bf16", 1),
    ("n16", 128, (64,) * 16, 777, "f32", 2),
    ("n3", 96, (32, 64, 96), 130, "bf16", 2),
    ("n64", 64, (32,) * 64, 200, "f32", 2),
    ("wide_d", 4096, (64, 192, 128, 128), 70, "bf16", 2),
    # decode-sized batches (at most 64 tokens) take the one-block-per-token router
    ("decode_n16", 128, (64,) * 16, 40, "f32", 2),
    ("decode_n3", 96, (32, 64, 96), 64, "bf16", 2),
    ("decode_top1", 256, (128, 384, 192, 320), 33, "bf16", 1),
    ("decode_wide", 4096, (64, 192, 128, 128, 64, 192, 128, 128), 64, "bf16", 2),
    ("decode_n24", 64, (32,) * 24, 50, "bf16", 2),      # block router + the fused decode-sized permute
    ("decode_n64_top1", 64, (32,) * 64, 64, "f32", 1),
    # batches beyond 4096 tokens (or with more than 16 experts, from 1024 tokens) take the router that keeps
    # W_gate in LDS: every padded expert count, both dtypes, ragged token counts, several groups per block
    ("stream_n8", 256, (128, 384, 192, 320, 224, 288, 256, 256), 5000, "bf16", 2),
    ("stream_n8_f32", 256, (128, 384, 192, 320, 224, 288, 256, 256), 4133, "f32", 2),
    ("stream_n2", 64, (32, 96), 4200, "f32", 2),
    ("stream_n3", 96, (32, 64, 96), 4111, "bf16", 2),
    ("stream_n4_top1", 128, (32, 224, 96, 160), 4500, "bf16", 1),
    ("stream_n16", 128, (64,) * 16, 6001, "f32", 2),
    ("stream_n24", 64, (32,) * 24, 1500, "bf16", 2),
    ("stream_n64", 64, (32,) * 64, 3000, "f32", 2),
    ("stream_n64_bf16", 96, (32,) * 64, 1025, "bf16", 2),
    ("stream_ragged_d", 1120, (64, 192, 128, 128), 4100, "bf16", 2),
    ("stream_many_groups", 32, (32,) * 8, 40000, "bf16", 2),
    # the same router on the float64 matrix instruction (d a multiple of 256, at most 16 experts): both padded
    # expert counts, expert counts that are no multiple of 4, both dtypes, k = 1, ragged token counts, several
    # groups per workgroup, and a matrix that is one size too large for it (the vector form takes over)
    ("mfma_n3", 256, (32, 64, 96), 4111, "bf16", 2),
    ("mfma_n5_f32", 512, (32,) * 5, 4500, "f32", 2),
    ("mfma_n12", 256, (32,) * 12, 4200, "bf16", 2),
    ("mfma_n16_f32_top1", 512, (32,) * 16, 5001, "f32", 1),
    ("mfma_many_groups", 256, (32,) * 8, 40001, "bf16", 2),
    ("mfma_d768", 768, (64,) * 8, 4097, "bf16", 2),
    ("mfma_d2048", 2048, (32,) * 8, 4160, "bf16", 2),
    ("mfma_too_large_n16_d1024", 1024, (32,) * 16, 4100, "bf16", 2),
    # scan over more than 4 blocks per thread, with one and with several 16-column steps
    ("scan_long_runs", 32, (32,) * 8, 140001, "bf16", 2),
    ("scan_long_runs_n40", 32, (32,) * 40, 35001, "f32", 2),
    # more than 16 experts on a small batch, and an expert count that is not a power of two: the router that
    # reads (a padded copy of) W_gate from memory
    ("block_n24", 64, (32,) * 24, 300, "bf16", 2),
    ("block_n40_f32", 96, (32,) * 40, 333, "f32", 2),
]


@pytest.mark.parametrize("case", ROUTE_CASES, ids=[c[0] for c in ROUTE_CASES])
def test_route_parity(case):
    name, d, d_ff, T, dtype, k = case
    inp = make(name, d, d_ff, T, dtype, k)
    r = _runner(inp)
    r.route()
    check_routing(inp, r.routing_host())


def test_route_with_bias_and_empty_expert():
    bias = np.array([0, 0, -100.0, 0, 3.0, 0, 0, 0], dtype=np.float32)
    inp = make("bias", 256, (128, 384, 192, 320, 224, 288, 256, 256), 700, "bf16", bias=bias)
    r = _runner(inp)
    r.route()
    got = r.routing_host()
    check_routing(inp, got)
    assert got["counts"][2] == 0 and got["counts"][4] > 300


@pytest.mark.parametrize("T,d", [(50, 128), (5000, 128), (5000, 256)],
                         ids=["token_router", "stream_router", "mfma_router"])
def test_route_masked_experts_second_pick_differs_from_first(T, d):
    # every expert but one masked out by an infinite negative bias: the second pick is the lowest other index
    # (as in a stable descending sort) with gate weight 0, never a repeat of the first
    from oracle import modse_oracle as orc2
    for keep in (0, 5):
        bias = np.full(8, -np.inf, dtype=np.float32)
        bias[keep] = 0.0
        inp = make("masked", d, (64,) * 8, T, "f32", bias=bias, seed=9 + keep)
        r = _runner(inp)
        r.route()
        got = r.routing_host()
        ref = orc2.route(inp.x, inp.W_gate, 8, 2, bias)
        assert (got["topk_idx"] == ref.topk_idx).all()
        assert (got["topk_idx"][:, 0] == keep).all() and (got["topk_idx"][:, 1] == (1 if keep == 0 else 0)).all()
        assert (got["topk_w"] == np.array([1.0, 0.0], dtype=np.float32)).all()
        counts, offsets, row_of, src_of = orc2.permutation_from_indices(got["topk_idx"], 8)
        assert (got["counts"] == counts).all() and (got["row_of"] == row_of).all() and (got["src_of"] == src_of).all()


def test_route_exact_ties_go_to_lower_index():
    # identical W_gate columns -> identical logits for every expert: experts 0 and 1 win
    inp = make("ties", 128, (64, 64, 64, 64), 100, "f32")
    inp.W_gate[:] = inp.W_gate[:, :1]
    r = _runner(inp)
    r.route()
    got = r.routing_host()
    assert (got["topk_idx"] == [0, 1]).all()
    assert got["near_tie_count"][0] == 100
    assert np.abs(got["topk_w"] - 0.5).max() == 0


FWD_CASES = [
    ("c0", 256, (128, 384, 192, 320, 224, 288, 256, 256), 512, "f32", 2),
    ("c0_ragged", 256, (128, 384, 192, 320, 224, 288, 256, 256), 333, "f32", 2),
    ("f32_top1", 128, (32, 224, 96, 160), 200, "f32", 1),
    ("bf16_mid", 512, (96, 416, 160, 352, 224, 288, 256, 256), 1000, "bf16", 2),
    ("bf16_tails", 320, (32, 608, 288, 352), 1531, "bf16", 2),
    ("bf16_top1", 256, (128, 384, 192, 320), 300, "bf16", 1),
    ("bf16_one_token", 256, (128, 384), 1, "bf16", 2),
    # decode-sized batches: 64-row tiles and a split-K down-projection (ragged widths, chunk tails)
    ("bf16_decode", 512, (96, 416, 160, 352, 224, 288, 256, 256), 64, "bf16", 2),
    ("bf16_decode_17", 320, (32, 608, 288, 352), 17, "bf16", 2),
    ("bf16_decode_long_k", 256, (2080, 64, 1056, 992), 30, "bf16", 2),
    ("f32_decode", 256, (128, 384, 192, 320, 224, 288, 256, 256), 48, "f32", 2),
    # d_model that is not a multiple of 64 (a K tail in the decode kernel)
    ("bf16_decode_d96", 96, (32, 608, 288, 352), 20, "bf16", 2),
    ("bf16_decode_64_tokens_one_expert", 128, (160, 96), 64, "bf16", 1),
]


@pytest.mark.parametrize("case", FWD_CASES, ids=[c[0] for c in FWD_CASES])
def test_layer_fwd_parity(case):
    name, d, d_ff, T, dtype, k = case
    inp = make(name, d, d_ff, T, dtype, k)
    r = _runner(inp)
    r.fwd()
    from paper_2409_12210_amd.harness import to_host
    got = r.routing_host()
    idx, n_near = check_routing(inp, got)
    y_ref = orc.layer_fwd(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, d_ff, k, inp.logit_bias,
                          topk_idx=idx if n_near else None)
    assert max_rel(to_host(r.y), y_ref) <= TOL[dtype]
    # routing_out = NULL gives the same y, bit for bit
    y1 = r.y.clone()
    r.fwd(with_routing=False)
    import torch
    torch.cuda.synchronize()
    assert torch.equal(y1, r.y)


def test_layer_fwd_empty_expert_and_zero_tokens():
    from paper_2409_12210_amd.harness import to_host
    bias = np.array([0, -100.0, 0, 0], dtype=np.float32)
    d_ff = (128, 384, 192, 320)
    inp = make("empty", 256, d_ff, 400, "bf16", bias=bias)
    r = _runner(inp)
    r.fwd()
    got = r.routing_host()
    assert got["counts"][1] == 0
    y_ref = orc.layer_fwd(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, d_ff, 2, bias)
    assert max_rel(to_host(r.y), y_ref) <= TOL["bf16"]
    # T == 0 is a no-op that must not touch the GPU
    inp0 = make("zero", 256, d_ff, 0, "bf16")
    r0 = _runner(inp0)
    r0.fwd()
    r0.route()


def test_equal_size_experts_match_uniform_moe():
    from paper_2409_12210_amd.harness import to_host
    d_ff = (256,) * 8
    inp = make("uniform", 256, d_ff, 600, "bf16")
    r = _runner(inp)
    r.fwd()
    y_ref = orc.layer_fwd_dense(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, d_ff, 2)
    assert max_rel(to_host(r.y), y_ref) <= TOL["bf16"]


BWD_CASES = [
    ("c0", 256, (128, 384, 192, 320, 224, 288, 256, 256), 512, "f32", 2),
    ("f32_ragged", 128, (32, 224, 96, 160), 203, "f32", 2),
    ("f32_top1", 128, (32, 224, 96, 160), 150, "f32", 1),
    ("bf16_mid", 512, (96, 416, 160, 352, 224, 288, 256, 256), 1000, "bf16", 2),
    ("bf16_tails", 320, (32, 608, 288, 352), 1531, "bf16", 2),
    ("bf16_decode", 320, (32, 608, 288, 352), 40, "bf16", 2),   # forward with saved activations: no split-K
    # many experts: the fused weight-gradient plan is full (3 x 64 problems), several experts get no token
    ("bf16_n64", 64, tuple(32 * (1 + e % 4) for e in range(64)), 300, "bf16", 2),
    ("f32_n32", 96, tuple(32 * (1 + e % 3) for e in range(32)), 257, "f32", 2),
]


def check_grads(r, inp, idx, tol):
    from paper_2409_12210_amd.harness import to_host
    c = inp.cfg
    g = orc.layer_bwd(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, c.d_ff, c.top_k, inp.dY, inp.logit_bias,
                      topk_idx=idx)
    errs = {"dX": max_rel(to_host(r.dX), g.dX), "dW_gate": max_rel(to_host(r.dW_gate), g.dW_gate),
            "dW1": max_rel(to_host(r.dW1), g.dW1), "dW3": max_rel(to_host(r.dW3), g.dW3),
            "dW2": max_rel(to_host(r.dW2), g.dW2)}
    for name, e in errs.items():
        assert e <= tol, (name, e, errs)
    return g


@pytest.mark.parametrize("case", BWD_CASES, ids=[c[0] for c in BWD_CASES])
def test_layer_bwd_parity(case):
    import torch
    name, d, d_ff, T, dtype, k = case
    inp = make(name, d, d_ff, T, dtype, k, need_dy=True)
    r = _runner(inp, need_bwd=True)
    r.fwd()
    r.bwd()
    idx, _ = check_routing(inp, r.routing_host())
    g = check_grads(r, inp, idx, TOL[dtype])
    # accumulate = 1 adds to the existing weight gradients
    before = r.dW1.clone()
    r.bwd(accumulate=True)
    torch.cuda.synchronize()
    assert max_rel(r.dW1.cpu().numpy(), 2 * g.dW1) <= TOL[dtype]
    assert torch.allclose(r.dW1, 2 * before, rtol=1e-5, atol=0)


def test_bwd_expert_without_tokens_gets_zero_gradient():
    bias = np.array([0, -100.0, 0, 0], dtype=np.float32)
    d_ff = (128, 384, 192, 320)
    inp = make("empty_bwd", 256, d_ff, 300, "bf16", need_dy=True, bias=bias)
    r = _runner(inp, need_bwd=True)
    r.dW1.fill_(7.0)
    r.dW2.fill_(7.0)
    r.fwd()
    r.bwd()
    idx, _ = check_routing(inp, r.routing_host())
    check_grads(r, inp, idx, TOL["bf16"])
    assert float(r.dW1[128:512].abs().max()) == 0.0
    assert float(r.dW_gate[:, 1].abs().max()) == 0.0


def test_results_are_deterministic():
    import torch
    inp = make("det", 512, (96, 416, 160, 352, 224, 288, 256, 256), 1000, "bf16", need_dy=True)
    r = _runner(inp, need_bwd=True)
    r.fwd(); r.bwd()
    torch.cuda.synchronize()
    keep = [t.clone() for t in (r.y, r.dX, r.dW_gate, r.dW1, r.dW3, r.dW2, r.routing.row_of, r.routing.src_of)]
    r.fwd(); r.bwd()
    torch.cuda.synchronize()
    for a, b in zip(keep, (r.y, r.dX, r.dW_gate, r.dW1, r.dW3, r.dW2, r.routing.row_of, r.routing.src_of)):
        assert torch.equal(a, b)


def test_layer_replays_from_a_hip_graph():
    """The entry points allocate nothing and never synchronise, so a forward + backward pass can be captured
    once into a HIP graph and replayed; every replay must reproduce the eager results bit for bit (with
    eager work and synchronisations in between)."""
    import torch
    inp = make("graph", 256, (128, 384, 192, 320, 224, 288, 256, 256), 700, "bf16", need_dy=True)
    r = _runner(inp, need_bwd=True)
    r.fwd()
    r.bwd()
    torch.cuda.synchronize()
    want = {n: getattr(r, n).clone() for n in ("y", "dX", "dW_gate", "dW1", "dW3", "dW2")}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        r.fwd()          # warm-up on the capture stream
        r.bwd()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            r.fwd()
            r.bwd()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for n in want:
            getattr(r, n).zero_()                      # eager work between the replays
        x2 = (r.x.float() * 2).sum()                   # (a library reduction on the default stream)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, v in want.items():
            assert torch.equal(getattr(r, n), v), (rep, n)
        assert torch.isfinite(x2)
