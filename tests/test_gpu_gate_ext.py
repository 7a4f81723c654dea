"""GPU parity of the optional gate parts against the fp64 CPU oracle: the noise term of H(x) (Sec. 2
Eq. 4-5), the auxiliary load-balance loss (Sec. 3.2 Eq. 9-12) and the routing statistics (Appendix A).
Integers bit for bit (away from near-ties); floats to max|out - ref| <= tol * max|ref|, tol = 1e-4 (fp32)
or 2e-2 (bf16 inputs).  Probabilities, f, P, the loss and the pre-noise values are float32 results of
float64 arithmetic on the GPU: they are held to 1e-5."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import modse_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
GAMMA, EPS, ALPHA = 0.8, 1e-6, 0.01


def max_rel(a, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(a, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-300))


def host(t):
    return t.detach().to(torch.float32).cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def setup(d, d_ff, T, dtype, k, noise, aux, need_bwd, seed=5, noise_sigma=0.05):
    from paper_2409_12210_amd.harness import LayerRunner
    cfg = wl.LayerConfig("ext", d, tuple(d_ff), k, T, dtype, seed=seed, dy_seed=seed + 1)
    inp = wl.make_inputs(cfg, need_dy=need_bwd)
    Wn = wl.make_noise_weights(cfg, sigma=noise_sigma) if noise else None
    r = LayerRunner.from_inputs(inp, need_bwd=need_bwd)
    r.enable_ext(W_noise=Wn, gamma=GAMMA, eps=EPS, aux_alpha=ALPHA if aux else None)
    on = orc.Noise(Wn, GAMMA, EPS) if noise else None
    return inp, r, on


CASES = [
    ("f32_n8", 256, (128, 384, 192, 320, 224, 288, 256, 256), 501, "f32", 2),
    ("bf16_n8", 512, (96, 416, 160, 352, 224, 288, 256, 256), 1000, "bf16", 2),
    ("top1_n4", 256, (128, 384, 192, 320), 300, "bf16", 1),
    ("n16", 128, (64,) * 16, 333, "f32", 2),
    ("n3", 96, (32, 64, 96), 130, "bf16", 2),
    ("n32", 64, (32,) * 32, 150, "f32", 2),
    ("n64_f32", 64, (32,) * 64, 203, "f32", 2),
    ("n64_bf16", 96, (32,) * 64, 333, "bf16", 2),
    ("n40_bf16", 64, (32,) * 40, 97, "bf16", 2),
    ("decode_n8", 256, (128, 384, 192, 320, 224, 288, 256, 256), 40, "bf16", 2),
]
LAYER_CASES = CASES[:4] + CASES[5:8] + CASES[-1:]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("noise,aux", [(True, True), (True, False), (False, True)])
def test_route_ext_parity(case, noise, aux):
    name, d, d_ff, T, dtype, k = case
    inp, r, on = setup(d, d_ff, T, dtype, k, noise, aux, False)
    N = len(d_ff)
    r.route()
    got = r.routing_host()
    ref = orc.route(inp.x, inp.W_gate, N, k, None, on)
    near = orc.near_tie_mask(ref.logits, k)
    assert (got["topk_idx"][:T][~near] == ref.topk_idx[~near]).all()
    assert np.abs(got["topk_w"][:T][~near] - ref.topk_w[~near]).max() < 2e-7
    counts, offsets, row_of, src_of = orc.permutation_from_indices(got["topk_idx"][:T], N)
    assert (got["counts"] == counts).all() and (got["row_of"][:T] == row_of).all()
    if noise:
        u = orc.noise_term(inp.x, on)[1]
        assert max_rel(host(r.ext.noise_pre)[:T], u) < 1e-5
    if aux:
        L, f, P, p = orc.aux_loss(ref.logits, ALPHA)
        assert max_rel(host(r.ext.probs)[:T], p) < 1e-5
        if not near.any():
            assert np.abs(host(r.ext.aux_f) - f).max() < 1e-7
        assert max_rel(host(r.ext.aux_P), P) < 1e-5
        assert abs(host(r.ext.aux_loss)[0] - L) < 1e-5 * L + (1e-3 * L if near.any() else 0)
        # f comes from the same first choices that fill slot 0
        assert np.abs(host(r.ext.aux_f) - np.bincount(got["topk_idx"][:T, 0], minlength=N) / T).max() < 1e-7


@pytest.mark.parametrize("case", LAYER_CASES, ids=[c[0] for c in LAYER_CASES])
@pytest.mark.parametrize("noise,aux", [(True, True), (False, True), (True, False)])
def test_layer_fwd_bwd_ext_parity(case, noise, aux):
    name, d, d_ff, T, dtype, k = case
    inp, r, on = setup(d, d_ff, T, dtype, k, noise, aux, True)
    tol = TOL[dtype]
    aux_grad = 400.0 * T   # weight of L_a in the loss: large enough that its gradient shows beside dY's
    r.fwd()
    r.bwd(aux_grad=aux_grad)
    torch.cuda.synchronize()
    idx = host(r.routing.topk_idx)[:T]
    y_ref = orc.layer_fwd(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, inp.cfg.d_ff, k, topk_idx=idx, noise=on)
    assert max_rel(host(r.y), y_ref) <= tol
    G = orc.layer_bwd(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, inp.cfg.d_ff, k, inp.dY, topk_idx=idx, noise=on,
                      aux_alpha=ALPHA if aux else None, aux_grad=aux_grad)
    assert max_rel(host(r.dX), G.dX) <= tol
    assert max_rel(host(r.dW_gate), G.dW_gate) <= tol
    assert max_rel(host(r.dW1), G.dW1) <= tol
    assert max_rel(host(r.dW3), G.dW3) <= tol
    assert max_rel(host(r.dW2), G.dW2) <= tol
    if noise:
        assert max_rel(host(r.dW_noise), G.dW_noise) <= tol
        assert abs(host(r.dgamma)[0] - G.dgamma) <= tol * max(abs(G.dgamma), np.abs(G.dW_noise).max())
    if aux:
        # the auxiliary term really is in the gradient: without it dW_gate differs
        G0 = orc.layer_bwd(inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2, inp.cfg.d_ff, k, inp.dY, topk_idx=idx, noise=on,
                           need_weight_grads=False)
        assert max_rel(G0.dW_gate, G.dW_gate) > 0.1


def test_ext_accumulate_and_plain_path_unchanged():
    d, d_ff, T = 256, (128, 384, 192, 320, 224, 288, 256, 256), 400
    inp, r, on = setup(d, d_ff, T, "f32", 2, True, True, True)
    r.fwd()
    r.bwd(aux_grad=1.0)
    torch.cuda.synchronize()
    first = {n: host(getattr(r, n)).copy() for n in ("dW_noise", "dgamma", "dW_gate")}
    r.bwd(accumulate=True, aux_grad=1.0)
    torch.cuda.synchronize()
    for n, v in first.items():
        assert max_rel(host(getattr(r, n)), 2 * v) < 1e-6, n
    # an extension with both parts switched off gives the plain layer, bit for bit
    from paper_2409_12210_amd.harness import LayerRunner
    a = LayerRunner.from_inputs(inp, need_bwd=True)
    b = LayerRunner.from_inputs(inp, need_bwd=True)
    b.enable_ext()
    for q in (a, b):
        q.fwd()
        q.bwd()
    torch.cuda.synchronize()
    for n in ("y", "dX", "dW_gate", "dW1"):
        assert torch.equal(getattr(a, n), getattr(b, n)), n


def test_routing_stats_parity():
    from paper_2409_12210_amd.harness import LayerRunner
    for (d, d_ff, T, dtype, k) in [(256, (128, 384, 192, 320, 224, 288, 256, 256), 5000, "bf16", 2),
                                   (128, (64,) * 16, 777, "f32", 2), (256, (128, 384, 192, 320), 300, "bf16", 1),
                                   (64, (32,) * 64, 50, "f32", 2)]:
        cfg = wl.LayerConfig("st", d, tuple(d_ff), k, T, dtype, seed=9, dy_seed=10)
        inp = wl.make_inputs(cfg)
        r = LayerRunner.from_inputs(inp)
        r.route()
        sc, sm = r.stats()
        torch.cuda.synchronize()
        idx = host(r.routing.topk_idx)[:T]
        ref = orc.routing_stats(idx, d_ff)
        assert (host(sc) == ref.slot_counts).all()
        sm = host(sm)
        for j in range(k):
            assert (np.isinf(sm[j]) and np.isinf(ref.slot_ratio[j])) or abs(sm[j] - ref.slot_ratio[j]) < 1e-5 * ref.slot_ratio[j]
        assert (np.isinf(sm[k]) and np.isinf(ref.total_ratio)) or abs(sm[k] - ref.total_ratio) < 1e-5 * ref.total_ratio
        assert abs(sm[k + 1] - ref.avg_hidden) < 1e-5 * ref.avg_hidden
