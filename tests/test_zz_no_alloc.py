"""modse_route_static, the entry point that allocates nothing (its scratch is a device array inside the
library), against modse_route on the same inputs: every routing output bit for bit, on two calls in a row
that share the array, the second with fewer tokens.  Collected last on purpose."""
import numpy as np
import pytest
import torch

import paper_2409_12210_amd as m
import workloads as wl
from paper_2409_12210_amd.harness import LayerRunner, to_host

pytestmark = pytest.mark.gpu

FIELDS = ("topk_idx", "topk_w", "counts", "offsets", "row_of", "src_of", "near_tie_count")

# (name, d_model, d_ff, dtype, top_k, T of the first call, T of the second call)
CASES = [
    ("blocks_then_tokens", 256, (128, 384, 192, 320, 224, 288, 256, 256), "f32", 2, 5000, 50),
    ("bf16_ragged", 512, (96, 416, 160, 352, 224, 288, 256, 256), "bf16", 2, 20001, 1237),
    ("n64", 64, (32,) * 64, "f32", 2, 3000, 200),
    ("top1_tokens", 256, (128, 384, 192, 320), "bf16", 1, 64, 1),
]


def route_both(name, d, d_ff, dtype, k, T, seed):
    cfg = wl.LayerConfig(name, d, tuple(d_ff), k, T, dtype, seed=seed, dy_seed=seed + 1)
    r = LayerRunner.from_inputs(wl.make_inputs(cfg))
    r.route()
    want = r.routing_host()
    other = m.Routing.empty(T, len(d_ff), k, "cuda")
    for f in FIELDS:  # stale contents must not survive
        getattr(other, f).fill_(-7)
    before = torch.cuda.memory_allocated()
    m.modse_route_static(d, list(d_ff), k, dtype, T, r.x, r.W_gate, r.bias, other)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for f in FIELDS:
        got = to_host(getattr(other, f))
        assert got.dtype == want[f].dtype and got.shape == want[f].shape, f
        assert np.array_equal(got.view(np.int32), want[f].view(np.int32)), (name, T, f)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_route_static_matches_route_on_two_calls_in_a_row(case):
    name, d, d_ff, dtype, k, T_first, T_second = case
    route_both(name, d, d_ff, dtype, k, T_first, seed=11)
    route_both(name, d, d_ff, dtype, k, T_second, seed=12)


def test_route_static_rejects_more_tokens_than_the_array_serves():
    d_ff = [32] * 64
    T = 1 << 18
    x = torch.zeros(8, device="cuda")
    r = m.Routing.empty(8, 64, 2, "cuda")
    code = m.modse_route_static(64, d_ff, 2, "f32", T, x, x, None, r, raise_on_error=False)
    assert code == 3 and "workspace" in m.modse_status_string(code)
    with pytest.raises(m.ModseError):
        m.modse_route_static(64, d_ff, 2, "f32", T, x, x, None, r)
