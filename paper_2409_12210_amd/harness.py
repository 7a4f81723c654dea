"""Device-memory plumbing around the C ABI for tests and the benchmark: uploads host arrays as torch
tensors, allocates outputs and workspace, calls the binding, downloads results.  No arithmetic of the
layer happens here."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B


def to_device(a: Optional[np.ndarray], dtype: str, device="cuda"):
    """Host fp32 array -> device tensor of the layer's element type (bf16 values must already be
    bf16-representable; the conversion is then exact)."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


class LayerRunner:
    """Holds one layer's device tensors and calls modse_route / modse_layer_fwd / modse_layer_bwd."""

    def __init__(self, d_model, d_ff, top_k, dtype, T, x, W_gate, W1, W3, W2, logit_bias=None, dY=None,
                 need_bwd=False, device="cuda"):
        self.d, self.d_ff, self.k, self.dtype, self.T = int(d_model), [int(f) for f in d_ff], int(top_k), dtype, int(T)
        self.N, self.F = len(self.d_ff), int(sum(self.d_ff))
        self.device = device
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.x = to_device(x, dtype, device)
        self.W_gate = to_device(W_gate, dtype, device)
        self.W1 = to_device(W1, dtype, device)
        self.W3 = to_device(W3, dtype, device)
        self.W2 = to_device(W2, dtype, device)
        self.dY = to_device(dY, dtype, device)
        self.bias = None if logit_bias is None else torch.from_numpy(
            np.ascontiguousarray(logit_bias, dtype=np.float32)).to(device)
        self.need_bwd = need_bwd
        self.routing = B.Routing.empty(max(self.T, 1), self.N, self.k, device)
        self.y = torch.empty((self.T, self.d), dtype=self.tdtype, device=device)
        if need_bwd:  # the forward call is given `saved`: a small workspace
            ws_bytes = max(B.modse_workspace_size(self.d, self.d_ff, self.k, dtype, self.T, B.WS_FWD_SAVED),
                           B.modse_workspace_size(self.d, self.d_ff, self.k, dtype, self.T, B.WS_BWD))
        else:
            ws_bytes = B.modse_workspace_size(self.d, self.d_ff, self.k, dtype, self.T, B.WS_FWD)
        self.ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=device)
        self.saved = None
        if need_bwd:
            self.saved = torch.empty(max(B.modse_saved_size(self.d, self.d_ff, self.k, dtype, self.T), 256),
                                     dtype=torch.uint8, device=device)
            f32 = dict(dtype=torch.float32, device=device)
            self.dX = torch.empty((self.T, self.d), dtype=self.tdtype, device=device)
            self.dW_gate = torch.zeros((self.d, self.N), **f32)
            self.dW1 = torch.zeros((self.F, self.d), **f32)
            self.dW3 = torch.zeros((self.F, self.d), **f32)
            self.dW2 = torch.zeros(self.d * self.F, **f32)

    def enable_ext(self, W_noise=None, gamma=1.0, eps=1e-6, aux_alpha=None):
        """Switch on the optional gate parts: the noise term (W_noise given) and/or the auxiliary loss
        (aux_alpha given); allocates the buffers they need.  fwd / route / bwd then go through the *_ext calls."""
        f32 = dict(dtype=torch.float32, device=self.device)
        e = B.GateExt()
        Tn = max(self.T, 1)
        if W_noise is not None:
            e.W_noise = to_device(W_noise, self.dtype, self.device)
            e.gamma = torch.tensor([float(gamma)], **f32)
            e.eps = float(eps)
            e.noise_pre = torch.empty((Tn, self.N), **f32)
            self.dW_noise = torch.zeros((self.d, self.N), **f32)
            self.dgamma = torch.zeros(1, **f32)
        if aux_alpha is not None:
            e.aux_alpha = float(aux_alpha)
            e.probs = torch.empty((Tn, self.N), **f32)
            e.aux_f = torch.empty(self.N, **f32)
            e.aux_P = torch.empty(self.N, **f32)
            e.aux_loss = torch.empty(1, **f32)
        self.ext = e
        return e

    def stats(self):
        """slot_counts [k, N] and summary [k + 2] of the last routing (device tensors)."""
        sc = torch.empty((self.k, self.N), dtype=torch.int32, device=self.device)
        sm = torch.empty(self.k + 2, dtype=torch.float32, device=self.device)
        B.modse_routing_stats(*self._args(), self.routing, sc, sm)
        return sc, sm

    @classmethod
    def from_inputs(cls, inp, need_bwd=False, device="cuda"):
        c = inp.cfg
        return cls(c.d_model, c.d_ff, c.top_k, c.dtype, c.n_tokens, inp.x, inp.W_gate, inp.W1, inp.W3, inp.W2,
                   inp.logit_bias, inp.dY, need_bwd, device)

    def _args(self):
        return (self.d, self.d_ff, self.k, self.dtype, self.T)

    def route(self):
        if getattr(self, "ext", None) is not None:
            B.modse_route_ext(*self._args(), self.x, self.W_gate, self.bias, self.ext, self.routing, self.ws)
        else:
            B.modse_route(*self._args(), self.x, self.W_gate, self.bias, self.routing, self.ws)

    def fwd(self, with_routing=True, save=None):
        save = self.need_bwd if save is None else save
        if bool(save) != bool(self.need_bwd):
            raise ValueError("the workspace of this runner was sized for save == need_bwd")
        if getattr(self, "ext", None) is not None:
            B.modse_layer_fwd_ext(*self._args(), self.x, self.W_gate, self.bias, self.ext, self.W1, self.W3, self.W2,
                                  self.y, self.routing if with_routing else None, self.saved if save else None,
                                  self.ws)
            return
        B.modse_layer_fwd(*self._args(), self.x, self.W_gate, self.bias, self.W1, self.W3, self.W2, self.y,
                          self.routing if with_routing else None, self.saved if save else None, self.ws)

    def bwd(self, accumulate=False, aux_grad=1.0):
        if getattr(self, "ext", None) is not None:
            B.modse_layer_bwd_ext(*self._args(), self.x, self.W_gate, self.ext, aux_grad, self.W1, self.W3, self.W2,
                                  self.routing, self.saved, self.dY, self.dX, self.dW_gate,
                                  getattr(self, "dW_noise", None), getattr(self, "dgamma", None), self.dW1, self.dW3,
                                  self.dW2, accumulate, self.ws)
            return
        B.modse_layer_bwd(*self._args(), self.x, self.W_gate, self.W1, self.W3, self.W2, self.routing, self.saved,
                          self.dY, self.dX, self.dW_gate, self.dW1, self.dW3, self.dW2, accumulate, self.ws)

    def routing_host(self):
        torch.cuda.synchronize()
        r = self.routing
        return {k: to_host(getattr(r, k)) for k in
                ("topk_idx", "topk_w", "counts", "offsets", "row_of", "src_of", "near_tie_count")}
