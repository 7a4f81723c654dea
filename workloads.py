"""Seeded synthetic inputs for one MoDSE FFN layer.

This module is shared by the CPU oracle's tests and by the GPU path's tests and
benchmark.  It holds data generation only: shapes, random draws and dtype
rounding.  None of the layer's arithmetic (router, gating, experts, gradients)
lives here, and it imports neither the oracle nor the HIP binding.

Shapes follow the paper's setting: 8 experts, top-2 routing (Table 1), four
size pairs whose hidden widths sum to twice the uniform width (Sec. 3.1, the
pair constraint), d_model 2048 as in the 700Mx8 model.  Values are synthetic:
x ~ N(0,1); W_gate, W1, W3, W2 ~ N(0, 0.02^2); dY ~ N(0,1).

Random numbers come from numpy's counter-based Philox generator, one stream per
tensor keyed by (seed, tensor id), so a tensor does not change when another one
is resized.  For bf16 configs every tensor is rounded once to bf16
(round-to-nearest-even) on the host; both the oracle and the GPU consume those
rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np

TENSOR_IDS = {"x": 1, "W_gate": 2, "W1": 3, "W3": 4, "W2": 5, "dY": 6, "W_noise": 7}


@dataclass(frozen=True)
class LayerConfig:
    name: str
    d_model: int
    d_ff: tuple            # per-expert hidden width, expert order; pair p = experts (2p, 2p+1)
    top_k: int
    n_tokens: int
    dtype: str             # "f32" or "bf16"
    seed: int = 0
    dy_seed: int = 1
    zipf_s: Optional[float] = None   # skewed-routing stress case if set

    @property
    def n_experts(self) -> int:
        return len(self.d_ff)

    @property
    def F(self) -> int:
        return int(sum(self.d_ff))


# Expert size pairs of the paper's two models (Table 2), used as a fixture and
# as an optional harsher-ratio shape.
PAPER_PAIRS_300M = ((6912, 768), (6144, 1536), (4608, 3072), (3840, 3840))
PAPER_PAIRS_700M = ((9216, 1024), (8192, 2048), (6144, 4096), (5120, 5120))


def _flat(pairs):
    return tuple(int(v) for p in pairs for v in p)


CONFIGS: Dict[str, LayerConfig] = {
    # tiny fp32 parity case
    "C0": LayerConfig("C0", 256, (128, 384, 192, 320, 224, 288, 256, 256), 2, 512, "f32", seed=0),
    # headline bf16 forward case and its uniform twin
    "C1": LayerConfig("C1", 2048, (2816, 8448, 4224, 7040, 4928, 6336, 5632, 5632), 2, 16384, "bf16", seed=0),
    "C1U": LayerConfig("C1U", 2048, (5632,) * 8, 2, 16384, "bf16", seed=0),
    # skewed routing stress case (bias comes from tests/golden/zipf_bias_C2.txt)
    "C2": LayerConfig("C2", 2048, (2816, 8448, 4224, 7040, 4928, 6336, 5632, 5632), 2, 16384, "bf16", seed=0,
                      zipf_s=1.2),
    # decode-shaped weight-streaming case
    "C3": LayerConfig("C3", 4096, (7168, 21504, 10752, 17920, 12544, 16128, 14336, 14336), 2, 64, "bf16", seed=0),
    # training step
    "C4": LayerConfig("C4", 2048, (2816, 8448, 4224, 7040, 4928, 6336, 5632, 5632), 2, 32768, "bf16", seed=1),
    "C4U": LayerConfig("C4U", 2048, (5632,) * 8, 2, 32768, "bf16", seed=1),
    # the paper's own 700Mx8 widths (9:1 size ratio)
    "P700": LayerConfig("P700", 2048, _flat(PAPER_PAIRS_700M), 2, 16384, "bf16", seed=0),
}


def with_tokens(cfg: LayerConfig, n_tokens: int) -> LayerConfig:
    return replace(cfg, n_tokens=int(n_tokens), name=f"{cfg.name}@T{n_tokens}")


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array holding bf16-representable values (RNE)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array of bf16-representable values -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(seed: int, tensor: str, shape, sigma: float, dtype: str) -> np.ndarray:
    key = (int(seed) << 8) | TENSOR_IDS[tensor]
    g = np.random.Generator(np.random.Philox(key=key))
    a = g.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    if dtype == "bf16":
        a = round_to_bf16(a)
    return a


@dataclass
class LayerInputs:
    cfg: LayerConfig
    x: np.ndarray          # [T, d]
    W_gate: np.ndarray     # [d, N]
    W1: np.ndarray         # [F, d]  expert e owns rows foff[e]:foff[e+1]
    W3: np.ndarray         # [F, d]
    W2: np.ndarray         # [d*F] flat; expert e at d*foff[e], shape [d, f_e] row-major
    dY: Optional[np.ndarray] = None      # [T, d]
    logit_bias: Optional[np.ndarray] = None   # [N] float32 or None
    foff: List[int] = field(default_factory=list)


def expert_offsets(d_ff) -> List[int]:
    off = [0]
    for f in d_ff:
        off.append(off[-1] + int(f))
    return off


def make_inputs(cfg: LayerConfig, need_dy: bool = False, logit_bias=None) -> LayerInputs:
    T, d, N, F = cfg.n_tokens, cfg.d_model, cfg.n_experts, cfg.F
    x = _normal(cfg.seed, "x", (T, d), 1.0, cfg.dtype)
    Wg = _normal(cfg.seed, "W_gate", (d, N), 0.02, cfg.dtype)
    W1 = _normal(cfg.seed, "W1", (F, d), 0.02, cfg.dtype)
    W3 = _normal(cfg.seed, "W3", (F, d), 0.02, cfg.dtype)
    W2 = _normal(cfg.seed, "W2", (d * F,), 0.02, cfg.dtype)
    dY = _normal(cfg.dy_seed, "dY", (T, d), 1.0, cfg.dtype) if need_dy else None
    lb = None if logit_bias is None else np.ascontiguousarray(logit_bias, dtype=np.float32)
    return LayerInputs(cfg, x, Wg, W1, W3, W2, dY, lb, expert_offsets(cfg.d_ff))


def make_noise_weights(cfg: LayerConfig, sigma: float = 0.02) -> np.ndarray:
    """W_noise [d, N] of the optional noise term of the gate, drawn like the other weights (own stream)."""
    return _normal(cfg.seed, "W_noise", (cfg.d_model, cfg.n_experts), sigma, cfg.dtype)


def zipf_target_shares(d_ff, s: float) -> np.ndarray:
    """Target share of the T*k assignments per expert: rank experts by width,
    widest first (ties -> lower index); share proportional to rank^-s."""
    order = sorted(range(len(d_ff)), key=lambda e: (-d_ff[e], e))
    w = np.array([(r + 1) ** (-s) for r in range(len(d_ff))], dtype=np.float64)
    w /= w.sum()
    out = np.zeros(len(d_ff))
    for r, e in enumerate(order):
        out[e] = w[r]
    return out


def load_bias_fixture(path: str) -> np.ndarray:
    """Read a logit-bias fixture: '#' comment lines, then one float per line."""
    vals = []
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                vals.append(float(line))
    return np.array(vals, dtype=np.float32)


def sample_tokens(T: int, n: int, seed: int = 12345) -> np.ndarray:
    """A sorted, seeded sample of n distinct token indices out of T."""
    g = np.random.Generator(np.random.Philox(key=seed))
    if n >= T:
        return np.arange(T)
    return np.sort(g.choice(T, size=n, replace=False))
