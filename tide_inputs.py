"""Seeded synthetic inputs for the TIDE MoE-step hot path.

This module only *draws data*: expert / router weights, the per-expert router
bias, and the drifting hidden-state stream, at the shapes of the five workload
configurations.  It contains none of the method's arithmetic (no routing, no
expert evaluation, no refresh rule) and is the one module that both the CPU
oracle's tests and the HIP path's tests import.

bf16 tensors are carried as ``numpy.uint16`` bit patterns (the upper half of the
IEEE fp32 word), so that neither numpy nor the consumers need a bf16 dtype.

Paper context: the workloads stand in for LLaDA2.0-mini / LLaDA2.0-flash
(256 routed experts, top-8; Sec. 4.1 "Models and Datasets") decoding with a
block length of 32 (Table 1 caption), whose expert routing is temporally stable
(mean adjacent-step cosine similarity 0.985, Sec. 3.2).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Iterator, Optional, Tuple

import numpy as np

GATING_SOFTMAX = 0
GATING_SIGMOID = 1

BIAS_NONE = 0
BIAS_LOGIT = 1      # bias added to the router logit before the gate
BIAS_SELECT = 2     # bias added to the gate score for selection only


@dataclasses.dataclass(frozen=True)
class TideWorkload:
    """Shape + schedule of one synthetic workload (symbols follow the paper
    where it has them: E experts, k per token, tau = refresh interval ``K``,
    GPU expert budget B = ``C``)."""
    name: str
    d: int            # hidden size
    E: int            # routed experts per layer
    k: int            # experts per token
    I: int            # SwiGLU intermediate size
    n_shared: int     # always-resident shared experts (0 or 1)
    N: int            # tokens per denoise step (sequences x block length)
    S: int            # denoise steps per block
    K: int            # refresh interval (the paper's tau)
    C: int            # GPU cache capacity in experts (the paper's B)
    L: int            # MoE layers
    gating: int
    bias_mode: int
    seed: int = 20179

    @property
    def expert_elems(self) -> int:
        return 3 * self.d * self.I

    @property
    def expert_bytes(self) -> int:
        return 2 * self.expert_elems

    def replace(self, **kw) -> "TideWorkload":
        return dataclasses.replace(self, **kw)


# The five configurations (tokens per step N = batch x block length 32).
CONFIGS = {
    0: TideWorkload("cfg0-tiny", d=256, E=16, k=2, I=128, n_shared=0, N=8, S=4, K=2, C=8, L=1,
                    gating=GATING_SOFTMAX, bias_mode=BIAS_NONE),
    1: TideWorkload("cfg1-mini-layer", d=2048, E=256, k=8, I=512, n_shared=1, N=32, S=32, K=4, C=64, L=1,
                    gating=GATING_SIGMOID, bias_mode=BIAS_LOGIT),
    2: TideWorkload("cfg2-mini-stack", d=2048, E=256, k=8, I=512, n_shared=1, N=256, S=32, K=4, C=64, L=20,
                    gating=GATING_SIGMOID, bias_mode=BIAS_LOGIT),
    3: TideWorkload("cfg3-flash-layer", d=4096, E=256, k=8, I=1024, n_shared=1, N=512, S=32, K=4, C=64, L=1,
                    gating=GATING_SIGMOID, bias_mode=BIAS_LOGIT),
    4: TideWorkload("cfg4-flash-stack", d=4096, E=256, k=8, I=1024, n_shared=1, N=2048, S=32, K=4, C=64, L=32,
                    gating=GATING_SIGMOID, bias_mode=BIAS_LOGIT),
}

# tensor ids for sub-stream keys
_T_GATE, _T_UP, _T_DOWN, _T_ROUTER, _T_BIAS, _T_HIDDEN = range(6)

WEIGHT_STD = 0.02
ZIPF_S = 1.1
BIAS_GAMMA = 0.25


# --------------------------------------------------------------------------
# bf16 <-> fp32 bit helpers (data preparation only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(wl: TideWorkload, layer: int, tensor: int, index: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([wl.seed, layer, tensor, index])
    return np.random.Generator(np.random.SFC64(ss))


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------
def expert_weights(wl: TideWorkload, layer: int, expert: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """bf16 bits of (W_gate[I,d], W_up[I,d], W_down[d,I]) ~ N(0, 0.02^2).

    ``expert`` in [0, E) is a routed expert; ``expert == E`` is the shared one."""
    out = []
    for t, shape in ((_T_GATE, (wl.I, wl.d)), (_T_UP, (wl.I, wl.d)), (_T_DOWN, (wl.d, wl.I))):
        g = _rng(wl, layer, t, expert)
        w = g.standard_normal(shape, dtype=np.float32) * np.float32(WEIGHT_STD)
        out.append(f32_to_bf16_bits(w))
    return tuple(out)


def router_weights(wl: TideWorkload, layer: int) -> np.ndarray:
    """fp32 router matrix W_r[E,d] ~ N(0, 0.02^2)."""
    g = _rng(wl, layer, _T_ROUTER)
    return (g.standard_normal((wl.E, wl.d), dtype=np.float32) * np.float32(WEIGHT_STD)).astype(np.float32)


def router_bias(wl: TideWorkload, layer: int) -> Optional[np.ndarray]:
    """Per-expert offset that skews expert popularity Zipf-like:
    b[e] = -gamma * s * ln(rank_e), rank = seeded permutation of 1..E."""
    if wl.bias_mode == BIAS_NONE:
        return None
    g = _rng(wl, layer, _T_BIAS)
    rank = g.permutation(wl.E) + 1
    b = -BIAS_GAMMA * ZIPF_S * np.log(rank.astype(np.float64))
    return b.astype(np.float32)


# --------------------------------------------------------------------------
# hidden-state stream
# --------------------------------------------------------------------------
def hidden_stream(wl: TideWorkload, layer: int, n_steps: Optional[int] = None) -> Iterator[np.ndarray]:
    """Yield the bf16 bits of the step input h_t[N,d] for t = 0..S-1.

    h_0 ~ N(0,1); h_t = 0.95 h_{t-1} + 0.05 eps_t in fp32; each step's input is
    the bf16 rounding of h_t (the fp32 state itself is carried unrounded)."""
    g = _rng(wl, layer, _T_HIDDEN)
    steps = wl.S if n_steps is None else n_steps
    h = g.standard_normal((wl.N, wl.d), dtype=np.float32)
    for t in range(steps):
        if t > 0:
            eps = g.standard_normal((wl.N, wl.d), dtype=np.float32)
            h = np.float32(0.95) * h + np.float32(0.05) * eps
        yield f32_to_bf16_bits(h)


def initial_resident(wl: TideWorkload) -> np.ndarray:
    """Cold-start placement: experts 0..C-1 sit in slots 0..C-1."""
    return np.arange(wl.C, dtype=np.int32)


def refresh_steps(wl: TideWorkload) -> list:
    """Steps at which the driver refreshes before routing (t > 0, t % K == 0)."""
    return [t for t in range(1, wl.S) if t % wl.K == 0]
