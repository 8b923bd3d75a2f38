"""Seeded synthetic inputs for the SparseMoE expert hot path.

This module only *draws inputs*: tensors with the shapes and value
distributions of the paper's OLMoE-shaped MoE layers (Table 1: hidden size,
expert intermediate size, expert count, top-k; context 2048).  It contains
none of the layer's arithmetic (no softmax, top-k, permutation, SwiGLU,
combine) and imports neither the HIP binding nor the CPU oracle, so both can
be fed the very same bits.

bfloat16 tensors are carried on the host as ``uint16`` bit patterns; the
values are drawn in fp32 and rounded to nearest-even.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict

import numpy as np


@dataclass(frozen=True)
class MoEConfig:
    """Shape of one MoE layer invocation (paper notation in brackets).

    T tokens [T = EP*S], d hidden [H], E experts in the whole layer [N],
    k experts per token [K], f expert intermediate size, local experts
    ``[e_begin, e_begin + e_count)`` [n_start..n_end, NR = e_count].
    """

    name: str
    T: int
    d: int
    E: int
    k: int
    f: int
    e_begin: int = 0
    e_count: int = -1          # -1: all experts are local (no expert parallelism)
    logits: str = "router"     # "router" | "zipf" | "iid" | "fur"
    renormalize: int = 1
    seed: int = 0

    @property
    def n_local(self) -> int:
        return self.E if self.e_count < 0 else self.e_count

    @property
    def R_cap(self) -> int:
        """Upper bound on routed rows (T*k); the real R is known after routing."""
        return self.T * self.k


# The five workload shapes this build is measured and tested on.
CONFIGS: Dict[str, MoEConfig] = {
    # tiny layer the CPU oracle finishes in well under a second
    "tiny": MoEConfig("tiny", T=256, d=128, E=8, k=2, f=256),
    # OLMoE / Mula-7B-A1B shape (Table 1), 4 sequences of context 2048
    "olmoe": MoEConfig("olmoe", T=8192, d=2048, E=64, k=8, f=1024),
    # tiny shapes, Zipf(1.2) expert loads with two experts that get no token
    "skew": MoEConfig("skew", T=256, d=128, E=8, k=2, f=256, logits="zipf"),
    # one expert-parallel rank's share: 8 local experts of 64, ~32768 routed rows
    "ep_share": MoEConfig("ep_share", T=32768, d=4096, E=64, k=8, f=2048,
                          e_begin=0, e_count=8, logits="iid"),
    # fine-grained MoE: many small groups
    "fine": MoEConfig("fine", T=16384, d=2048, E=128, k=8, f=512),
    # the larger models of Table 1 under 12-way expert parallelism (Section 4.2): one rank's share
    # of the experts, tokens of all 12 ranks (12 sequences of context 2048)
    "mula100b_ep12": MoEConfig("mula100b_ep12", T=24576, d=3072, E=144, k=8, f=1536, e_begin=0, e_count=12),
    "mula220b_ep12": MoEConfig("mula220b_ep12", T=24576, d=3072, E=240, k=8, f=1536, e_begin=20, e_count=20),
    # the headline shape under forced uniform routing (Section 4.3): every expert gets exactly
    # T*k/E rows, in a fixed pattern
    "olmoe_fur": MoEConfig("olmoe_fur", T=8192, d=2048, E=64, k=8, f=1024, logits="fur"),
}


def with_overrides(cfg: MoEConfig, **kw) -> MoEConfig:
    return replace(cfg, **kw)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    """N(0, std) drawn in fp32, chunked so large tensors do not double memory."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for s in range(0, n, step):
        e = min(n, s + step)
        v = rng.standard_normal(e - s, dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        out[s:e] = f32_to_bf16_bits(v)
    return out.reshape(shape)


def zipf_bias(E: int, logit_std: float, s: float = 1.2, n_empty: int = 2) -> np.ndarray:
    """Per-expert additive logit bias that skews expert loads.

    The first ``E - n_empty`` experts get ``c * ln p_e`` with
    ``p_e ~ (e+1)^-s`` and ``c = logit_std / 1.283`` (the Gaussian logit noise
    stands in for Gumbel noise of unit scale, whose std is 1.283), the last
    ``n_empty`` experts get -1e4 and are never selected.
    """
    b = np.full(E, -1.0e4, dtype=np.float32)
    live = E - n_empty
    p = (np.arange(live, dtype=np.float64) + 1.0) ** (-s)
    p /= p.sum()
    b[:live] = (logit_std / 1.283 * np.log(p)).astype(np.float32)
    return b


def fur_logits(T: int, E: int, k: int) -> np.ndarray:
    """Logits that force uniform routing: slot i of token t goes to expert (t*k + i) mod E, with
    decreasing logits 1, 1 - 1/k, ... for its k slots and -20 for every other expert.  When E
    divides T*k every expert gets exactly T*k/E rows."""
    logits = np.full((T, E), -20.0, dtype=np.float32)
    t = np.arange(T)[:, None]
    i = np.arange(k)[None, :]
    logits[t, (t * k + i) % E] = (1.0 - i / k).astype(np.float32)
    return logits


def make_inputs(cfg: MoEConfig, with_weights: bool = True) -> Dict[str, np.ndarray]:
    """Draw one batch for ``cfg``.

    Returns a dict of host arrays:
      x      uint16 [T, d]      activations, N(0,1) as bf16 bits
      dout   uint16 [T, d]      upstream gradient, N(0,1) as bf16 bits
      logits float32 [T, E]     router logits (input of the routing step)
      Wg,Wu  uint16 [n_local, f, d], Wd uint16 [n_local, d, f]   N(0,0.02) as bf16 bits
      Wr     float32 [E, d]     the router weight the logits were made with ("router" and "zipf" only)
    Router logits are ``x @ Wr.T`` with ``Wr ~ N(0,0.02)`` fp32 ("router"),
    the same plus a Zipf bias ("zipf"), i.i.d. N(0,1) ("iid": every
    k-subset of experts is equally likely, as for already-dispatched tokens),
    or the fixed balanced pattern of ``fur_logits`` ("fur").
    """
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    T, d, E, f, nl = cfg.T, cfg.d, cfg.E, cfg.f, cfg.n_local
    out: Dict[str, np.ndarray] = {}
    out["x"] = _normal_bf16(rng, (T, d), 1.0)
    out["dout"] = _normal_bf16(rng, (T, d), 1.0)
    if cfg.logits == "iid":
        out["logits"] = rng.standard_normal((T, E), dtype=np.float32)
    elif cfg.logits == "fur":
        out["logits"] = fur_logits(T, E, cfg.k)
    else:
        Wr = rng.standard_normal((E, d), dtype=np.float32) * np.float32(0.02)
        logits = bf16_bits_to_f32(out["x"]) @ Wr.T
        if cfg.logits == "zipf":
            logits = logits + zipf_bias(E, float(logits.std()))[None, :]
        out["logits"] = np.ascontiguousarray(logits, dtype=np.float32)
        out["Wr"] = Wr
    if with_weights:
        out["Wg"] = _normal_bf16(rng, (nl, f, d), 0.02)
        out["Wu"] = _normal_bf16(rng, (nl, f, d), 0.02)
        out["Wd"] = _normal_bf16(rng, (nl, d, f), 0.02)
    return out
