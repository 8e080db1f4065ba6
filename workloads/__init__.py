"""Seeded synthetic workloads for the fragment outer step.

This module only *makes inputs*: decoder-shaped parameter lists and random
replicas around a random global model.  It holds none of the method's
arithmetic (no outer gradient, no codec, no optimizer, no merge) and is the one
module that both the GPU tests/benchmark and the CPU oracle tests may import.

The tensors stand in for the outer gradients of the paper's C4 / Dolma runs
(Section 3.2 and the architecture table of the appendix give the shapes; the
trained weights themselves are not available): a global model g ~ N(0, 0.02),
zero outer momentum, per-replica deltas of a chosen distribution, and tau
further inner steps of N(0, 1e-4) noise per replica.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import torch

UNIT_PRE, UNIT_POST = -1, -2
GEN_CHUNK = 1 << 24          # elements generated per seeded draw (part of the recipe)


# --------------------------------------------------------------------------- shapes

@dataclass(frozen=True)
class DecoderShape:
    name: str
    n_layers: int
    d_model: int
    d_ffn: int
    vocab: int = 32000

    def units(self) -> Tuple[List[int], List[int], List[str]]:
        """Flat parameter-group list (numel, owning block, name) in model order:
        embedding, per block [attn norm, q, k, v, o, ffn norm, up, down], final norm, head."""
        d, f, v = self.d_model, self.d_ffn, self.vocab
        numel, block, names = [v * d], [UNIT_PRE], ["embed"]
        for i in range(self.n_layers):
            for nm, sz in (("attn_norm", d), ("q", d * d), ("k", d * d), ("v", d * d), ("o", d * d),
                           ("ffn_norm", d), ("up", d * f), ("down", f * d)):
                numel.append(sz), block.append(i), names.append(f"block{i}.{nm}")
        numel += [d, v * d]
        block += [UNIT_POST, UNIT_POST]
        names += ["final_norm", "head"]
        return numel, block, names


SHAPES: Dict[str, DecoderShape] = {
    "100m": DecoderShape("100m", 12, 768, 3072),
    "1b": DecoderShape("1b", 24, 2048, 8192),
    "4b": DecoderShape("4b", 36, 3072, 12288),
}


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration: what is synchronised, by how many replicas, how."""
    name: str
    shape: Optional[str]        # key of SHAPES, or None for a single flat span
    flat_numel: int             # used when shape is None
    P: int
    H: int
    tau: int
    M: int
    alpha: float
    lr: float
    mu: float
    delta: str                  # "normal" | "student_t3" | "outliers" | "shared<percent>"
    fmt: str                    # "e3m0" | "e4m3" | "bf16" | "fp32"
    seed: int = 0


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", None, 1 << 20, 1, 100, 1, 2, 0.5, 0.7, 0.9, "normal", "e3m0"),
    "100m": Workload("100m", "100m", 0, 3, 100, 1, 2, 0.5, 0.7, 0.9, "normal", "e3m0"),
    "1b": Workload("1b", "1b", 0, 4, 100, 5, 4, 0.5, 0.7, 0.9, "student_t3", "e3m0"),
    "4b_p6": Workload("4b_p6", "4b", 0, 6, 100, 1, 2, 0.5, 0.7, 0.9, "normal", "e3m0"),
    "4b_p1": Workload("4b_p1", "4b", 0, 1, 100, 1, 2, 0.5, 0.7, 0.9, "normal", "e3m0"),
    "stress": Workload("stress", "1b", 0, 4, 100, 1, 8, 0.5, 0.7, 0.9, "outliers", "e3m0"),
}


# ----------------------------------------------------------------------- generators

def _seed(base: int, unit: int, worker: int, role: str, chunk: int) -> int:
    h = hashlib.blake2b(f"{base}/{unit}/{worker}/{role}/{chunk}".encode(), digest_size=8).digest()
    return int.from_bytes(h, "little") & ((1 << 62) - 1)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _randn(n, device, seed):
    return torch.randn(n, dtype=torch.float32, device=device, generator=_gen(device, seed))


def _delta(kind: str, n: int, device, seed: int) -> torch.Tensor:
    if kind == "normal":
        return _randn(n, device, seed) * 1e-3
    if kind == "student_t3":
        # t(3) = Z / sqrt(chi2_3 / 3), chi2_3 = sum of three squared normals
        z = _randn(4 * n, device, seed).view(4, n)
        chi2 = (z[1:] ** 2).sum(0)
        return z[0] / torch.sqrt(chi2 / 3.0) * 1e-3
    if kind == "outliers":
        z = _randn(2 * n, device, seed).view(2, n)
        u = torch.rand(n, dtype=torch.float32, device=device, generator=_gen(device, seed + 1))
        big = torch.where(z[1] >= 0, 1e-1, -1e-1).to(torch.float32)
        return torch.where(u < 1e-3, big, z[0] * 1e-3)
    raise ValueError(kind)


def fill_span(g: torch.Tensor, mom: torch.Tensor, w_send: List[torch.Tensor],
              w_now: List[torch.Tensor], *, unit: int, tau: int, delta: str, base_seed: int = 0):
    """Fill one span's slices in place.  g, mom: fp32 [n]; w_send[m], w_now[m]: bf16 [n]
    (w_now[m] may be the same tensor as w_send[m] when tau == 0)."""
    n, device = g.numel(), g.device
    for c, lo in enumerate(range(0, n, GEN_CHUNK)):
        hi = min(lo + GEN_CHUNK, n)
        k = hi - lo
        gc = _randn(k, device, _seed(base_seed, unit, -1, "g", c)) * 0.02
        g[lo:hi] = gc
        mom[lo:hi] = 0
        rho, common = 0.0, None
        if delta.startswith("shared"):
            # replicas' outer gradients correlate with coefficient rho (one common component)
            rho = float(delta[len("shared"):]) / 100.0
            common = _randn(k, device, _seed(base_seed, unit, -2, "shared", c)) * 1e-3
        for m in range(len(w_send)):
            if common is not None:
                own = _delta("normal", k, device, _seed(base_seed, unit, m, "delta", c))
                d = common * rho ** 0.5 + own * (1.0 - rho) ** 0.5
            else:
                d = _delta(delta, k, device, _seed(base_seed, unit, m, "delta", c))
            ws = (gc - d).to(torch.bfloat16)
            w_send[m][lo:hi] = ws
            if tau > 0:
                adv = ws.to(torch.float32)
                for step in range(tau):
                    adv = adv + _randn(k, device, _seed(base_seed, unit, m, f"inner{step}", c)) * 1e-4
                w_now[m][lo:hi] = adv.to(torch.bfloat16)


def make_span(n: int, M: int, *, tau: int = 1, delta: str = "normal", unit: int = 0,
              base_seed: int = 0, device="cpu"):
    """Allocate and fill one stand-alone span.  Returns (g, mom, w_send, w_now)."""
    g = torch.empty(n, dtype=torch.float32, device=device)
    mom = torch.empty(n, dtype=torch.float32, device=device)
    w_send = [torch.empty(n, dtype=torch.bfloat16, device=device) for _ in range(M)]
    w_now = w_send if tau == 0 else [torch.empty(n, dtype=torch.bfloat16, device=device)
                                     for _ in range(M)]
    fill_span(g, mom, w_send, w_now, unit=unit, tau=tau, delta=delta, base_seed=base_seed)
    return g, mom, w_send, w_now


def bf16_bits(t: torch.Tensor):
    """bf16 tensor -> numpy uint16 bit patterns (host copy)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view("uint16").copy()


def bits_bf16(a, device="cpu") -> torch.Tensor:
    """numpy uint16 bit patterns -> bf16 tensor."""
    return torch.from_numpy(a.view("int16").copy()).view(torch.bfloat16).to(device)
