"""Synthetic workloads: the benchmark/test configurations and their seeded inputs.

Holds no arithmetic of the method -- only shapes, seeds and random draws.  Both
the GPU tests/benchmark and the CPU oracle's tests draw their inputs from here
so that the two sides see identical bits.

The shapes stand in for the paper's workloads: sentence-classification batches
(32 sentences, k=4; Sec. 4.1 and the text-classification hyper-parameter table),
character-level language modelling with context up to 8192 (Sec. 4.2, context
length ablation), 8 heads of width 64 (language-modelling hyper-parameter
table: d=512, h=8).  Values are i.i.d. normal; no dataset is involved.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np

SEED_BASE = 191104070
TENSOR_INDEX = {"Q": 0, "K": 1, "V": 2, "Rel": 3, "dO": 4}
REL_STD = 0.02


@dataclass(frozen=True)
class Workload:
    name: str
    index: int          # configuration number (1-based), enters the seed
    n: int              # tokens (power of two)
    k: int              # connection density
    causal: bool
    B: int
    H: int
    D: int
    dtype: str          # "f32" or "bf16": storage type of Q,K,V,Rel,dO,out
    backward: bool
    length_mix: str = ""  # "" = every sequence has n tokens; else the recipe of make_lengths

    @property
    def num_nodes(self) -> int:
        return 2 * self.n - 1

    @property
    def num_levels(self) -> int:
        return self.n.bit_length()          # log2(n) + 1 for a power of two

    @property
    def rel_width(self) -> int:
        return 2 * (self.k + 1) + 1

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", 1, 512, 4, False, 1, 1, 64, "f32", False),
    "cls": Workload("cls", 2, 512, 4, False, 32, 8, 64, "bf16", True),
    "lm": Workload("lm", 3, 8192, 8, True, 4, 8, 64, "bf16", True),
    "xl": Workload("xl", 4, 65536, 4, True, 1, 8, 64, "bf16", True),
}
for _k in (2, 4, 8, 16, 32):
    WORKLOADS["ksweep%d" % _k] = Workload("ksweep%d" % _k, 5, 4096, _k, False, 8, 8, 64, "bf16", True)


# the sentence-classification batch with sentences of different lengths padded to n (the text
# corpora of Sec. 4.1 hold sentences and reviews of very different lengths)
WORKLOADS["cls_lengths"] = replace(WORKLOADS["cls"], name="cls_lengths", index=6, length_mix="reviews")
# forward only, as in the paper's inference throughput comparison (Sec. 4.4)
WORKLOADS["lm_infer"] = replace(WORKLOADS["lm"], name="lm_infer", backward=False)
WORKLOADS["lm_lengths"] = replace(WORKLOADS["lm"], name="lm_lengths", index=7, B=8, length_mix="reviews")
# the density of the paper's character-level language models (Sec. 4.2: k = 64 on contexts of 8192)
WORKLOADS["charlm"] = replace(WORKLOADS["lm"], name="charlm", index=8, k=64)


def make_lengths(w: Workload) -> np.ndarray:
    """Token counts of the B sequences of a workload, int32.  "reviews": log-normal lengths with
    median 0.4 n and sigma 0.6, clipped to [8, n] -- a long-tailed mix like that of review
    and sentence corpora, where a batch padded to its longest member is about half padding."""
    if not w.length_mix:
        return np.full(w.B, w.n, dtype=np.int32)
    if w.length_mix != "reviews":
        raise ValueError("unknown length mix %r" % (w.length_mix,))
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 1000 * w.index + 77))
    x = np.exp(rng.normal(np.log(0.4 * w.n), 0.6, size=w.B))
    return np.clip(np.rint(x), 8, w.n).astype(np.int32)


def shrink(w: Workload, **kw) -> Workload:
    """A smaller/larger variant of a workload (same seeds family)."""
    return replace(w, **kw)


def round_to_bf16(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Round float32 to the nearest bfloat16 (ties to even).

    Returns (the rounded values as float32, the 16-bit patterns as uint16)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    bits = (r >> np.uint32(16)).astype(np.uint16)
    return r.view(np.float32), bits


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _draw(w: Workload, name: str, shape, std: float) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 1000 * w.index + TENSOR_INDEX[name]))
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x


def make_inputs(w: Workload, with_dO: bool = True) -> Dict[str, np.ndarray]:
    """Seeded inputs of a workload as float32 arrays already rounded to w.dtype.

    Q,K,V,dO: [B,H,N,D] ~ N(0,1);  Rel: [levels, W, D] ~ N(0, 0.02^2)."""
    shp = (w.B, w.H, w.num_nodes, w.D)
    out = {
        "Q": _draw(w, "Q", shp, 1.0),
        "K": _draw(w, "K", shp, 1.0),
        "V": _draw(w, "V", shp, 1.0),
        "Rel": _draw(w, "Rel", (w.num_levels, w.rel_width, w.D), REL_STD),
    }
    if with_dO:
        out["dO"] = _draw(w, "dO", shp, 1.0)
    if w.dtype == "bf16":
        for key in list(out):
            out[key] = round_to_bf16(out[key])[0]
    elif w.dtype != "f32":
        raise ValueError("unknown dtype %r" % (w.dtype,))
    return out
