"""Seeded synthetic workloads for SpecTr-GBV verification.

This module only manufactures inputs (logits and draft tokens); it contains none
of the verification arithmetic and is the one piece of code that both the GPU
tests/benchmark and the CPU oracle tests use.

The paper evaluates on LLM logits (Section 6: DeepSeek / CodeLlama / Vicuna
pairs on five public datasets); neither weights nor datasets are available
here, so Gaussian logits with a Zipf-boosted head stand in for them.  What is
kept from the real workload is its *structure* (Algorithm 3): for one prefix,
K drafts are sampled i.i.d. from the draft model, position by position, and
every conditional distribution is a function of the token block it is
conditioned on -- two drafts that share their first r tokens see the same row
r of both models (row 0 is shared by all K drafts).

Recipe for one row (conditioned on prefix index b and token block x^r):
  target logits  z_q ~ N(0, sigma_t^2) i.i.d. over the vocabulary;
  head boost     `head` distinct token ids, chosen uniformly, get
                 + (boost - zipf_a * ln(rank)), rank = 1..head;
  draft logits   z_p = draft_scale * z_q + N(0, sigma_d^2);
  bf16 configs   both rows are rounded to bfloat16 (round-to-nearest-even)
                 before anything else looks at them;
  draft token    x^(r+1) ~ softmax(z_p / T) (Gumbel-max on the stored values),
                 drawn independently for each draft k.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Sequence

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    K: int
    L: int
    V: int
    dtype: str            # "f32" or "bf16"
    sigma_t: float
    sigma_d: float
    draft_scale: float = 1.0
    head: int = 0
    zipf_a: float = 1.1
    boost: float = 6.0
    temperature: float = 1.0

    @property
    def row_pairs(self) -> int:
        return self.batch * self.K * self.L

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def algorithmic_bytes(self) -> int:
        """Every (target, draft) row pair r = 0..L-1 read once, plus one row pair per prefix
        for the final token."""
        return (self.row_pairs + self.batch) * self.V * 2 * self.elem_bytes


# The five configurations of the benchmark definition (cfg3 has three noise levels).
WORKLOADS: Dict[str, Workload] = {
    "cfg1": Workload("cfg1", 1, 2, 4, 1000, "f32", 2.0, 0.5, temperature=1.0),
    "cfg2": Workload("cfg2", 8, 4, 5, 32000, "f32", 3.0, 1.0, head=50, zipf_a=1.1, temperature=1.0),
    "cfg3": Workload("cfg3", 64, 8, 8, 32000, "f32", 3.0, 1.0, head=50, zipf_a=1.1, temperature=0.8),
    "cfg3_lo": Workload("cfg3_lo", 64, 8, 8, 32000, "f32", 3.0, 0.25, head=50, zipf_a=1.1, temperature=0.8),
    "cfg3_hi": Workload("cfg3_hi", 64, 8, 8, 32000, "f32", 3.0, 2.0, head=50, zipf_a=1.1, temperature=0.8),
    "cfg4": Workload("cfg4", 32, 8, 8, 128256, "bf16", 3.0, 1.0, head=200, zipf_a=1.1, temperature=1.0),
    "cfg5": Workload("cfg5", 128, 16, 8, 152064, "bf16", 3.5, 1.5, draft_scale=0.8, head=500, zipf_a=1.05,
                     temperature=0.7),
}


def with_batch(w: Workload, batch: int) -> Workload:
    return replace(w, batch=batch)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _row_rng(seed: int, b: int, block: Sequence[int]) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([0x5EC6B7, seed, b, len(block), *[int(t) for t in block]]))


def _token_rng(seed: int, b: int, k: int, r: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([0x70CE4, seed, b, k, r]))


def _make_row(w: Workload, seed: int, b: int, block: Sequence[int], need_draft: bool):
    rng = _row_rng(seed, b, block)
    zq = rng.standard_normal(w.V, dtype=np.float32) * np.float32(w.sigma_t)
    if w.head > 0:
        ids = rng.choice(w.V, size=min(w.head, w.V), replace=False)
        ranks = np.arange(1, ids.size + 1, dtype=np.float64)
        zq[ids] += (w.boost - w.zipf_a * np.log(ranks)).astype(np.float32)
    zp = None
    if need_draft:
        zp = np.float32(w.draft_scale) * zq + rng.standard_normal(w.V, dtype=np.float32) * np.float32(w.sigma_d)
    if w.dtype == "bf16":
        zq = f32_to_bf16_bits(zq)
        zp = f32_to_bf16_bits(zp) if zp is not None else None
    return zq, zp


def make_prefix(w: Workload, seed: int, b: int):
    """Inputs of prefix b: target [K, L+1, V], draft [K, L, V], tokens [K, L] (int32).

    Logit arrays are float32, or uint16 holding bfloat16 bits for bf16 workloads.
    """
    store = np.uint16 if w.dtype == "bf16" else np.float32
    target = np.empty((w.K, w.L + 1, w.V), dtype=store)
    draft = np.empty((w.K, w.L, w.V), dtype=store)
    tokens = np.empty((w.K, w.L), dtype=np.int32)
    inv_T = np.float32(1.0 / w.temperature)
    for r in range(w.L + 1):
        cache = {}
        for k in range(w.K):
            block = tuple(int(t) for t in tokens[k, :r])
            if block not in cache:
                cache[block] = _make_row(w, seed, b, block, need_draft=(r < w.L))
            zq, zp = cache[block]
            target[k, r] = zq
            if r < w.L:
                draft[k, r] = zp
                zpf = bf16_bits_to_f32(zp) if w.dtype == "bf16" else zp
                g = _token_rng(seed, b, k, r).gumbel(size=w.V).astype(np.float32)
                tokens[k, r] = int(np.argmax(zpf * inv_T + g))
    return target, draft, tokens


def make_inputs(w: Workload, seed: int = 0, prefixes: Optional[Sequence[int]] = None):
    """Stack make_prefix over the batch (or over the listed prefix indices).

    The prefix index b seeds the rows, so a subset reproduces exactly the rows the full
    batch would hold at those indices.
    """
    idx = list(range(w.batch)) if prefixes is None else list(prefixes)
    store = np.uint16 if w.dtype == "bf16" else np.float32
    target = np.empty((len(idx), w.K, w.L + 1, w.V), dtype=store)
    draft = np.empty((len(idx), w.K, w.L, w.V), dtype=store)
    tokens = np.empty((len(idx), w.K, w.L), dtype=np.int32)
    for j, b in enumerate(idx):
        target[j], draft[j], tokens[j] = make_prefix(w, seed, b)
    return target, draft, tokens


def tables_to_inputs(p_of, q_of, V: int, L: int, K: int, n: int, seed: int):
    """Inputs for n independent prefixes that all share small conditional tables.

    p_of(block) / q_of(block) return the length-V probability vectors (strictly positive)
    conditioned on the token block (a tuple).  Logits are the float32 logs of those
    probabilities; drafts are drawn i.i.d. from p with numpy.  Used by the Monte-Carlo
    pins of the oracle.
    """
    import itertools
    rng = np.random.default_rng(seed)
    tokens = np.empty((n, K, L), dtype=np.int32)
    target = np.empty((n, K, L + 1, V), dtype=np.float32)
    draft = np.empty((n, K, L, V), dtype=np.float32)
    u = rng.random((n, K, L))
    code = np.zeros((n, K), dtype=np.int64)          # block as a base-V number
    for r in range(L + 1):
        blocks = list(itertools.product(range(V), repeat=r))
        logq = np.stack([np.log(np.asarray([float(v) for v in q_of(bl)], dtype=np.float64)) for bl in blocks])
        target[:, :, r, :] = logq.astype(np.float32)[code]
        if r == L:
            break
        p = np.stack([np.asarray([float(v) for v in p_of(bl)], dtype=np.float64) for bl in blocks])
        draft[:, :, r, :] = np.log(p).astype(np.float32)[code]
        cdf = np.cumsum(p, axis=1) / p.sum(axis=1, keepdims=True)
        t = (u[:, :, r, None] >= cdf[code]).sum(axis=-1)
        t = np.minimum(t, V - 1).astype(np.int32)
        tokens[:, :, r] = t
        code = code * V + t
    return target, draft, tokens
