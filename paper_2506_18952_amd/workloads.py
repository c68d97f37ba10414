"""Seeded synthetic logit workloads for the HSD batched-verify step.

This module serves both the HIP path's tests/benchmark and the CPU oracle's
tests.  It holds no step of the method (no softmax, entropy, acceptance test or
inverse CDF): drafted tokens are drawn with the Gumbel-max construction
(argmax of logits/T plus Gumbel noise), which needs none of them.

The paper (Section 4.1) evaluates on two public question-answering suites with
trained models; neither is available nor ever measured at the verify step, so
LLM-shaped synthetic logits stand in for them: a Gaussian body, a Zipf-like
rank-frequency head over a per-row random permutation, and occasional
near-deterministic ("peaked") rows.  Every sequence has its own PCG64 stream
keyed on (data seed, config, sequence index), so any subset of sequences can be
regenerated bit-identically.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

DATA_SEED = 20250618


# --------------------------------------------------------------------------- bf16 helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_f32(logits: np.ndarray) -> np.ndarray:
    return logits if logits.dtype == np.float32 else bf16_bits_to_f32(logits)


# --------------------------------------------------------------------------- workload container
@dataclass
class Workload:
    name: str
    B: int
    gamma: int
    V: int
    dtype: str                         # "f32" | "bf16" (bf16 arrays hold uint16 bit patterns)
    temperature: float
    taus: List[float]                  # entropy thresholds (nats) to run with
    seed: int                          # Philox seed of the verify call
    target: np.ndarray                 # [B, gamma+1, V]
    draft: np.ndarray                  # [B, gamma, V]
    tokens: np.ndarray                 # [B, gamma] int32
    row_temperature: Optional[np.ndarray] = None   # [B] float32, 0 => greedy row
    models: List[np.ndarray] = field(default_factory=list)  # hierarchical: drafter first, target last
    seq_ids: Optional[np.ndarray] = None           # global sequence indices when a subset was generated

    @property
    def logit_bytes(self) -> int:
        return self.target.nbytes + self.draft.nbytes


def _rng(cfg: int, b: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([DATA_SEED, cfg, int(b)]))


def _gumbel_argmax(rng: np.random.Generator, rows_f32: np.ndarray, T: float) -> np.ndarray:
    """Draw one token per row from softmax(rows/T) without computing it: argmax(rows/T + Gumbel)."""
    e = rng.standard_exponential(size=rows_f32.shape, dtype=np.float32)
    np.maximum(e, np.float32(1e-37), out=e)
    np.log(e, out=e)                       # Gumbel = -log(Exp(1))
    e *= np.float32(-1.0)
    e += rows_f32 / np.float32(T)
    return np.argmax(e, axis=-1).astype(np.int32)


def _store(dst: np.ndarray, b: int, rows_f32: np.ndarray, dtype: str) -> np.ndarray:
    """Write rows into dst[b] in the workload's dtype; return the stored values as float32."""
    if dtype == "bf16":
        bits = f32_to_bf16_bits(rows_f32)
        dst[b] = bits
        return bf16_bits_to_f32(bits)
    dst[b] = rows_f32
    return rows_f32


def _zipf_rows(rng: np.random.Generator, n_rows: int, V: int, sigma: float, slope: float,
               zipf_table: Optional[np.ndarray]) -> np.ndarray:
    x = rng.standard_normal(size=(n_rows, V), dtype=np.float32)
    x *= np.float32(sigma)
    if zipf_table is not None:
        for r in range(n_rows):
            x[r] += zipf_table[rng.permutation(V)]
    return x


def _zipf_table(V: int, slope: float) -> np.ndarray:
    return (-slope * np.log(np.arange(1, V + 1, dtype=np.float64))).astype(np.float32)


def _parallel(fn, items: Sequence[int]) -> None:
    workers = max(1, min(16, os.cpu_count() or 1, len(items)))
    if workers == 1:
        for it in items:
            fn(it)
        return
    with ThreadPoolExecutor(max_workers=workers) as ex:
        list(ex.map(fn, items))


# --------------------------------------------------------------------------- the generic recipe
def _make(cfg: int, name: str, B: int, gamma: int, V: int, dtype: str, temperature: float,
          tau_fracs: Sequence[float], seed: int, sigma: float, zipf_slope: Optional[float],
          draft_sigma: float, peak_prob: float = 0.0, peak_boost: float = 12.0,
          greedy_below: int = 0, seqs: Optional[Sequence[int]] = None) -> Workload:
    ids = np.arange(B, dtype=np.int64) if seqs is None else np.asarray(list(seqs), dtype=np.int64)
    n = len(ids)
    np_dt = np.uint16 if dtype == "bf16" else np.float32
    target = np.empty((n, gamma + 1, V), dtype=np_dt)
    draft = np.empty((n, gamma, V), dtype=np_dt)
    tokens = np.empty((n, gamma), dtype=np.int32)
    table = None if zipf_slope is None else _zipf_table(V, zipf_slope)
    rowT = None
    if greedy_below > 0:
        rowT = np.where(ids < greedy_below, 0.0, temperature).astype(np.float32)

    def one(k: int) -> None:
        b = int(ids[k])
        rng = _rng(cfg, b)
        P = _zipf_rows(rng, gamma + 1, V, sigma, zipf_slope or 0.0, table)
        if peak_prob > 0.0:
            hit = rng.random(gamma + 1) < peak_prob
            where = rng.integers(0, V, size=gamma + 1)
            for j in range(gamma + 1):
                if hit[j]:
                    P[j, where[j]] += np.float32(peak_boost)
        D = P[:gamma] + np.float32(draft_sigma) * rng.standard_normal(size=(gamma, V), dtype=np.float32)
        _store(target, k, P, dtype)
        Dq = _store(draft, k, D, dtype)
        if rowT is not None and rowT[k] == 0.0:
            tokens[k] = np.argmax(Dq, axis=-1).astype(np.int32)
        else:
            tokens[k] = _gumbel_argmax(rng, Dq, temperature)

    _parallel(one, list(range(n)))
    lnV = math.log(V)
    return Workload(name=name, B=n, gamma=gamma, V=V, dtype=dtype, temperature=temperature,
                    taus=[float(np.float32(f * lnV)) for f in tau_fracs], seed=seed,
                    target=target, draft=draft, tokens=tokens, row_temperature=rowT,
                    seq_ids=None if seqs is None else ids)


# --------------------------------------------------------------------------- the five named configurations
def config1(seqs=None) -> Workload:
    """B=1, gamma=4, V=32000, fp32, T=1: N(0,2^2) target, draft = target + N(0,0.5^2)."""
    return _make(1, "cfg1_B1_g4_V32000_f32", 1, 4, 32000, "f32", 1.0, [0.5], 0,
                 sigma=2.0, zipf_slope=None, draft_sigma=0.5, seqs=seqs)


def config2(seqs=None) -> Workload:
    """B=64, gamma=5, V=32000, bf16, T=1: N(0,2^2) + Zipf(1.1) target, draft = target + N(0,1)."""
    return _make(2, "cfg2_B64_g5_V32000_bf16", 64, 5, 32000, "bf16", 1.0, [0.5], 1,
                 sigma=2.0, zipf_slope=1.1, draft_sigma=1.0, seqs=seqs)


def config3(seqs=None, B: int = 256) -> Workload:
    """B=256, gamma=8, V=128256, bf16, T=0.8: Zipf(1.2), 30% peaked rows (+12), draft noise 0.75."""
    return _make(3, f"cfg3_B{B}_g8_V128256_bf16", B, 8, 128256, "bf16", 0.8, [0.25, 0.5, 0.75], 2,
                 sigma=2.0, zipf_slope=1.2, draft_sigma=0.75, peak_prob=0.3, seqs=seqs)


def config5(seqs=None, B: int = 1024) -> Workload:
    """B=1024, gamma=4, V=256000, fp32: first half greedy rows, second half T=0.7; N(0,3^2)+Zipf(1.0)."""
    return _make(5, f"cfg5_B{B}_g4_V256000_f32", B, 4, 256000, "f32", 0.7, [0.5], 4,
                 sigma=3.0, zipf_slope=1.0, draft_sigma=0.5, greedy_below=B // 2, seqs=seqs)


def config4(seqs=None, B: int = 128, V: int = 151936, gamma: int = 8) -> Workload:
    """Two-level hierarchy, bf16, T=1: base = N(0,2^2)+Zipf(1.1) of gamma+2 rows;
    small drafter = base[:gamma]+N(0,1), intermediate = base[:gamma+1]+N(0,0.4^2), target = base."""
    cfg, dtype, T = 4, "bf16", 1.0
    ids = np.arange(B, dtype=np.int64) if seqs is None else np.asarray(list(seqs), dtype=np.int64)
    n = len(ids)
    small = np.empty((n, gamma, V), dtype=np.uint16)
    mid = np.empty((n, gamma + 1, V), dtype=np.uint16)
    tgt = np.empty((n, gamma + 2, V), dtype=np.uint16)
    tokens = np.empty((n, gamma), dtype=np.int32)
    table = _zipf_table(V, 1.1)

    def one(k: int) -> None:
        rng = _rng(cfg, int(ids[k]))
        base = _zipf_rows(rng, gamma + 2, V, 2.0, 1.1, table)
        s = base[:gamma] + np.float32(1.0) * rng.standard_normal(size=(gamma, V), dtype=np.float32)
        m = base[:gamma + 1] + np.float32(0.4) * rng.standard_normal(size=(gamma + 1, V), dtype=np.float32)
        sq = _store(small, k, s, dtype)
        _store(mid, k, m, dtype)
        _store(tgt, k, base, dtype)
        tokens[k] = _gumbel_argmax(rng, sq, T)

    _parallel(one, list(range(n)))
    lnV = math.log(V)
    return Workload(name=f"cfg4_B{n}_g{gamma}_V{V}_bf16_2level", B=n, gamma=gamma, V=V, dtype=dtype,
                    temperature=T, taus=[float(np.float32(0.4 * lnV)), float(np.float32(0.6 * lnV))],
                    seed=3, target=tgt, draft=small, tokens=tokens, models=[small, mid, tgt],
                    seq_ids=None if seqs is None else ids)


def small_case(B: int, gamma: int, V: int, dtype: str = "f32", temperature: float = 1.0,
               tau_frac: float = 0.5, seed: int = 7, sigma: float = 2.0, zipf_slope: Optional[float] = 1.1,
               draft_sigma: float = 0.75, peak_prob: float = 0.2, greedy_below: int = 0,
               case_id: int = 100) -> Workload:
    """A free-form small workload with the same recipe, for ragged shapes and edge cases."""
    return _make(case_id, f"small_B{B}_g{gamma}_V{V}_{dtype}", B, gamma, V, dtype, temperature, [tau_frac],
                 seed, sigma=sigma, zipf_slope=zipf_slope, draft_sigma=draft_sigma, peak_prob=peak_prob,
                 greedy_below=greedy_below)


# --------------------------------------------------------------------------- token trees
@dataclass
class TreeWorkload:
    name: str
    B: int
    N: int                             # nodes per sequence
    V: int
    dtype: str
    temperature: float
    tau: float
    seed: int
    widths: List[int]                  # nodes per depth
    target: np.ndarray                 # [B, N+1, V] row c: context c (0 = the prefix, n+1 = after node n)
    draft: np.ndarray                  # [B, N, V]
    node_token: np.ndarray             # [B, N] int32
    node_parent: np.ndarray            # [B, N] int32, -1 = child of the prefix

    @property
    def logit_bytes(self) -> int:
        return self.target.nbytes + self.draft.nbytes


def tree_parents(widths: Sequence[int]) -> np.ndarray:
    """Breadth-first numbering: the i-th node of a depth hangs under node i mod (width of the depth above)."""
    par: List[int] = []
    first_prev, w_prev = -1, 1
    for d, w in enumerate(widths):
        first = len(par)
        for i in range(w):
            par.append(-1 if d == 0 else first_prev + (i % w_prev))
        first_prev, w_prev = first, w
    return np.asarray(par, dtype=np.int32)


def tree_case(B: int, widths: Sequence[int], V: int, dtype: str = "f32", temperature: float = 1.0,
              tau_frac: float = 0.5, seed: int = 9, sigma: float = 2.0, zipf_slope: Optional[float] = 1.1,
              draft_sigma: float = 0.75, peak_prob: float = 0.2, peak_boost: float = 12.0,
              case_id: int = 700, random_topology: bool = False) -> TreeWorkload:
    """Token trees with the recipe of the chains: every context has its own target row and a draft row that is
    the target row plus noise; the children of a context are independent draws from its draft row.
    random_topology: every sequence draws its own tree of sum(widths) nodes, node n under a uniformly chosen
    earlier node or the prefix."""
    par = tree_parents(widths)
    N = len(par)
    parents = np.tile(par, (B, 1))
    np_dt = np.uint16 if dtype == "bf16" else np.float32
    target = np.empty((B, N + 1, V), dtype=np_dt)
    draft = np.empty((B, N, V), dtype=np_dt)
    tokens = np.empty((B, N), dtype=np.int32)
    table = None if zipf_slope is None else _zipf_table(V, zipf_slope)

    def one(b: int) -> None:
        rng = _rng(case_id, b)
        P = _zipf_rows(rng, N + 1, V, sigma, zipf_slope or 0.0, table)
        if peak_prob > 0.0:
            hit = rng.random(N + 1) < peak_prob
            where = rng.integers(0, V, size=N + 1)
            for j in range(N + 1):
                if hit[j]:
                    P[j, where[j]] += np.float32(peak_boost)
        D = P[:N] + np.float32(draft_sigma) * rng.standard_normal(size=(N, V), dtype=np.float32)
        _store(target, b, P, dtype)
        Dq = _store(draft, b, D, dtype)
        if random_topology:
            parents[b] = [int(rng.integers(-1, n)) for n in range(N)]
        tokens[b] = _gumbel_argmax(rng, Dq[parents[b] + 1], temperature)

    _parallel(one, list(range(B)))
    return TreeWorkload(name=f"tree_B{B}_w{'-'.join(str(w) for w in widths)}_V{V}_{dtype}", B=B, N=N, V=V, dtype=dtype,
                        temperature=temperature, tau=float(np.float32(tau_frac * math.log(V))), seed=seed,
                        widths=list(widths), target=target, draft=draft, node_token=tokens,
                        node_parent=parents)
