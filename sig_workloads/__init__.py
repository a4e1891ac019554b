"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module holds no signature arithmetic: it only draws random paths, random
upstream gradients and random word lists.  Both sides consume exactly the fp32
arrays produced here.

The paper benchmarks on unspecified random paths of shape (B, M, d) (Section
"Benchmarks"); the five workloads below take its shapes (d 2..16, depth 4..6,
signature sizes 30..70k) and fix a distribution for each.

Recipe (all draws in fp64 from numpy.random.default_rng(seed), increments are
cumulatively summed from X_0 = 0 and the points cast to fp32 once):

  c1   B=32  L=64   d=2  depth 4            dX ~ N(0, 1/L) i.i.d.
  c2   B=256 L=256  d=4  depth 6            channels 1..3 N(0, 1/L); channel 0 is time, every increment 1/L
  c3   B=128 L=1024 d=8  depth 5            sigma_c = 10**U(-1,1) per channel; dX^(c) ~ N(0, sigma_c^2/L)
  c4a  B=512 L=512  d=6  weights (1,1,2,2,3,3), cutoff 8     dX ~ N(0, 1/L)
  c4b  B=512 L=512  d=10 random prefix-closed set, 10000 words, max length 6   dX ~ N(0, 1/L)
  c5   B=64  L=4096 d=16 depth 4            per channel AR(1), phi=0.5, unit variance, dX = e_t/sqrt(L)

grad_coeffs ~ N(0,1) fp32 from default_rng(1000 + seed).
"""
from __future__ import annotations

import random
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

Word = Tuple[int, ...]


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    B: int
    L: int
    d: int
    kind: str                      # "truncated" | "anisotropic" | "words"
    depth: Optional[int] = None    # truncated
    weights: Optional[Tuple[float, ...]] = None   # anisotropic
    cutoff: Optional[float] = None                # anisotropic
    n_words: Optional[int] = None  # words
    max_len: Optional[int] = None  # words
    dist: str = "iid"              # "iid" | "time0" | "scaled" | "ar1"
    note: str = ""


WORKLOADS = {
    "c1": Workload("c1", 0, 32, 64, 2, "truncated", depth=4, dist="iid"),
    "c2": Workload("c2", 1, 256, 256, 4, "truncated", depth=6, dist="time0"),
    "c3": Workload("c3", 2, 128, 1024, 8, "truncated", depth=5, dist="scaled"),
    "c4a": Workload("c4a", 3, 512, 512, 6, "anisotropic",
                    weights=(1.0, 1.0, 2.0, 2.0, 3.0, 3.0), cutoff=8.0, dist="iid"),
    "c4b": Workload("c4b", 3, 512, 512, 10, "words", n_words=10000, max_len=6, dist="iid"),
    "c5": Workload("c5", 4, 64, 4096, 16, "truncated", depth=4, dist="ar1"),
}


def make_increments(dist: str, seed: int, B: int, L: int, d: int) -> np.ndarray:
    """fp64 increments [B, L, d] for one of the four distributions."""
    rng = np.random.default_rng(seed)
    if L == 0:
        return np.zeros((B, 0, d))
    if dist == "iid":
        return rng.standard_normal((B, L, d)) / np.sqrt(L)
    if dist == "time0":
        dx = rng.standard_normal((B, L, d)) / np.sqrt(L)
        dx[:, :, 0] = 1.0 / L
        return dx
    if dist == "scaled":
        sigma = 10.0 ** rng.uniform(-1.0, 1.0, size=d)
        return rng.standard_normal((B, L, d)) * (sigma / np.sqrt(L))
    if dist == "ar1":
        phi = 0.5
        e = np.empty((B, L, d))
        prev = rng.standard_normal((B, d))
        xi = rng.standard_normal((B, L, d))
        s = np.sqrt(1.0 - phi * phi)
        for t in range(L):
            prev = phi * prev + s * xi[:, t, :]
            e[:, t, :] = prev
        return e / np.sqrt(L)
    raise ValueError(f"unknown distribution {dist!r}")


def make_path(dist: str, seed: int, B: int, L: int, d: int) -> np.ndarray:
    """fp32 points [B, L+1, d] starting at 0."""
    dx = make_increments(dist, seed, B, L, d)
    pts = np.zeros((B, L + 1, d))
    if L:
        np.cumsum(dx, axis=1, out=pts[:, 1:, :])
    return np.ascontiguousarray(pts.astype(np.float32))


def make_grad_coeffs(seed: int, B: int, n_coeffs: int) -> np.ndarray:
    """fp32 upstream gradient [B, n_coeffs] ~ N(0,1)."""
    rng = np.random.default_rng(1000 + seed)
    return np.ascontiguousarray(rng.standard_normal((B, n_coeffs)).astype(np.float32))


def random_prefix_closed_words(seed: int, d: int, n_words: int, max_len: int) -> List[Word]:
    """Grow a prefix-closed set: pick a uniformly random existing word (the empty
    word included), skip it if it already has max_len letters, append a uniform
    letter, skip duplicates; stop at n_words non-empty words.  Returned in growth
    order (so it is NOT sorted)."""
    rnd = random.Random(seed)
    pool: List[Word] = [()]
    seen = {()}
    out: List[Word] = []
    cap = sum(d ** k for k in range(1, max_len + 1))
    if n_words > cap:
        raise ValueError("more words requested than exist")
    while len(out) < n_words:
        base = pool[rnd.randrange(len(pool))]
        if len(base) >= max_len:
            continue
        w = base + (rnd.randrange(d),)
        if w in seen:
            continue
        seen.add(w)
        pool.append(w)
        out.append(w)
    return out


def words_to_csr(words: Sequence[Word]) -> Tuple[np.ndarray, np.ndarray]:
    """Flatten a word list to (letters int32, offsets int64[n+1])."""
    offsets = np.zeros(len(words) + 1, dtype=np.int64)
    for k, w in enumerate(words):
        offsets[k + 1] = offsets[k] + len(w)
    letters = np.fromiter((c for w in words for c in w), dtype=np.int32, count=int(offsets[-1]))
    return letters, offsets


def workload_path(wl: Workload, B: Optional[int] = None, L: Optional[int] = None) -> np.ndarray:
    return make_path(wl.dist, wl.seed, wl.B if B is None else B, wl.L if L is None else L, wl.d)


def workload_word_list(wl: Workload) -> Optional[List[Word]]:
    """The user word list of a 'words' workload (growth order); None otherwise."""
    if wl.kind != "words":
        return None
    return random_prefix_closed_words(wl.seed, wl.d, wl.n_words, wl.max_len)
