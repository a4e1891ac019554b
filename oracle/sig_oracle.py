"""Python face of the fp64 CPU oracle.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module and
this module never imports the product package.

Contents
  * word-set construction written independently of the GPU library's builder
    (Section 3.1 prefix-closed sets; Appendix A canonical order; Definition 7.1
    weighted degree),
  * ctypes wrappers around sig_oracle.c (dense tensor-algebra route and
    per-word eq.-3 route, forward and reverse-mode backward),
  * the error measures used by the parity tests.

Parity pins: every function here is pinned by tests/test_oracle_pins.py against
closed forms, algebraic identities, brute-force iterated sums and fp64 finite
differences.  Nothing is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Iterable, List, Optional, Sequence, Tuple

import numpy as np

Word = Tuple[int, ...]
_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sig_oracle.c")
_LIB = os.path.join(_HERE, "libsig_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile sig_oracle.c with gcc (-O2, OpenMP).  Building the checker is not using it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c99", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, p = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.sig_oracle_threads.restype = ctypes.c_int
        lib.sig_oracle_set_threads.argtypes = [i32]
        lib.sig_oracle_dense_size.restype = ctypes.c_size_t
        lib.sig_oracle_dense_size.argtypes = [i32, i32]
        lib.sig_oracle_tensor_product.argtypes = [i32, i32, p, p, p]
        lib.sig_oracle_forward_dense.argtypes = [p, i64, i64, i32, i32, p]
        lib.sig_oracle_backward_dense.argtypes = [p, p, i64, i64, i32, i32, p]
        lib.sig_oracle_forward_words.argtypes = [p, i64, i64, i32, i64, p, p, p, p]
        lib.sig_oracle_backward_words.argtypes = [p, p, i64, i64, i32, i64, p, p, p, p]
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().sig_oracle_threads())


def set_threads(n: int) -> None:
    _load().sig_oracle_set_threads(int(n))


# ----------------------------------------------------------------------------------------------
# word sets (independent of the GPU library's C++ builder)
# ----------------------------------------------------------------------------------------------

def truncated_words(d: int, depth: int) -> List[Word]:
    """All non-empty words of length <= depth, level-major and lexicographic inside a
    level, i.e. ordered by the base-d encoding plus level offset (Appendix A)."""
    out: List[Word] = []
    level: List[Word] = [()]
    for _ in range(depth):
        level = [w + (i,) for w in level for i in range(d)]
        out.extend(level)
    return out


def anisotropic_words(d: int, weights: Sequence[float], cutoff: float) -> List[Word]:
    """Non-empty words with weighted degree <= cutoff (Definition 7.1).  The degree is the
    left-to-right fp64 sum of the letters' weights; a word is kept iff sum <= cutoff."""
    if len(weights) != d or any(not (g > 0.0) for g in weights):
        raise ValueError("weights must be d positive numbers")
    out: List[Word] = []
    level: List[Tuple[Word, float]] = [((), 0.0)]
    while level:
        nxt: List[Tuple[Word, float]] = []
        for w, deg in level:
            for i in range(d):
                s = deg + float(weights[i])
                if s <= cutoff:
                    nxt.append((w + (i,), s))
        out.extend(w for w, _ in nxt)
        level = nxt
    return sort_canonical(out)


def lyndon_words(d: int, depth: int) -> List[Word]:
    """Lyndon words of length 1..depth over {0..d-1}: words strictly smaller than every proper rotation of themselves
    (tested word by word), by length then lexicographic."""
    import itertools
    out: List[Word] = []
    for n in range(1, depth + 1):
        for w in itertools.product(range(d), repeat=n):
            if all(w < w[k:] + w[:k] for k in range(1, n)):
                out.append(w)
    return out


def logsig_word_set(d: int, depth: int) -> List[Word]:
    """Every word shorter than depth plus the Lyndon words of length depth, canonical order."""
    return sort_canonical(truncated_words(d, depth - 1) + [w for w in lyndon_words(d, depth) if len(w) == depth]) \
        if depth > 1 else [(i,) for i in range(d)]


def tensor_log(d: int, depth: int, S: np.ndarray) -> np.ndarray:
    """Tensor logarithm of a dense element 1 + x laid out [1 | level 1 | .. | level depth] (Section 3.3):
    log(1 + x) = sum_{k=1..depth} (-1)^{k+1} x^k / k with truncated tensor products; the result has level 0 = 0."""
    x = np.array(S, dtype=np.float64)
    x[0] = 0.0
    one_plus = np.zeros_like(x)
    out = np.zeros_like(x)
    power = np.zeros_like(x)
    power[0] = 1.0                                   # x^0
    for k in range(1, depth + 1):
        power = tensor_product(d, depth, power, x)   # x^k (its levels below k vanish)
        out += ((-1.0) ** (k + 1) / k) * power
    return out


def logsig_from_path(X: np.ndarray, depth: int) -> np.ndarray:
    """Log-signature in Lyndon-word coordinates: the coefficients of the Lyndon words in the tensor logarithm of the
    full truncated signature; [B, number of Lyndon words]."""
    B, _, d = X.shape
    words = truncated_words(d, depth)
    index = {w: k for k, w in enumerate(words)}
    cols = [index[w] for w in lyndon_words(d, depth)]
    S = forward_dense(X, depth)
    out = np.zeros((B, len(cols)))
    for b in range(B):
        L = tensor_log(d, depth, np.concatenate([[1.0], S[b]]))[1:]
        out[b] = L[cols]
    return out


def forward_windows(X: np.ndarray, W: Sequence[Word], windows: Sequence[Tuple[int, int]]) -> np.ndarray:
    """Signatures over windows (Section 5): window (l, r) is the path restricted to its points l..r.  One plain forward
    evaluation per window on the sliced path; [B, K, |W|]."""
    B = X.shape[0]
    out = np.zeros((B, len(windows), len(W)))
    for k, (l, r) in enumerate(windows):
        out[:, k, :] = forward_words(np.ascontiguousarray(X[:, l:r + 1]), W)
    return out


def backward_windows(X: np.ndarray, W: Sequence[Word], windows: Sequence[Tuple[int, int]], G: np.ndarray) -> np.ndarray:
    """Gradient of sum_{b,k,w} G[b,k,w] S_{t_l,t_r}(X_b, w) with respect to the points: the per-window gradients added
    into the points they came from."""
    out = np.zeros(X.shape, dtype=np.float64)
    for k, (l, r) in enumerate(windows):
        out[:, l:r + 1] += backward_words(np.ascontiguousarray(X[:, l:r + 1]), W, np.ascontiguousarray(G[:, k, :]))
    return out


def graph_words(d: int, edges: Iterable[Tuple[int, int]], depth: int) -> List[Word]:
    """Words of length <= depth in which every pair of consecutive letters is an edge of the given directed graph
    (Section 7.1); all single letters are words."""
    E = set((int(a), int(b)) for a, b in edges)
    out: List[Word] = [(i,) for i in range(d)]
    level = list(out)
    for _ in range(2, depth + 1):
        level = [w + (j,) for w in level for j in range(d) if (w[-1], j) in E]
        out.extend(level)
    return sort_canonical(out)


def leadlag_sparse_words(d: int, depth: int) -> List[Word]:
    """Sparse lead-lag word set of Section 8 over the alphabet (lag_0..lag_{d-1}, lead_0..lead_{d-1}) = (0..2d-1): every
    concatenation of the generators (lead_i), (lag_i, lead_i), (lead_i, lag_i) with at most `depth` letters, found here
    by testing every candidate word for such a factorisation (no enumeration by generators)."""
    gens = set()
    for i in range(d):
        gens.update({(d + i,), (i, d + i), (d + i, i)})

    def factorises(w: Word) -> bool:
        ok = [False] * (len(w) + 1)
        ok[0] = True
        for e in range(1, len(w) + 1):
            ok[e] = (ok[e - 1] and w[e - 1:e] in gens) or (e >= 2 and ok[e - 2] and w[e - 2:e] in gens)
        return ok[len(w)]

    out: List[Word] = []
    level: List[Word] = [()]
    for _ in range(depth):
        # a word can only factorise if each of its letters sits next to its partner or is a lead letter; grow by one
        # letter and keep every prefix of a factorising word as a candidate (prefixes of prefixes are candidates too)
        level = [w + (c,) for w in level for c in range(2 * d)
                 if _leadlag_prefix_possible(w + (c,), d)]
        out.extend(w for w in level if factorises(w))
    return sort_canonical(out)


def _leadlag_prefix_possible(w: Word, d: int) -> bool:
    """True if w is a prefix of some concatenation of generators: w minus a possibly dangling last letter factorises."""
    gens = set()
    for i in range(d):
        gens.update({(d + i,), (i, d + i), (d + i, i)})
    ok = [False] * (len(w) + 1)
    ok[0] = True
    for e in range(1, len(w) + 1):
        ok[e] = (ok[e - 1] and w[e - 1:e] in gens) or (e >= 2 and ok[e - 2] and w[e - 2:e] in gens)
    return ok[len(w)] or ok[len(w) - 1]


def leadlag_transform(X: np.ndarray) -> np.ndarray:
    """Lead-lag path of Section 8: X [B, n, d] -> [B, 2 n - 1, 2 d], rows (X_k, X_k) and (X_k, X_{k+1}) alternating;
    channels 0..d-1 are the lag copy, d..2d-1 the lead copy."""
    B, n, d = X.shape
    out = np.empty((B, 2 * n - 1, 2 * d), dtype=X.dtype)
    out[:, 0::2, :d] = X
    out[:, 0::2, d:] = X
    out[:, 1::2, :d] = X[:, :-1]
    out[:, 1::2, d:] = X[:, 1:]
    return out


def sort_canonical(words: Iterable[Word]) -> List[Word]:
    return sorted(set(tuple(int(c) for c in w) for w in words), key=lambda w: (len(w), w))


def prefix_closure(words: Iterable[Word]) -> List[Word]:
    """Smallest prefix-closed set containing the given words (Definition 3.3), canonical
    order, the empty word left out."""
    s = set()
    for w in words:
        w = tuple(int(c) for c in w)
        for k in range(1, len(w) + 1):
            s.add(w[:k])
    return sort_canonical(s)


def word_tables(closed: Sequence[Word], user: Optional[Sequence[Word]] = None) -> Dict[str, np.ndarray]:
    """parent / last-letter / level-start tables of a canonical prefix-closed set, and the
    canonical index of every user word."""
    index = {w: k for k, w in enumerate(closed)}
    n = len(closed)
    parent = np.full(n, -1, dtype=np.int32)
    letter = np.zeros(n, dtype=np.int32)
    max_len = max((len(w) for w in closed), default=0)
    level_start = np.zeros(max_len + 2, dtype=np.int32)
    for k, w in enumerate(closed):
        letter[k] = w[-1]
        if len(w) > 1:
            parent[k] = index[w[:-1]]
        level_start[len(w) + 1] += 1
    level_start = np.cumsum(level_start).astype(np.int32)
    tabs = {"parent": parent, "letter": letter, "level_start": level_start}
    if user is not None:
        tabs["user_index"] = np.array([index[tuple(int(c) for c in w)] for w in user], dtype=np.int64)
    return tabs


def _csr(closed: Sequence[Word]):
    index = {w: k for k, w in enumerate(closed)}
    offs = np.zeros(len(closed) + 1, dtype=np.int64)
    for k, w in enumerate(closed):
        offs[k + 1] = offs[k] + len(w)
    letters = np.zeros(max(int(offs[-1]), 1), dtype=np.int32)
    pidx = np.zeros(max(int(offs[-1]), 1), dtype=np.int64)
    for k, w in enumerate(closed):
        o = int(offs[k])
        for r, c in enumerate(w):
            letters[o + r] = c
            pidx[o + r] = index[w[: r + 1]]          # KeyError here means the set is not prefix-closed
    return letters, offs, pidx


# ----------------------------------------------------------------------------------------------
# forward / backward
# ----------------------------------------------------------------------------------------------

def _as_path(path) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(path), dtype=np.float32)
    if a.ndim != 3:
        raise ValueError("path must be [B, L+1, d]")
    return a


def dense_size(d: int, depth: int) -> int:
    return int(_load().sig_oracle_dense_size(d, depth))


def tensor_product(d: int, depth: int, A: np.ndarray, Bt: np.ndarray) -> np.ndarray:
    """Truncated tensor product of two dense elements laid out [1 | level 1 | ... | level depth]."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    Bt = np.ascontiguousarray(Bt, dtype=np.float64)
    C = np.zeros_like(A)
    _load().sig_oracle_tensor_product(d, depth, A.ctypes.data, Bt.ctypes.data, C.ctypes.data)
    return C


def forward_dense(path, depth: int, keep_level0: bool = False) -> np.ndarray:
    """Truncated signature, fp64 [B, sum_{n=1..depth} d^n] in canonical order."""
    X = _as_path(path)
    B, P, d = X.shape
    tot = dense_size(d, depth)
    out = np.zeros((B, tot), dtype=np.float64)
    rc = _load().sig_oracle_forward_dense(X.ctypes.data, B, P, d, depth, out.ctypes.data)
    if rc:
        raise RuntimeError(f"oracle forward_dense failed ({rc})")
    return out if keep_level0 else out[:, 1:]


def backward_dense(path, depth: int, grad_coeffs) -> np.ndarray:
    """d(sum grad*S)/d path for the truncated signature, fp64 [B, L+1, d]."""
    X = _as_path(path)
    B, P, d = X.shape
    tot = dense_size(d, depth)
    g = np.zeros((B, tot), dtype=np.float64)
    g[:, 1:] = np.asarray(grad_coeffs, dtype=np.float64)
    gp = np.zeros((B, P, d), dtype=np.float64)
    rc = _load().sig_oracle_backward_dense(X.ctypes.data, g.ctypes.data, B, P, d, depth, gp.ctypes.data)
    if rc:
        raise RuntimeError(f"oracle backward_dense failed ({rc})")
    return gp


def forward_words(path, closed: Sequence[Word]) -> np.ndarray:
    """Coefficients of a canonical prefix-closed word set via eq. 3, fp64 [B, |W|]."""
    X = _as_path(path)
    B, P, d = X.shape
    letters, offs, pidx = _csr(closed)
    out = np.zeros((B, len(closed)), dtype=np.float64)
    rc = _load().sig_oracle_forward_words(X.ctypes.data, B, P, d, len(closed), letters.ctypes.data,
                                          offs.ctypes.data, pidx.ctypes.data, out.ctypes.data)
    if rc:
        raise RuntimeError(f"oracle forward_words failed ({rc})")
    return out


def backward_words(path, closed: Sequence[Word], grad_coeffs) -> np.ndarray:
    X = _as_path(path)
    B, P, d = X.shape
    letters, offs, pidx = _csr(closed)
    g = np.ascontiguousarray(np.asarray(grad_coeffs, dtype=np.float64))
    assert g.shape == (B, len(closed))
    gp = np.zeros((B, P, d), dtype=np.float64)
    rc = _load().sig_oracle_backward_words(X.ctypes.data, g.ctypes.data, B, P, d, len(closed), letters.ctypes.data,
                                           offs.ctypes.data, pidx.ctypes.data, gp.ctypes.data)
    if rc:
        raise RuntimeError(f"oracle backward_words failed ({rc})")
    return gp


def gather_from_dense(dense: np.ndarray, d: int, words: Sequence[Word]) -> np.ndarray:
    """Pick the coefficients of `words` out of a dense truncated result (level 0 dropped):
    index = level offset + base-d encoding (Appendix A)."""
    idx = np.empty(len(words), dtype=np.int64)
    for k, w in enumerate(words):
        n = len(w)
        off = sum(d ** m for m in range(1, n))
        phi = 0
        for c in w:
            phi = phi * d + c
        idx[k] = off + phi
    return dense[:, idx]


# ----------------------------------------------------------------------------------------------
# error measures used by the parity tests
# ----------------------------------------------------------------------------------------------

def level_errors(test: np.ndarray, ref: np.ndarray, lengths: np.ndarray) -> Dict[int, float]:
    """For every word length n: max over paths of  max_{|w|=n} |test-ref| / ||ref restricted to
    length n||_2  (per path).  A level whose reference is identically zero must match exactly."""
    out: Dict[int, float] = {}
    test = np.asarray(test, dtype=np.float64)
    for n in sorted(set(int(x) for x in lengths)):
        m = lengths == n
        num = np.abs(test[:, m] - ref[:, m]).max(axis=1)
        den = np.sqrt((ref[:, m] ** 2).sum(axis=1))
        with np.errstate(divide="ignore", invalid="ignore"):
            r = np.where(den > 0, num / den, np.where(num == 0, 0.0, np.inf))
        out[n] = float(r.max()) if r.size else 0.0
    return out


def grad_errors(test: np.ndarray, ref: np.ndarray) -> np.ndarray:
    """Per path  ||test-ref||_inf / ||ref||_inf."""
    test = np.asarray(test, dtype=np.float64)
    B = ref.shape[0]
    num = np.abs(test - ref).reshape(B, -1).max(axis=1)
    den = np.abs(ref).reshape(B, -1).max(axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        return np.where(den > 0, num / den, np.where(num == 0, 0.0, np.inf))
