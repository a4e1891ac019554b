"""Pins for the fp64 CPU oracle: every check here is against something the paper or the
mathematics fixes, computed in this file without calling the oracle for the expected value.

A plausible mistake in the oracle (dropped term, wrong factorial, transposed tensor product,
wrong sign in the chain rule, off-by-one in the level layout) fails at least one of them.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import sig_oracle as O
from sig_workloads import make_path, random_prefix_closed_words

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def word_index(d, w):
    off = sum(d ** m for m in range(1, len(w)))
    phi = 0
    for c in w:
        phi = phi * d + c
    return off + phi


def levels_of(flat, d, N):
    """Split [sum d^n] into list of arrays shaped (d,)*n, n=1..N."""
    out, o = [], 0
    for n in range(1, N + 1):
        out.append(flat[o:o + d ** n].reshape((d,) * n))
        o += d ** n
    return out


def np_tensor_product(A, Bl, d, N):
    """Independent truncated tensor product with numpy outer products.  A, Bl: lists
    [level0 scalar, level1, ..., levelN] of ndarrays shaped (d,)*n."""
    C = []
    for n in range(N + 1):
        acc = np.zeros((d,) * n)
        for k in range(n + 1):
            acc = acc + np.multiply.outer(A[k], Bl[n - k])
        C.append(acc)
    return C


def with_level0(flat, d, N):
    return [np.array(1.0)] + levels_of(flat, d, N)


# ---------------------------------------------------------------------------------------------
# sizes and ordering
# ---------------------------------------------------------------------------------------------

def test_sizes_match_paper_tables():
    rows = []
    with open(os.path.join(GOLDEN, "paper_signature_sizes.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            d, N, printed, unit = (int(x) for x in line.split())
            rows.append((d, N, printed, unit))
    assert len(rows) >= 12
    for d, N, printed, unit in rows:
        n = len(O.truncated_words(d, N)) if d ** N < 400000 else None
        exact = sum(d ** k for k in range(1, N + 1))
        if n is not None:
            assert n == exact
        assert O.dense_size(d, N) == exact + 1
        if unit == 1:
            assert exact == printed
        else:
            assert abs(exact - printed) <= unit / 2 + 1e-9, (d, N, exact, printed)


def test_truncated_order_is_base_d_encoding():
    d, N = 3, 4
    W = O.truncated_words(d, N)
    for k, w in enumerate(W):
        assert word_index(d, w) == k
    tabs = O.word_tables(W)
    # Appendix A: prefix = floor(phi/d), last letter = phi mod d
    lev_off = [0]
    for n in range(1, N + 1):
        lev_off.append(lev_off[-1] + d ** n)
    for k, w in enumerate(W):
        n = len(w)
        phi = k - lev_off[n - 1]
        assert tabs["letter"][k] == phi % d
        if n == 1:
            assert tabs["parent"][k] == -1
        else:
            assert tabs["parent"][k] == lev_off[n - 2] + phi // d
    assert list(tabs["level_start"]) == [0] + lev_off


def test_level_start_layout():
    W = O.truncated_words(2, 3)
    t = O.word_tables(W)
    # level_start[n] = index of the first word of length n (n = 1..max_len), level_start[max_len+1] = |W|
    assert list(t["level_start"]) == [0, 0, 2, 6, 14]


def test_anisotropic_bruteforce_and_special_case():
    d, gam, r = 3, (1.0, 2.0, 1.5), 4.0
    W = O.anisotropic_words(d, gam, r)
    maxlen = int(r / min(gam))
    brute = []
    for n in range(1, maxlen + 1):
        for w in itertools.product(range(d), repeat=n):
            if sum(gam[c] for c in w) <= r:
                brute.append(w)
    assert W == sorted(brute, key=lambda w: (len(w), w))
    # every prefix present
    s = set(W)
    assert all(w[:k] in s for w in W for k in range(1, len(w)))
    # gamma = 1, r = N is plain truncation
    assert O.anisotropic_words(3, (1.0, 1.0, 1.0), 4.0) == O.truncated_words(3, 4)


def test_anisotropic_c4a_count_from_recurrence():
    # words of weighted degree exactly r for weights (1,1,2,2,3,3): c(r) = 2c(r-1)+2c(r-2)+2c(r-3)
    c = {0: 1}
    for r in range(1, 9):
        c[r] = 2 * c.get(r - 1, 0) + 2 * c.get(r - 2, 0) + 2 * c.get(r - 3, 0)
    total = sum(c[r] for r in range(1, 9))
    assert total == 5754
    W = O.anisotropic_words(6, (1, 1, 2, 2, 3, 3), 8)
    assert len(W) == total
    assert max(len(w) for w in W) == 8


def test_prefix_closure_and_user_index():
    user = [(2, 0, 1), (1,), (2, 0), (0, 0, 0, 1), (2, 0, 1)]
    C = O.prefix_closure(user)
    assert C == [(0,), (1,), (2,), (0, 0), (2, 0), (0, 0, 0), (2, 0, 1), (0, 0, 0, 1)]
    t = O.word_tables(C, user)
    assert list(t["user_index"]) == [6, 1, 4, 7, 6]
    # parent/letter round trip
    for k, w in enumerate(C):
        rec, q = [], k
        while q != -1:
            rec.append(int(t["letter"][q]))
            q = int(t["parent"][q])
        assert tuple(reversed(rec)) == w


# ---------------------------------------------------------------------------------------------
# forward
# ---------------------------------------------------------------------------------------------

def test_single_segment_closed_form():
    # Proposition 3.1: level n of the signature of one linear piece is dX^{(x)n}/n!
    rng = np.random.default_rng(5)
    d, N = 4, 5
    X = np.zeros((3, 2, d), dtype=np.float32)
    X[:, 0] = rng.standard_normal((3, d)).astype(np.float32)
    X[:, 1] = rng.standard_normal((3, d)).astype(np.float32)
    S = O.forward_dense(X, N)
    for b in range(3):
        dx = X[b, 1].astype(np.float64) - X[b, 0].astype(np.float64)
        lv = levels_of(S[b], d, N)
        t = np.array(1.0)
        for n in range(1, N + 1):
            t = np.multiply.outer(t, dx)
            np.testing.assert_allclose(lv[n - 1], t / math.factorial(n), rtol=1e-13, atol=1e-300)


def test_one_point_path_is_identity():
    X = np.ones((2, 1, 3), dtype=np.float32)
    assert np.all(O.forward_dense(X, 3) == 0.0)
    assert O.forward_dense(X, 3, keep_level0=True)[0, 0] == 1.0
    assert np.all(O.forward_words(X, O.truncated_words(3, 3)) == 0.0)


def brute_iterated_sum(dx, w):
    """S(w) = sum over j_1 <= ... <= j_n of prod dX_{j_r}^{(w_r)} / prod_j (multiplicity of j)!"""
    L = dx.shape[0]
    n = len(w)
    tot = 0.0
    for js in itertools.combinations_with_replacement(range(L), n):
        p = 1.0
        for r, j in enumerate(js):
            p *= dx[j, w[r]]
        den = 1
        for j in set(js):
            den *= math.factorial(js.count(j))
        tot += p / den
    return tot


@pytest.mark.parametrize("L", [2, 3])
def test_bruteforce_iterated_sums(L):
    d, N = 3, 4
    X = make_path("iid", 11 + L, 2, L, d)
    S = O.forward_dense(X, N)
    W = O.truncated_words(d, N)
    Sw = O.forward_words(X, W)
    for b in range(2):
        dx = np.diff(X[b].astype(np.float64), axis=0)
        for k, w in enumerate(W):
            ref = brute_iterated_sum(dx, w)
            assert abs(S[b, k] - ref) <= 1e-13 * max(1.0, abs(ref))
            assert abs(Sw[b, k] - ref) <= 1e-13 * max(1.0, abs(ref))


def test_chen_under_concatenation():
    d, N = 3, 4
    X = make_path("iid", 21, 2, 12, d)
    cut = 5
    S_all = O.forward_dense(X, N)
    S_a = O.forward_dense(X[:, :cut + 1], N)
    S_b = O.forward_dense(X[:, cut:], N)
    for b in range(2):
        C = np_tensor_product(with_level0(S_a[b], d, N), with_level0(S_b[b], d, N), d, N)
        flat = np.concatenate([c.ravel() for c in C[1:]])
        np.testing.assert_allclose(flat, S_all[b], rtol=1e-12, atol=1e-15)
        # the oracle's own product is the same operation
        A = np.concatenate([[1.0], S_a[b]])
        Bt = np.concatenate([[1.0], S_b[b]])
        np.testing.assert_allclose(O.tensor_product(d, N, A, Bt)[1:], flat, rtol=1e-13, atol=1e-16)
        # and it is not commutative: swapping the factors must NOT give the same thing
        assert np.abs(O.tensor_product(d, N, Bt, A)[1:] - flat).max() > 1e-6


def test_time_reversal_is_inverse():
    d, N = 2, 5
    X = make_path("iid", 31, 1, 9, d)
    S = O.forward_dense(X, N)[0]
    R = O.forward_dense(X[:, ::-1].copy(), N)[0]
    C = np_tensor_product(with_level0(S, d, N), with_level0(R, d, N), d, N)
    assert abs(C[0] - 1.0) < 1e-15
    for n in range(1, N + 1):
        assert np.abs(C[n]).max() < 1e-13


def shuffle(u, v):
    if not u:
        return [v]
    if not v:
        return [u]
    return [(u[0],) + w for w in shuffle(u[1:], v)] + [(v[0],) + w for w in shuffle(u, v[1:])]


def test_shuffle_identities():
    d, N = 3, 5
    X = make_path("scaled", 41, 2, 7, d)
    S = O.forward_dense(X, N)
    val = lambda b, w: S[b, word_index(d, w)]
    for b in range(2):
        for i in range(d):
            for j in range(d):
                assert abs(val(b, (i,)) * val(b, (j,)) - val(b, (i, j)) - val(b, (j, i))) < 1e-12
        for u, v in [((0, 1), (2,)), ((2, 1), (0, 0)), ((1,), (0, 2, 1)), ((0, 1, 2), (2, 1)), ((1, 1), (1, 2, 0))]:
            lhs = val(b, u) * val(b, v)
            rhs = sum(val(b, w) for w in shuffle(u, v))
            assert abs(lhs - rhs) < 1e-11 * max(1.0, abs(lhs))


def test_level1_and_symmetrised_levels():
    d, N = 3, 4
    X = make_path("iid", 51, 2, 10, d)
    S = O.forward_dense(X, N)
    for b in range(2):
        tot = X[b, -1].astype(np.float64) - X[b, 0].astype(np.float64)
        lv = levels_of(S[b], d, N)
        np.testing.assert_allclose(lv[0], tot, rtol=1e-13, atol=1e-15)
        t = np.array(1.0)
        for n in range(1, N + 1):
            t = np.multiply.outer(t, tot)
            sym = np.zeros_like(lv[n - 1])
            for perm in itertools.permutations(range(n)):
                sym += np.transpose(lv[n - 1], perm)
            # sum over all permutations of level n equals (X_L - X_0)^{(x)n}
            np.testing.assert_allclose(sym, t, rtol=1e-11, atol=1e-13)


def test_levy_area():
    # antisymmetric part of level 2 = signed area: 1/2 sum_j (X_{j-1}-X_0) x dX_j
    d = 2
    X = make_path("iid", 61, 3, 17, d)
    S = O.forward_dense(X, 2)
    for b in range(3):
        P = X[b].astype(np.float64)
        dx = np.diff(P, axis=0)
        rel = P[:-1] - P[0]
        area = 0.5 * np.sum(rel[:, 0] * dx[:, 1] - rel[:, 1] * dx[:, 0])
        lv2 = S[b, d:].reshape(d, d)
        assert abs(0.5 * (lv2[0, 1] - lv2[1, 0]) - area) < 1e-13


def test_reparametrisation_invariance():
    d, N = 3, 4
    X = make_path("iid", 71, 1, 6, d)[0].astype(np.float64)
    # work on values that survive the fp32 cast exactly: multiples of 2^-10
    X = np.round(X * 1024) / 1024
    base = O.forward_dense(X[None].astype(np.float32), N)[0]
    # (a) repeated point: a zero-length segment multiplies by exp(0) = 1
    rep = np.insert(X, 3, X[3], axis=0)
    np.testing.assert_allclose(O.forward_dense(rep[None].astype(np.float32), N)[0], base, rtol=0, atol=0)
    # (b) collinear midpoint (exactly representable)
    mid = np.insert(X, 3, 0.5 * (X[2] + X[3]), axis=0)
    np.testing.assert_allclose(O.forward_dense(mid[None].astype(np.float32), N)[0], base, rtol=1e-12, atol=1e-15)
    W = O.truncated_words(d, N)
    np.testing.assert_allclose(O.forward_words(mid[None].astype(np.float32), W)[0], base, rtol=1e-12, atol=1e-15)


def test_translation_invariance():
    d, N = 2, 4
    X = make_path("iid", 72, 1, 8, d)
    X = (np.round(X * 256) / 256).astype(np.float32)
    a = O.forward_dense(X, N)
    b = O.forward_dense((X + np.float32(3.0)).astype(np.float32), N)
    np.testing.assert_allclose(a, b, rtol=0, atol=0)


def test_dense_and_word_routes_agree_on_projection():
    d = 4
    words = random_prefix_closed_words(3, d, 300, 5)
    C = O.prefix_closure(words)
    assert len(C) == 300
    X = make_path("iid", 81, 3, 20, d)
    dense = O.forward_dense(X, 5)
    proj = O.gather_from_dense(dense, d, C)
    np.testing.assert_allclose(O.forward_words(X, C), proj, rtol=1e-11, atol=1e-14)


def test_planted_mistakes_are_caught_by_the_pins():
    """Mutated copies of the step (in this file, in numpy) must violate the closed form / Chen,
    so the pins above do discriminate."""
    d, N = 2, 3
    dx = np.array([0.3, -0.7])
    good = [np.array(1.0)]
    for n in range(1, N + 1):
        good.append(np.multiply.outer(good[-1], dx) / n)
    wrong_fact = [np.array(1.0)]
    for n in range(1, N + 1):
        wrong_fact.append(np.multiply.outer(wrong_fact[-1], dx) / (n + 1))
    assert np.abs(good[2] - wrong_fact[2]).max() > 1e-3
    A = [np.array(1.0), np.array([1.0, 2.0]), np.ones((2, 2)), np.ones((2, 2, 2))]
    AB = np_tensor_product(A, good, d, N)
    BA = np_tensor_product(good, A, d, N)
    assert np.abs(AB[2] - BA[2]).max() > 1e-3


# ---------------------------------------------------------------------------------------------
# backward
# ---------------------------------------------------------------------------------------------

def fd_grad(fun, X, h=1e-5):
    """Central differences of a scalar function of an fp64 array; fun casts nothing."""
    g = np.zeros_like(X)
    it = np.nditer(X, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        Xp = X.copy(); Xp[idx] += h
        Xm = X.copy(); Xm[idx] -= h
        g[idx] = (fun(Xp) - fun(Xm)) / (2 * h)
    return g


def _grid_path(seed, B, L, d):
    """Path whose coordinates are multiples of 2^-7 so that +-h steps of 2^-12 are exact in fp32."""
    X = make_path("iid", seed, B, L, d).astype(np.float64)
    return np.round(X * 128) / 128


def test_backward_dense_matches_finite_differences():
    d, N, B, L = 2, 4, 2, 5
    X = _grid_path(91, B, L, d)
    G = np.random.default_rng(1).standard_normal((B, sum(d ** n for n in range(1, N + 1))))
    ana = O.backward_dense(X.astype(np.float32), N, G)
    h = 2.0 ** -12
    fun = lambda Y: float((O.forward_dense(Y.astype(np.float32), N) * G).sum())
    num = fd_grad(fun, X, h)
    np.testing.assert_allclose(ana, num, rtol=2e-6, atol=2e-6)


def test_backward_words_matches_finite_differences_and_dense():
    d, B, L = 3, 2, 4
    words = random_prefix_closed_words(7, d, 40, 4)
    C = O.prefix_closure(words)
    X = _grid_path(92, B, L, d)
    G = np.random.default_rng(2).standard_normal((B, len(C)))
    ana = O.backward_words(X.astype(np.float32), C, G)
    h = 2.0 ** -12
    fun = lambda Y: float((O.forward_words(Y.astype(np.float32), C) * G).sum())
    num = fd_grad(fun, X, h)
    np.testing.assert_allclose(ana, num, rtol=2e-6, atol=2e-6)
    # the same gradient through the dense route: scatter G into the dense layout
    N = 4
    Gd = np.zeros((B, sum(d ** n for n in range(1, N + 1))))
    for k, w in enumerate(C):
        Gd[:, word_index(d, w)] = G[:, k]
    np.testing.assert_allclose(O.backward_dense(X.astype(np.float32), N, Gd), ana, rtol=1e-10, atol=1e-12)


def _fd_coordinates_and_directions(fun, ana, X, n_coord, n_dir, seed, h=2.0 ** -12):
    """Central differences of `fun` at `n_coord` random coordinates and along `n_dir` random directions of X against
    the analytic gradient `ana`; X lies on a grid on which the +-h steps are exact in fp32."""
    rng = np.random.default_rng(seed)
    flat = rng.choice(X.size, size=n_coord, replace=False)
    scale = np.abs(ana).max()
    for f in flat:
        idx = np.unravel_index(f, X.shape)
        Xp = X.copy(); Xp[idx] += h
        Xm = X.copy(); Xm[idx] -= h
        num = (fun(Xp) - fun(Xm)) / (2 * h)
        assert abs(num - ana[idx]) <= 2e-6 * max(scale, abs(num)), (idx, num, ana[idx])
    for _ in range(n_dir):
        V = rng.integers(-1, 2, size=X.shape).astype(np.float64)     # +-h V stays on the grid
        num = (fun(X + h * V) - fun(X - h * V)) / (2 * h)
        dot = float((ana * V).sum())
        assert abs(num - dot) <= 2e-6 * max(scale * np.sqrt(V.size), abs(num)), (num, dot)


def test_backward_finite_differences_on_c2_shaped_case():
    """The c2 word set (d = 4, depth 6, 5,460 words, time channel) on a small batch: 64 random coordinates and 8 random
    directions of the path against central differences of the dense forward oracle (Proposition 4.1)."""
    d, N, B, L = 4, 6, 2, 24
    X = np.round(make_path("time0", 96, B, L, d).astype(np.float64) * 128) / 128
    G = np.random.default_rng(6).standard_normal((B, sum(d ** n for n in range(1, N + 1))))
    ana = O.backward_dense(X.astype(np.float32), N, G)
    fun = lambda Y: float((O.forward_dense(Y.astype(np.float32), N) * G).sum())
    _fd_coordinates_and_directions(fun, ana, X, 64, 8, seed=7)


@pytest.mark.parametrize("d,N,L,dist,seed", [(8, 5, 10, "scaled", 10), (16, 4, 8, "ar1", 12)])
def test_backward_finite_differences_on_c3_and_c5_shaped_cases(d, N, L, dist, seed):
    """The c3 and c5 word sets (d = 8, depth 5: 37,448 words; d = 16, depth 4: 69,904 words) with their input
    distributions on a small batch: 64 random coordinates and 8 random directions against central differences."""
    B = 2
    X = np.round(make_path(dist, 90 + seed, B, L, d).astype(np.float64) * 128) / 128
    G = np.random.default_rng(seed).standard_normal((B, sum(d ** n for n in range(1, N + 1))))
    ana = O.backward_dense(X.astype(np.float32), N, G)
    fun = lambda Y: float((O.forward_dense(Y.astype(np.float32), N) * G).sum())
    _fd_coordinates_and_directions(fun, ana, X, 64, 8, seed=seed + 1)


def test_backward_finite_differences_on_c4a_shaped_case():
    """The c4a word set (d = 6, weights (1,1,2,2,3,3), degree <= 8: 5,754 words up to length 8) on a small batch, per-word
    route: 64 random coordinates and 8 random directions against central differences of the per-word forward oracle."""
    d, B, L = 6, 2, 12
    C = O.anisotropic_words(d, (1.0, 1.0, 2.0, 2.0, 3.0, 3.0), 8.0)
    assert len(C) == 5754
    X = _grid_path(97, B, L, d)
    G = np.random.default_rng(8).standard_normal((B, len(C)))
    ana = O.backward_words(X.astype(np.float32), C, G)
    fun = lambda Y: float((O.forward_words(Y.astype(np.float32), C) * G).sum())
    _fd_coordinates_and_directions(fun, ana, X, 64, 8, seed=9)


def test_backward_level1_closed_form():
    # L = sum_i c_i S(i) = c . (X_L - X_0): gradient is -c at the first point, +c at the last, 0 between
    d, N, L = 3, 3, 6
    X = make_path("iid", 93, 1, L, d)
    G = np.zeros((1, sum(d ** n for n in range(1, N + 1))))
    c = np.array([0.5, -2.0, 3.0])
    G[0, :d] = c
    g = O.backward_dense(X, N, G)[0]
    np.testing.assert_allclose(g[0], -c, atol=1e-14)
    np.testing.assert_allclose(g[-1], c, atol=1e-14)
    assert np.abs(g[1:-1]).max() < 1e-14


def test_backward_single_segment_closed_form():
    # one segment: S(w) = prod dX^{(w_r)}/n!  =>  dS(w)/d dX^{(i)} = (#i in w) * prod / dX^{(i)} / n!
    d, N = 3, 4
    X = np.zeros((1, 2, d), dtype=np.float32)
    X[0, 0] = [0.25, -0.5, 1.0]
    X[0, 1] = [1.0, 0.25, -0.75]
    dx = X[0, 1].astype(np.float64) - X[0, 0].astype(np.float64)
    W = O.truncated_words(d, N)
    G = np.random.default_rng(3).standard_normal((1, len(W)))
    expect = np.zeros(d)
    for k, w in enumerate(W):
        for r in range(len(w)):
            rest = 1.0
            for q in range(len(w)):
                if q != r:
                    rest *= dx[w[q]]
            expect[w[r]] += G[0, k] * rest / math.factorial(len(w))
    for g in (O.backward_dense(X, N, G)[0], O.backward_words(X, W, G)[0]):
        np.testing.assert_allclose(g[1], expect, rtol=1e-12)
        np.testing.assert_allclose(g[0], -expect, rtol=1e-12)


def test_backward_repeated_point_gets_consistent_gradient():
    # inserting a repeated point: the two copies' gradients add up to the original point's gradient
    d, N, L = 2, 4, 5
    X = _grid_path(94, 1, L, d).astype(np.float32)
    G = np.random.default_rng(4).standard_normal((1, sum(d ** n for n in range(1, N + 1))))
    g = O.backward_dense(X, N, G)[0]
    Xr = np.insert(X, 2, X[:, 2], axis=1)
    gr = O.backward_dense(Xr, N, G)[0]
    np.testing.assert_allclose(gr[2] + gr[3], g[2], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(np.delete(gr, [2, 3], axis=0), np.delete(g, 2, axis=0), rtol=1e-11, atol=1e-13)


def test_error_measures():
    ref = np.array([[3.0, 4.0, 0.0, 2.0]])
    lengths = np.array([1, 1, 2, 2])
    test = ref + np.array([[0.5, 0.0, 0.0, -0.2]])
    e = O.level_errors(test, ref, lengths)
    assert abs(e[1] - 0.1) < 1e-15 and abs(e[2] - 0.1) < 1e-15
    g = O.grad_errors(np.array([[[1.0, 2.5]]]), np.array([[[1.0, 2.0]]]))
    assert abs(g[0] - 0.25) < 1e-15


def test_leadlag_sparse_words_against_brute_force():
    """The sparse lead-lag set (Section 8) by its definition: all products of generators, enumerated by brute force
    over sequences of generators, against the oracle's membership test."""
    import itertools
    for d, depth in [(1, 4), (2, 4), (3, 3)]:
        gens = [(d + i,) for i in range(d)] + [(i, d + i) for i in range(d)] + [(d + i, i) for i in range(d)]
        brute = set()
        for p in range(1, depth + 1):
            for combo in itertools.product(gens, repeat=p):
                w = tuple(c for g in combo for c in g)
                if len(w) <= depth:
                    brute.add(w)
        assert O.leadlag_sparse_words(d, depth) == sorted(brute, key=lambda w: (len(w), w))


def test_graph_words_special_cases():
    # the complete graph with loops gives the truncation; a graph without edges only the letters
    full = [(a, b) for a in range(3) for b in range(3)]
    assert O.graph_words(3, full, 4) == O.truncated_words(3, 4)
    assert O.graph_words(4, [], 5) == [(i,) for i in range(4)]
    # a chain 0 -> 1 -> 2: words are the runs
    assert O.graph_words(3, [(0, 1), (1, 2)], 3) == [(0,), (1,), (2,), (0, 1), (1, 2), (0, 1, 2)]


def test_leadlag_area_is_quadratic_variation():
    """Level 2 of the lead-lag path holds the discrete quadratic (co)variation (the property Section 8 recalls; the
    lead copy moves first): S(lead_i, lag_j) - S(lag_i, lead_j) = sum_k dX^i_k dX^j_k, for i = j the antisymmetric
    part between the two copies of a coordinate."""
    rng = np.random.default_rng(5)
    X = np.cumsum(rng.standard_normal((2, 9, 2)), axis=1).astype(np.float32)
    Y = O.leadlag_transform(X)
    assert Y.shape == (2, 17, 4)
    assert np.array_equal(Y[:, 0], np.concatenate([X[:, 0], X[:, 0]], axis=-1))
    assert np.array_equal(Y[:, -1], np.concatenate([X[:, -1], X[:, -1]], axis=-1))
    d = 2
    W = O.truncated_words(2 * d, 2)
    Sg = O.forward_words(Y, W)
    dX = np.diff(X.astype(np.float64), axis=1)
    for i in range(d):
        for j in range(d):
            a = Sg[:, W.index((d + i, j))] - Sg[:, W.index((i, d + j))]
            np.testing.assert_allclose(a, (dX[:, :, i] * dX[:, :, j]).sum(axis=1), rtol=1e-10, atol=1e-12)


def test_windows_by_chen_and_finite_differences():
    """Signatures over windows (Section 5): S_{0,r} = S_{0,l} (x) S_{l,r} (Chen) ties every window to two expanding
    ones; the windowed gradient is checked against central differences of the windowed forward."""
    d, N, B, L = 2, 4, 2, 9
    W = O.truncated_words(d, N)
    X = _grid_path(95, B, L, d)
    windows = [(0, 9), (2, 7), (4, 5), (3, 3), (0, 4), (4, 9)]
    Sw = O.forward_windows(X.astype(np.float32), W, windows)
    assert Sw.shape == (B, len(windows), len(W))
    assert np.all(Sw[:, 3] == 0.0)                                     # a single point: the identity
    for k, (l, r) in enumerate(windows):
        if l == 0 or l == r:
            continue
        for b in range(B):
            head = np.concatenate([[1.0], O.forward_dense(X[b:b + 1, :l + 1].astype(np.float32), N)[0]])
            mid = np.concatenate([[1.0], Sw[b, k]])
            whole = O.forward_dense(X[b:b + 1, :r + 1].astype(np.float32), N)[0]
            np.testing.assert_allclose(O.tensor_product(d, N, head, mid)[1:], whole, rtol=1e-12, atol=1e-14)
    G = np.random.default_rng(3).standard_normal(Sw.shape)
    ana = O.backward_windows(X.astype(np.float32), W, windows, G)
    fun = lambda Y: float((O.forward_windows(Y.astype(np.float32), W, windows) * G).sum())
    num = fd_grad(fun, X, 2.0 ** -12)
    np.testing.assert_allclose(ana, num, rtol=2e-6, atol=2e-6)


def test_lyndon_words_and_tensor_log():
    """Log-signature coordinates (Section 3.3).  Counts by Witt's formula; a single segment has a log-signature of
    level 1 only; two segments give the Baker-Campbell-Hausdorff area term 1/2 (a_i b_j - a_j b_i) at the Lyndon word
    (i, j); exponentiating the logarithm returns the signature."""
    def mobius(n):
        r, p, m = 1, 2, n
        while p * p <= m:
            if m % p == 0:
                m //= p
                if m % p == 0:
                    return 0
                r = -r
            p += 1
        return -r if m > 1 else r
    for d, N in [(2, 6), (3, 4), (4, 3)]:
        lyn = O.lyndon_words(d, N)
        for n in range(1, N + 1):
            witt = sum(mobius(k) * d ** (n // k) for k in range(1, n + 1) if n % k == 0) // n
            assert sum(1 for w in lyn if len(w) == n) == witt
    # the orientation of the definition (a word strictly smaller than all of its proper rotations), as a literal list
    assert O.lyndon_words(2, 4) == [(0,), (1,), (0, 1), (0, 0, 1), (0, 1, 1), (0, 0, 0, 1), (0, 0, 1, 1), (0, 1, 1, 1)]
    assert O.lyndon_words(3, 2) == [(0,), (1,), (2,), (0, 1), (0, 2), (1, 2)]
    d, N = 3, 4
    lyn = O.lyndon_words(d, N)
    a = np.array([0.3, -0.7, 0.2])
    b = np.array([-0.4, 0.1, 0.9])
    one = np.stack([np.zeros(d), a])[None].astype(np.float32)
    L1 = O.logsig_from_path(one, N)[0]
    for k, w in enumerate(lyn):
        ref = float(np.float32(a[w[0]])) if len(w) == 1 else 0.0
        assert abs(L1[k] - ref) <= 1e-12
    two = np.stack([np.zeros(d), a, a + b])[None].astype(np.float32)
    af, bf = two[0, 1].astype(np.float64), (two[0, 2].astype(np.float64) - two[0, 1].astype(np.float64))
    L2 = O.logsig_from_path(two, N)[0]
    for k, w in enumerate(lyn):
        if len(w) == 1:
            assert abs(L2[k] - (af[w[0]] + bf[w[0]])) <= 1e-12
        if len(w) == 2:
            i, j = w
            assert i < j                                   # a Lyndon word of length 2 is increasing
            assert abs(L2[k] - 0.5 * (af[i] * bf[j] - af[j] * bf[i])) <= 1e-12
    assert sorted(w for w in lyn if len(w) == 2) == [(i, j) for i in range(d) for j in range(i + 1, d)]
    # exp(log S) = S on a longer path
    X = make_path("iid", 99, 1, 7, d)
    Sd = np.concatenate([[1.0], O.forward_dense(X, N)[0]])
    Lg = O.tensor_log(d, N, Sd)
    assert Lg[0] == 0.0
    ex = np.zeros_like(Sd)
    term = np.zeros_like(Sd)
    term[0] = 1.0
    ex += term
    for k in range(1, N + 1):
        term = O.tensor_product(d, N, term, Lg) / k
        ex += term
    np.testing.assert_allclose(ex, Sd, rtol=1e-12, atol=1e-14)
