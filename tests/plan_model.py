"""fp64 numpy model of what the table-driven kernels do with a launch plan.

Host-logic test helper: it interprets the unit programs exactly as the kernels' documentation
describes them (one accumulator row per word length, pre-order walk, LEAVE ops for the adjoint),
so that the planner and the step recursions can be checked against the oracle without a GPU.
It is not part of the product and not part of the oracle.
"""
import numpy as np

LEAF, ENTER, LEAVE = 0, 1, 2


def decode(op):
    op = int(op)
    return op & 0xfff, (op >> 12) & 0xf, (op >> 16) & 0xf, (op >> 20) & 3


def forward(plan, path, n_words):
    X = np.asarray(path, dtype=np.float64)
    B, P, d = X.shape
    out = np.full((B, n_words), np.nan)
    written = np.zeros(n_words, dtype=np.int64)
    for (op_off, n_ops, slot_off, n_slots) in plan["units"]:
        prog = [decode(o) for o in plan["ops"][op_off:op_off + n_ops]]
        sw = plan["slot_word"][slot_off:slot_off + n_slots]
        S = np.zeros((n_slots, B))
        A = {0: {t: np.ones(B) for t in range(0, 20)}}
        for j in range(1, P):
            dx = X[:, j] - X[:, j - 1]
            row = 0
            for letter, level, h, kind in prog:
                if kind == LEAVE:
                    continue
                s = S[row].copy()
                A[level] = {}
                for t in range(1, h + 1):
                    A[level][t] = s + dx[:, letter] / (t + 1) * A[level - 1][t + 1]
                S[row] = s + dx[:, letter] * A[level - 1][1]
                A[level][0] = S[row]
                row += 1
        for r, w in enumerate(sw):
            if w >= 0:
                out[:, w] = S[r]
                written[w] += 1
    return out, written


def backward(plan, path, coeffs, grad_coeffs):
    X = np.asarray(path, dtype=np.float64)
    B, P, d = X.shape
    L = P - 1
    gdx = np.zeros((B, L, d))
    for (op_off, n_ops, slot_off, n_slots) in plan["units"]:
        prog = [decode(o) for o in plan["ops"][op_off:op_off + n_ops]]
        sw = plan["slot_word"][slot_off:slot_off + n_slots]
        S = np.zeros((n_slots, B))
        Ab = np.zeros((n_slots, B))
        for r, w in enumerate(sw):
            wi = w if w >= 0 else ~w
            S[r] = coeffs[:, wi]
            if w >= 0:
                Ab[r] = grad_coeffs[:, wi]
        ones = {t: np.ones(B) for t in range(0, 20)}
        for st in range(L - 1, -1, -1):
            dx = X[:, st + 1] - X[:, st]
            am, ap, gb, slot = {0: ones}, {0: ones}, {0: {t: np.zeros(B) for t in range(20)}}, {}
            row = 0
            for letter, level, h, kind in prog:
                dxl = dx[:, letter]
                if kind == LEAF:
                    s, a = S[row].copy(), Ab[row]
                    S[row] = s - dxl * am[level - 1][1]
                    gdx[:, st, letter] += a * ap[level - 1][1]
                    gb[level - 1][1] = gb[level - 1][1] + dxl * a
                    row += 1
                elif kind == ENTER:
                    s = S[row].copy()
                    am[level] = {t: s - dxl / (t + 1) * am[level - 1][t + 1] for t in range(1, h + 1)}
                    sp = s - dxl * am[level - 1][1]
                    S[row] = sp
                    ap[level] = {t: sp + dxl / (t + 1) * ap[level - 1][t + 1] for t in range(1, h + 1)}
                    gb[level] = {t: np.zeros(B) for t in range(1, h + 1)}
                    slot[level] = row
                    row += 1
                else:
                    r = slot[level]
                    a = Ab[r].copy()
                    asum = a.copy()
                    gsum = a * ap[level - 1][1]
                    gb[level - 1][1] = gb[level - 1][1] + dxl * a
                    for t in range(1, h + 1):
                        g = gb[level][t]
                        asum += g
                        gsum += g / (t + 1) * ap[level - 1][t + 1]
                        gb[level - 1][t + 1] = gb[level - 1][t + 1] + dxl / (t + 1) * g
                    Ab[r] = asum
                    gdx[:, st, letter] += gsum
        # after stepping back through every segment the reconstructed signature must be S_{0,0} = 1,
        # i.e. zero on every non-empty word
        assert np.abs(S).max() < 1e-9 * max(1.0, np.abs(coeffs).max()), "reconstruction did not return to the identity"
    gp = np.zeros((B, P, d))
    gp[:, 1:] += gdx
    gp[:, :-1] -= gdx
    return gp
