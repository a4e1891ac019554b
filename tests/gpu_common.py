"""Shared helpers of the GPU parity tests: build a word set both ways, run the HIP path through the
C ABI, run the oracle on the same fp32 inputs, and measure the errors in the form the tolerances are
stated in.

Tolerances (written here once, used by every parity test):
  forward   per word length n:  max_b  max_{|w|=n} |gpu - oracle| / ||oracle_b restricted to length n||_2  <= 1e-4
  backward  per path:           ||gpu - oracle||_inf / ||oracle||_inf                                     <= 1e-3
The oracle gradient is itself pinned to fp64 central differences (tests/test_oracle_pins.py).
"""
import numpy as np

import paper_2602_24066_amd as S
from oracle import sig_oracle as O
from sig_workloads import WORKLOADS, make_grad_coeffs, workload_path, workload_word_list

FWD_TOL = 1e-4
BWD_TOL = 1e-3


def build_both(kind, d, depth=None, weights=None, cutoff=None, words=None):
    """Returns (gpu word set [uploaded], canonical word list from the oracle's builder)."""
    if kind == "truncated":
        ws = S.sig_wordset_build_truncated(d, depth)
        W = O.truncated_words(d, depth)
    elif kind == "anisotropic":
        ws = S.sig_wordset_build_anisotropic(d, weights, cutoff)
        W = O.anisotropic_words(d, weights, cutoff)
    else:
        ws = S.sig_wordset_build(d, words)
        W = O.prefix_closure(words)
    assert ws.size == len(W)
    ws.upload("cuda:0")
    return ws, W


def build_for_workload(wl):
    return build_both(wl.kind, wl.d, depth=wl.depth, weights=wl.weights, cutoff=wl.cutoff,
                      words=workload_word_list(wl))


def oracle_forward(X, W, kind, depth):
    if kind == "truncated":
        return O.forward_dense(X, depth)
    return O.forward_words(X, W)


def oracle_backward(X, W, kind, depth, G):
    if kind == "truncated":
        return O.backward_dense(X, depth, G)
    return O.backward_words(X, W, G)


def gpu_forward_backward(ws, X, G, checkpointed=False):
    """sig_forward + sig_backward, or the pair of calls that keeps the time-chunk signatures between them."""
    import torch
    xp = torch.from_numpy(X).cuda()
    if checkpointed:
        coeffs, ck = S.sig_forward_checkpointed(ws, xp)
        gp = S.sig_backward_checkpointed(ws, xp, coeffs, torch.from_numpy(G).cuda(), ck) if G is not None else None
    else:
        coeffs = S.sig_forward(ws, xp)
        gp = S.sig_backward(ws, xp, coeffs, torch.from_numpy(G).cuda()) if G is not None else None
    torch.cuda.synchronize()
    return coeffs.cpu().numpy(), (gp.cpu().numpy() if gp is not None else None)


def check_parity(ws, W, kind, depth, X, G, sample=None, what="", checkpointed=False):
    """Runs the HIP path on the whole batch and the oracle on `sample` (indices) or on everything."""
    coeffs, gp = gpu_forward_backward(ws, X, G, checkpointed)
    assert np.isfinite(coeffs).all(), what
    idx = np.arange(X.shape[0]) if sample is None else np.asarray(sample)
    Xs = np.ascontiguousarray(X[idx])
    ref = oracle_forward(Xs, W, kind, depth)
    lengths = np.array([len(w) for w in W])
    errs = O.level_errors(coeffs[idx], ref, lengths)
    for n, e in errs.items():
        assert e <= FWD_TOL, f"{what}: forward level {n} error {e:.3e} > {FWD_TOL}"
    gerr = None
    if G is not None:
        assert np.isfinite(gp).all(), what
        gref = oracle_backward(Xs, W, kind, depth, G[idx].astype(np.float64))
        gerr = O.grad_errors(gp[idx], gref)
        assert gerr.max() <= BWD_TOL, f"{what}: gradient error {gerr.max():.3e} > {BWD_TOL}"
    return errs, gerr
