"""The entry point that allocates nothing (sig_backward_static: the library's static device array instead of a
workspace argument) against sig_backward on the same inputs, through the C ABI; two calls in a row on every word set,
the second with a smaller input, so that what the first call left in the shared array must not leak into the second."""
import ctypes

import numpy as np
import pytest

import paper_2602_24066_amd as S
from oracle import sig_oracle as O
from sig_workloads import make_grad_coeffs, make_path, random_prefix_closed_words
from tests.gpu_common import BWD_TOL, build_both, oracle_backward

pytestmark = pytest.mark.gpu

CASES = [
    # kind, word-set arguments, (B, L) of the first call, (B, L) of the second
    ("truncated", dict(d=8, depth=5), (3, 21), (2, 9)),        # eight wavefronts per path add into the gradient array
    ("truncated", dict(d=16, depth=4), (2, 40), (1, 17)),
    ("truncated", dict(d=4, depth=6), (5, 40), (3, 8)),        # chunks of a path in one workgroup
    ("truncated", dict(d=6, depth=4), (4, 30), (2, 7)),        # a word per lane, compiled at run time
    ("words", dict(d=5, n_words=300, max_len=5), (70, 33), (66, 10)),   # straight-line kernels: transposed increments too
    ("anisotropic", dict(d=4, weights=(1.0, 1.0, 2.0, 3.0), cutoff=5.0), (9, 26), (4, 5)),
]


def _static_call(ws, xp, coeffs, grad, out):
    import torch
    lib = S.load_library()
    B, P, _ = xp.shape
    return lib.sig_backward_static(ws._h, ctypes.c_void_p(xp.data_ptr()), ctypes.c_void_p(coeffs.data_ptr()),
                                   ctypes.c_void_p(grad.data_ptr()), B, P, ctypes.c_void_p(out.data_ptr()),
                                   ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))


@pytest.mark.parametrize("case", range(len(CASES)))
def test_static_scratch_entry_point_matches_sig_backward(case):
    import torch
    kind, kw, first, second = CASES[case]
    d = kw["d"]
    words = random_prefix_closed_words(2100 + case, d, kw["n_words"], kw["max_len"]) if kind == "words" else None
    ws, W = build_both(kind, d, depth=kw.get("depth"), weights=kw.get("weights"), cutoff=kw.get("cutoff"), words=words)
    for call, (B, L) in enumerate((first, second)):
        X = make_path("iid", 2200 + 10 * case + call, B, L, d)
        G = make_grad_coeffs(2300 + 10 * case + call, B, ws.size)
        xp, grad = torch.from_numpy(X).cuda(), torch.from_numpy(G).cuda()
        coeffs = S.sig_forward(ws, xp)
        out = torch.full((B, L + 1, d), float("nan"), device="cuda")
        if call == 0 and ws.kernel_name(True, B, L + 1) in ("sig_bwd_jit", "sig_bwd_lanes"):
            # a run-time compiled kernel that this process has not loaded yet: refused, nothing enqueued
            assert _static_call(ws, xp, coeffs, grad, out) == -11
            torch.cuda.synchronize()
            assert torch.isnan(out).all()
        ref = S.sig_backward(ws, xp, coeffs, grad)          # the existing entry point (loads the kernel where needed)
        got = S.sig_backward_static(ws, xp, coeffs, grad, out)
        torch.cuda.synchronize()
        ref, got = ref.cpu().numpy(), got.cpu().numpy()
        assert np.isfinite(got).all()
        assert O.grad_errors(got, ref.astype(np.float64)).max() <= BWD_TOL, f"case {case} call {call}: differs from sig_backward"
        gref = oracle_backward(X, W, kind, kw.get("depth"), G.astype(np.float64))
        assert O.grad_errors(got, gref).max() <= BWD_TOL, f"case {case} call {call}: differs from the oracle"


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    ws, _ = build_both("truncated", 8, depth=5)
    B, P = 1024, 2049                                        # gradient of the increments alone: 64 MiB
    lib = S.load_library()
    assert lib.sig_backward_workspace_bytes(ws._h, B, P) > S.binding.SIG_STATIC_SCRATCH_BYTES
    dummy = torch.zeros(256, device="cuda")
    p = ctypes.c_void_p(dummy.data_ptr())                    # never dereferenced: the size check comes first
    assert lib.sig_backward_static(ws._h, p, p, p, B, P, p, None) == -7
    torch.cuda.synchronize()
