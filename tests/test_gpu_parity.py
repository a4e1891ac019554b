"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element."""
import numpy as np
import pytest

import paper_2602_24066_amd as S
from oracle import sig_oracle as O
from sig_workloads import (WORKLOADS, make_grad_coeffs, make_path, random_prefix_closed_words, workload_path)
from tests.gpu_common import BWD_TOL, FWD_TOL, build_both, build_for_workload, check_parity, gpu_forward_backward

pytestmark = pytest.mark.gpu


# small cases: spans several work units, a ragged last group of paths (B not a multiple of 64),
# single-segment and single-path inputs
SMALL = [
    ("truncated", dict(d=2, depth=4), 32, 64, "iid"),
    ("truncated", dict(d=3, depth=5), 70, 33, "scaled"),
    ("truncated", dict(d=4, depth=6), 5, 17, "time0"),
    ("truncated", dict(d=8, depth=3), 129, 9, "iid"),
    ("truncated", dict(d=16, depth=3), 3, 40, "ar1"),
    ("truncated", dict(d=8, depth=5), 3, 21, "scaled"),
    ("truncated", dict(d=16, depth=4), 2, 19, "ar1"),
    # d = 1: a level is a single number (X_L - X_0)^n / n!; a path that returns towards its start cancels
    # it in fp32, so the one-letter case uses the monotone time channel (level n = 1/n!)
    ("truncated", dict(d=1, depth=6), 2, 12, "time0"),
    ("truncated", dict(d=5, depth=1), 65, 12, "iid"),
    ("truncated", dict(d=3, depth=4), 1, 1, "iid"),
    ("truncated", dict(d=2, depth=10), 4, 25, "iid"),
    ("anisotropic", dict(d=6, weights=(1, 1, 2, 2, 3, 3), cutoff=6.0), 66, 30, "iid"),
    # the only word of length 7 here is letter 0 seven times, (X_L - X_0)^7 / 7!: as for d = 1 the channel must
    # be monotone for that level to be well conditioned in fp32
    ("anisotropic", dict(d=3, weights=(1.0, 2.0, 1.5), cutoff=7.0), 10, 21, "time0"),
    ("words", dict(d=10, n_words=1500, max_len=6), 67, 20, "iid"),
    ("words", dict(d=4, n_words=400, max_len=9), 12, 15, "iid"),
    ("words", dict(d=40, n_words=300, max_len=3), 9, 10, "iid"),
]


@pytest.mark.parametrize("case", range(len(SMALL)))
def test_small_cases_elementwise(case):
    kind, kw, B, L, dist = SMALL[case]
    d = kw["d"]
    words = None
    if kind == "words":
        words = random_prefix_closed_words(100 + case, d, kw["n_words"], kw["max_len"])
    ws, W = build_both(kind, d, depth=kw.get("depth"), weights=kw.get("weights"), cutoff=kw.get("cutoff"), words=words)
    X = make_path(dist, 200 + case, B, L, d)
    G = make_grad_coeffs(300 + case, B, ws.size)
    check_parity(ws, W, kind, kw.get("depth"), X, G, what=f"small[{case}]")


def d4_inputs(seed, B, L):
    """Inputs for the register-resident d = 4 kernels: the monotone time channel of c2, and paths whose increments
    change sign in every channel (iid; per-channel scales for longer paths), so that chunk-boundary adjoints and the
    products in LDS see both signs everywhere."""
    dists = ["time0", "iid"] + (["scaled"] if L >= 64 else [])
    return [(dist, make_path(dist, seed + 7 * k, B, L, 4)) for k, dist in enumerate(dists)]


# Time chunks (Chen's relation between chunk signatures): forced chunk counts, including chunk lengths that do not
# divide L and a last chunk of a single segment; the automatic choice is exercised by the small batches below.
@pytest.mark.parametrize("d,depth,B,L,chunks", [(4, 6, 3, 97, 3), (4, 6, 2, 65, 2), (4, 6, 1, 160, 5), (8, 5, 2, 100, 3),
                                                (16, 4, 1, 129, 4), (4, 6, 2, 600, 0), (16, 4, 3, 700, 0)])
def test_time_chunks(monkeypatch, d, depth, B, L, chunks):
    if chunks:
        monkeypatch.setenv("SIG_CHUNKS", str(chunks))
    else:
        monkeypatch.delenv("SIG_CHUNKS", raising=False)
    ws, W = build_both("truncated", d, depth=depth)
    G = make_grad_coeffs(600 + L, B, ws.size)
    lib = S.load_library()
    if chunks:
        assert lib.sig_forward_workspace_bytes(ws._h, B, L + 1) >= 4 * B * chunks * ws.size
    else:
        assert lib.sig_forward_workspace_bytes(ws._h, B, L + 1) > 0      # few paths: chunking is chosen by itself
    inputs = d4_inputs(500 + L, B, L) if d == 4 else [("iid", make_path("iid", 500 + L, B, L, d))]
    for dist, X in inputs:
        check_parity(ws, W, "truncated", depth, X, G, what=f"chunks d={d} N={depth} L={L} C={chunks} {dist}")


# d = 4 backward with one wavefront per (path, chunk) row, forced for batches that would not select it
@pytest.mark.parametrize("B,L,chunks", [(3, 97, 3), (5, 17, 0), (130, 40, 0), (2, 160, 5), (1, 1, 0), (70, 64, 2)])
def test_backward_one_wavefront_per_row(monkeypatch, B, L, chunks):
    monkeypatch.setenv("SIG_BWD_TAILS", "1")
    if chunks:
        monkeypatch.setenv("SIG_CHUNKS", str(chunks))
    else:
        monkeypatch.delenv("SIG_CHUNKS", raising=False)
    ws, W = build_both("truncated", 4, depth=6)
    G = make_grad_coeffs(800 + L, B, ws.size)
    for dist, X in d4_inputs(700 + L, B, L):
        check_parity(ws, W, "truncated", 6, X, G, what=f"tails B={B} L={L} C={chunks} {dist}")


# ... and its fused form: the 2, 4 or 8 chunks of a path in one workgroup, chunk signatures and boundary adjoints in
# LDS; the last three cases take it by themselves (8, 4 and 2 chunks)
@pytest.mark.parametrize("B,L,chunks", [(3, 97, 4), (1, 33, 4), (5, 64, 4), (2, 35, 4), (1, 300, 4), (2, 2000, 4),
                                        (3, 17, 2), (70, 40, 2), (2, 16, 2), (2, 801, 2),
                                        (3, 97, 8), (1, 64, 8), (2, 67, 8), (5, 255, 8), (1, 1500, 8),
                                        (200, 100, 0), (300, 64, 0), (1000, 24, 0)])
def test_backward_chunks_in_one_workgroup(monkeypatch, B, L, chunks):
    if chunks:
        monkeypatch.setenv("SIG_BWD_TAILS", str(chunks))
    else:
        monkeypatch.delenv("SIG_BWD_TAILS", raising=False)
    monkeypatch.delenv("SIG_CHUNKS", raising=False)
    ws, W = build_both("truncated", 4, depth=6)
    G = make_grad_coeffs(950 + L, B, ws.size)
    lib = S.load_library()
    gdx = (4 * B * L * 4 + 255) // 256 * 256
    assert lib.sig_backward_workspace_bytes(ws._h, B, L + 1) == gdx       # no chunk arrays in device memory
    for dist, X in d4_inputs(900 + L, B, L):
        check_parity(ws, W, "truncated", 6, X, G, what=f"fused tails B={B} L={L} C={chunks} {dist}")


# forward with the 2 or 4 chunks of a path in one workgroup (d = 4, depth 6), forced for any batch size; the last
# two cases take it by themselves (batch sizes in its range)
@pytest.mark.parametrize("B,L,chunks", [(3, 97, 4), (1, 32, 4), (5, 64, 4), (2, 35, 4), (1, 300, 4), (3, 17, 2),
                                        (70, 40, 2), (2, 16, 2), (2, 1001, 2), (130, 50, 0), (400, 33, 0)])
def test_forward_chunks_in_one_workgroup(monkeypatch, B, L, chunks):
    if chunks:
        monkeypatch.setenv("SIG_FWD_TAILS", str(chunks))
    else:
        monkeypatch.delenv("SIG_FWD_TAILS", raising=False)
    monkeypatch.delenv("SIG_CHUNKS", raising=False)
    ws, W = build_both("truncated", 4, depth=6)
    assert ws.kernel_name(False, B, L + 1) == "trunc_tails_fwd_kernel"
    G = make_grad_coeffs(1350 + L, B, ws.size)
    for dist, X in d4_inputs(1300 + L, B, L):
        check_parity(ws, W, "truncated", 6, X, G, what=f"fused forward B={B} L={L} C={chunks} {dist}")


# Forward and backward with the time-chunk signatures kept between the two calls (checkpointed form): every chunk
# count, chunk lengths that do not divide L, the launcher's own choice, and shapes where it takes no chunks at all
@pytest.mark.parametrize("d,depth,B,L,chunks", [(8, 5, 2, 200, 0), (8, 5, 3, 131, 2), (8, 5, 2, 197, 3), (8, 5, 1, 260, 4),
                                                (16, 4, 2, 150, 2), (16, 4, 1, 200, 3), (16, 4, 2, 333, 0), (8, 5, 2, 40, 0),
                                                (16, 4, 1, 530, 0), (8, 5, 2, 600, 7), (8, 5, 40, 300, 0), (8, 5, 1, 1100, 0),
                                                (4, 6, 3, 300, 0),
                                                (3, 4, 5, 100, 0)])
def test_checkpointed_forward_and_backward(d, depth, B, L, chunks):
    import torch
    ws, W = build_both("truncated", d, depth=depth)
    if chunks:
        ws.set_option("ckpt_chunks", chunks)
    lib = S.load_library()
    nck = int(lib.sig_checkpoint_bytes(ws._h, B, L + 1))
    wanted = {8: 256, 16: 128}.get(d, 0)                  # rows that fill the chip with two wavefronts per SIMD
    expect_chunks = chunks if chunks else (min(16, -(-wanted // B), L // 64) if d in (8, 16) and L >= 128 else 0)
    if not chunks and expect_chunks > 4:
        expect_chunks = 16 if expect_chunks >= 16 else (8 if expect_chunks >= 8 else 4)    # beyond four: powers of two
    assert nck == (4 * B * expect_chunks * ws.size + 255) // 256 * 256
    X = make_path("iid", 2500 + L, B, L, d)
    G = make_grad_coeffs(2600 + L, B, ws.size)
    xp, grad = torch.from_numpy(X).cuda(), torch.from_numpy(G).cuda()
    coeffs, ck = S.sig_forward_checkpointed(ws, xp)
    assert ck.numel() == nck
    gp = S.sig_backward_checkpointed(ws, xp, coeffs, grad, ck)
    torch.cuda.synchronize()
    coeffs, gp = coeffs.cpu().numpy(), gp.cpu().numpy()
    lengths = np.array([len(w) for w in W])
    for n, e in O.level_errors(coeffs, O.forward_dense(X, depth), lengths).items():
        assert e <= FWD_TOL, f"checkpointed forward, level {n}: {e:.3e}"
    gerr = O.grad_errors(gp, O.backward_dense(X, depth, G.astype(np.float64)))
    assert gerr.max() <= BWD_TOL, f"checkpointed backward: {gerr.max():.3e}"


def _no_repeat_words(d, n):
    """Words of up to n letters in which no letter follows itself: closed under prefixes and suffixes."""
    out, level = [], [(i,) for i in range(d)]
    for _ in range(n):
        out += level
        level = [w + (i,) for w in level for i in range(d) if i != w[-1]]
    return out


# The same pair of calls on word sets closed under suffixes (anisotropic sets; a word list that is): chunk counts by the
# library's rule (two and eight) and forced (two, three, four), chunk lengths that do not divide L, a batch of more than one lane group, against the
# oracle; and a list that lacks suffixes, which takes no chunks.  (Every length of these sets has several words: a length
# with a single word is ill-conditioned under the forward error measure for any summation order.)
WORD_CHUNK_CASES = {
    "aniso3": ("anisotropic", 3, (1.0, 1.25, 1.5), 4.5, None, 5, 200, 3, 3),
    "aniso6": ("anisotropic", 6, (1, 1, 2, 2, 3, 3), 8.0, None, 70, 257, 0, 2),
    "aniso6-forced": ("anisotropic", 6, (1, 1, 2, 2, 3, 3), 8.0, None, 70, 257, 4, 4),
    "aniso3-rule": ("anisotropic", 3, (1.0, 1.25, 1.5), 4.5, None, 2, 1030, 0, 8),
    "aniso2-forced": ("anisotropic", 2, (0.3, 0.4), 1.6, None, 3, 300, 2, 2),
    "no-repeat": ("list", 3, None, None, "no-repeat", 9, 130, 2, 2),
    "random": ("list", 4, None, None, "random", 4, 200, 0, 0),
}


@pytest.mark.parametrize("case", list(WORD_CHUNK_CASES))
def test_checkpointed_word_sets(case):
    import torch
    kind, d, weights, cutoff, which, B, L, forced, expect_chunks = WORD_CHUNK_CASES[case]
    words = None
    if which == "no-repeat":
        words = _no_repeat_words(d, 5)
    elif which == "random":
        words = random_prefix_closed_words(11, d, 80, 5)
    ws, W = build_both(kind, d, weights=weights, cutoff=cutoff, words=words)
    if forced:
        ws.set_option("ckpt_chunks", forced)
    assert ws.suffix_closed == (which != "random")
    lib = S.load_library()
    nck = int(lib.sig_checkpoint_bytes(ws._h, B, L + 1))
    assert nck == (4 * B * expect_chunks * ws.size + 255) // 256 * 256
    X = make_path("iid", 5100 + L, B, L, d)
    G = make_grad_coeffs(5200 + L, B, ws.size)
    xp, grad = torch.from_numpy(X).cuda(), torch.from_numpy(G).cuda()
    coeffs, ck = S.sig_forward_checkpointed(ws, xp)
    gp = S.sig_backward_checkpointed(ws, xp, coeffs, grad, ck)
    plain = S.sig_forward(ws, xp)
    gplain = S.sig_backward(ws, xp, plain, grad)
    torch.cuda.synchronize()
    if expect_chunks:                      # the checkpoint holds the signatures of the chunks: the first is that of the first Lc segments
        Lc = -(-L // expect_chunks)
        first = ck.view(torch.float32)[: B * expect_chunks * ws.size].view(B, expect_chunks, ws.size)[:, 0].cpu().numpy()
        ref_first = O.forward_words(np.ascontiguousarray(X[:, : Lc + 1]), W)
        for n, e in O.level_errors(first, ref_first, np.array([len(w) for w in W])).items():
            assert e <= FWD_TOL, f"{case}: first chunk signature, level {n}: {e:.3e}"
    coeffs, gp = coeffs.cpu().numpy(), gp.cpu().numpy()
    lengths = np.array([len(w) for w in W])
    ref = O.forward_words(X, W)
    for n, e in O.level_errors(coeffs, ref, lengths).items():
        assert e <= FWD_TOL, f"{case}: checkpointed forward, level {n}: {e:.3e}"
    gref = O.backward_words(X, W, G.astype(np.float64))
    gerr = O.grad_errors(gp, gref)
    assert gerr.max() <= BWD_TOL, f"{case}: checkpointed backward: {gerr.max():.3e}"
    assert O.grad_errors(gplain.cpu().numpy(), gref).max() <= BWD_TOL
    # sig_forward takes the same chunks, with the chunk signatures in its workspace
    for n, e in O.level_errors(plain.cpu().numpy(), ref, lengths).items():
        assert e <= FWD_TOL, f"{case}: sig_forward, level {n}: {e:.3e}"


@pytest.mark.parametrize("d,depth,B,L", [(8, 5, 3, 1100), (16, 4, 2, 1030)])
def test_plain_backward_takes_time_chunks_for_few_long_paths(d, depth, B, L):
    """sig_backward on few long paths of a full truncation recomputes the chunk signatures and walks four chunks side
    by side (its workspace then holds four chunk arrays); the result is the oracle's, and that of the entry point
    with the static scratch array, which always walks whole paths."""
    import torch
    ws, W = build_both("truncated", d, depth=depth)
    lib = S.load_library()
    gdx = (4 * B * L * d + 255) // 256 * 256
    per_array = (4 * B * 4 * ws.size + 255) // 256 * 256
    assert lib.sig_backward_workspace_bytes(ws._h, B, L + 1) == gdx + 4 * per_array
    X = make_path("iid", 6100 + L, B, L, d)
    G = make_grad_coeffs(6200 + L, B, ws.size)
    xp, grad = torch.from_numpy(X).cuda(), torch.from_numpy(G).cuda()
    coeffs = S.sig_forward(ws, xp)
    gp = S.sig_backward(ws, xp, coeffs, grad)
    gs = torch.empty_like(xp)
    S.sig_backward_static(ws, xp, coeffs, grad, gs)
    torch.cuda.synchronize()
    O.set_threads(2)
    try:
        gref = O.backward_dense(X, depth, G.astype(np.float64))
    finally:
        O.set_threads(16)
    assert O.grad_errors(gp.cpu().numpy(), gref).max() <= BWD_TOL
    assert O.grad_errors(gs.cpu().numpy(), gref).max() <= BWD_TOL


def test_checkpointed_word_sets_reject_bad_buffers():
    """Buffers that are missing, too small or misaligned are refused with an error code before anything is launched."""
    import ctypes
    import torch
    ws, W = build_both("anisotropic", 3, weights=(1.0, 1.25, 1.5), cutoff=4.5)
    ws.set_option("ckpt_chunks", 3)
    lib = S.load_library()
    B, L = 5, 200
    nck = int(lib.sig_checkpoint_bytes(ws._h, B, L + 1))
    nf = int(lib.sig_forward_checkpointed_workspace_bytes(ws._h, B, L + 1))
    nb = int(lib.sig_backward_checkpointed_workspace_bytes(ws._h, B, L + 1))
    assert nck > 0 and nf > 0 and nb > 0
    xp = torch.from_numpy(make_path("iid", 5300, B, L, 3)).cuda()
    grad = torch.from_numpy(make_grad_coeffs(5301, B, ws.size)).cuda()
    coeffs = torch.full((B, ws.size), 3.0, dtype=torch.float32, device="cuda")
    gpath = torch.full((B, L + 1, 3), 3.0, dtype=torch.float32, device="cuda")
    ck = torch.zeros(nck + 256, dtype=torch.uint8, device="cuda")
    wk = torch.zeros(max(nf, nb) + 256, dtype=torch.uint8, device="cuda")
    assert ck.data_ptr() % 256 == 0 and wk.data_ptr() % 256 == 0
    P = ctypes.c_void_p

    def fwd(ckp, ckn, wp, wn):
        return lib.sig_forward_checkpointed(ws._h, P(xp.data_ptr()), B, L + 1, P(coeffs.data_ptr()), P(ckp), ckn, P(wp), wn, None)

    def bwd(ckp, ckn, wp, wn):
        return lib.sig_backward_checkpointed(ws._h, P(xp.data_ptr()), P(coeffs.data_ptr()), P(grad.data_ptr()), P(ckp), ckn, B, L + 1,
                                             P(gpath.data_ptr()), P(wp), wn, None)

    for call, need in ((fwd, nf), (bwd, nb)):
        assert call(ck.data_ptr(), nck - 1, wk.data_ptr(), need) == -5
        assert call(0, nck, wk.data_ptr(), need) == -5
        assert call(ck.data_ptr(), nck, wk.data_ptr(), need - 1) == -5
        assert call(ck.data_ptr(), nck, 0, need) == -5
        assert call(ck.data_ptr() + 4, nck, wk.data_ptr(), need) == -1
        assert call(ck.data_ptr(), nck, wk.data_ptr() + 4, need) == -1
    torch.cuda.synchronize()
    assert (coeffs == 3.0).all() and (gpath == 3.0).all() and (ck == 0).all()      # nothing ran
    assert fwd(ck.data_ptr(), nck, wk.data_ptr(), nf) == 0 and bwd(ck.data_ptr(), nck, wk.data_ptr(), nb) == 0
    torch.cuda.synchronize()
    gref = O.backward_words(xp.cpu().numpy(), W, grad.cpu().numpy().astype(np.float64))
    assert O.grad_errors(gpath.cpu().numpy(), gref).max() <= BWD_TOL


# Every tile shape of the d = 16 and d = 8 backward kernels, forced on batches far too small to take them by themselves:
# tiles that do not divide the number of segments, a single ragged tile, with and without time chunks
@pytest.mark.parametrize("d,depth,tile", [(16, 4, 4), (16, 4, 8), (16, 4, 12), (16, 4, 16), (8, 5, 4), (8, 5, 8), (8, 5, 16)])
@pytest.mark.parametrize("B,L,chunks", [(2, 77, 0), (1, 9, 0), (3, 150, 2)])
def test_backward_tile_shapes(d, depth, tile, B, L, chunks):
    import torch
    ws, W = build_both("truncated", d, depth=depth)
    ws.set_option("bwd_tile", tile)
    X = make_path("iid", 2900 + L + tile, B, L, d)
    G = make_grad_coeffs(3000 + L + tile, B, ws.size)
    gref = O.backward_dense(X, depth, G.astype(np.float64))
    xp, grad = torch.from_numpy(X).cuda(), torch.from_numpy(G).cuda()
    if chunks:
        ws.set_option("ckpt_chunks", chunks)
        coeffs, ck = S.sig_forward_checkpointed(ws, xp)
        gp = S.sig_backward_checkpointed(ws, xp, coeffs, grad, ck)
    else:
        coeffs = S.sig_forward(ws, xp)
        gp = S.sig_backward(ws, xp, coeffs, grad)
    torch.cuda.synchronize()
    gerr = O.grad_errors(gp.cpu().numpy(), gref)
    assert gerr.max() <= BWD_TOL, f"d={d} tile={tile} B={B} L={L} chunks={chunks}: {gerr.max():.3e}"


@pytest.mark.parametrize("d,depth,B,L", [(8, 5, 2, 300), (16, 4, 2, 400), (4, 6, 3, 257)])
def test_reconstruction_returns_to_the_empty_signature(d, depth, B, L):
    """Stepping the terminal signature back through all segments (Proposition 4.6) must end at the signature of the
    empty path (Lemma 4.5): the kernels report the largest coefficient they are left with, and the gradient of the
    same call is the ordinary one."""
    import torch
    ws, W = build_both("truncated", d, depth=depth)
    X = make_path("iid", 2700 + L, B, L, d)
    G = make_grad_coeffs(2800 + L, B, ws.size)
    xp, grad = torch.from_numpy(X).cuda(), torch.from_numpy(G).cuda()
    coeffs = S.sig_forward(ws, xp)
    gp, resid = S.sig_backward_residual(ws, xp, coeffs, grad)
    torch.cuda.synchronize()
    resid = resid.cpu().numpy()
    scale = float(coeffs.abs().max())
    assert resid.shape == (B,) and np.all(resid >= 0.0) and resid.max() <= 1e-4 * max(scale, 1.0), (resid, scale)
    gerr = O.grad_errors(gp.cpu().numpy(), O.backward_dense(X, depth, G.astype(np.float64)))
    assert gerr.max() <= BWD_TOL
    # a terminal signature that is not the path's own does not come back to zero: the check discriminates
    wrong = coeffs.clone()
    wrong[:, 0] += 0.5
    _, resid2 = S.sig_backward_residual(ws, xp, wrong, grad)
    assert float(resid2.min()) > 0.1


def test_forward_fused_and_four_wavefront_kernels_agree():
    ws, W = build_both("truncated", 4, depth=6)
    X = make_path("time0", 21, 200, 255, 4)
    G = make_grad_coeffs(22, 200, ws.size)
    ws.set_option("fwd_tails", 0)
    assert ws.kernel_name(False, 200, 256) == "trunc_mfma_fwd_kernel"
    c0, _ = gpu_forward_backward(ws, X, G)
    ws.set_option("fwd_tails", -1)
    assert ws.kernel_name(False, 200, 256) == "trunc_tails_fwd_kernel"
    c4, _ = gpu_forward_backward(ws, X, G)
    lengths = np.array([len(w) for w in W])
    for n, e in O.level_errors(c4, c0.astype(np.float64), lengths).items():
        assert e <= 1e-5, (n, e)


def test_rows_that_are_not_16_byte_aligned():
    """coeffs / grad_coeffs four bytes off a 16-byte boundary: the d = 4 kernels that use vector loads and stores step
    aside for the ones that do not, with the same results."""
    import torch
    ws, W = build_both("truncated", 4, depth=6)
    B, L = 130, 70
    X = make_path("time0", 31, B, L, 4)
    G = make_grad_coeffs(32, B, ws.size)
    xp = torch.from_numpy(X).cuda()
    buf_c = torch.empty(B * ws.size + 1, dtype=torch.float32, device="cuda")
    buf_g = torch.empty(B * ws.size + 1, dtype=torch.float32, device="cuda")
    c_off = buf_c[1:].view(B, ws.size)
    g_off = buf_g[1:].view(B, ws.size)
    assert c_off.data_ptr() % 16 == 4 and c_off.is_contiguous()
    g_off.copy_(torch.from_numpy(G))
    S.sig_forward(ws, xp, out=c_off)
    gp_off = S.sig_backward(ws, xp, c_off, g_off)
    c = S.sig_forward(ws, xp)
    gp = S.sig_backward(ws, xp, c, torch.from_numpy(G).cuda())
    lengths = np.array([len(w) for w in W])
    for n, e in O.level_errors(c_off.cpu().numpy(), c.cpu().numpy().astype(np.float64), lengths).items():
        assert e <= 1e-5, (n, e)
    assert O.grad_errors(gp_off.cpu().numpy(), gp.cpu().numpy().astype(np.float64)).max() <= 1e-4
    for n, e in O.level_errors(c_off.cpu().numpy(), O.forward_words(X, W), lengths).items():
        assert e <= FWD_TOL, (n, e)
    assert O.grad_errors(gp_off.cpu().numpy(), O.backward_words(X, W, G.astype(np.float64))).max() <= BWD_TOL


def test_chunked_and_unchunked_agree():
    ws, W = build_both("truncated", 4, depth=6)
    X = make_path("iid", 11, 4, 128, 4)
    G = make_grad_coeffs(12, 4, ws.size)
    ws.set_option("chunks", 1)
    c1, g1 = gpu_forward_backward(ws, X, G)
    ws.set_option("chunks", 4)
    c4, g4 = gpu_forward_backward(ws, X, G)
    lengths = np.array([len(w) for w in W])
    for n, e in O.level_errors(c4, c1.astype(np.float64), lengths).items():
        assert e <= 1e-5, (n, e)
    assert O.grad_errors(g4, g1.astype(np.float64)).max() <= 1e-4


@pytest.mark.parametrize("kind", ["anisotropic", "words"])
def test_table_driven_kernels(monkeypatch, kind):
    """With run-time specialisation switched off the table-driven kernels serve the same word sets."""
    monkeypatch.setenv("SIG_NO_JIT", "1")
    if kind == "anisotropic":
        ws, W = build_both(kind, 4, weights=(1.0, 1.0, 2.0, 3.0), cutoff=5.0)
    else:
        ws, W = build_both(kind, 6, words=random_prefix_closed_words(77, 6, 800, 5))
    assert ws.kernel_name(False) == "fwd_generic_kernel" and ws.kernel_name(True) == "bwd_generic_kernel"
    X = make_path("iid", 78, 70, 19, ws.dim)
    G = make_grad_coeffs(79, 70, ws.size)
    check_parity(ws, W, kind, None, X, G, what=f"table-driven {kind}")


def test_many_short_paths():
    """More paths than the register-resident kernels take in one launch (65,535): the specialised kernels serve a
    full truncation too.  Sampled paths against the oracle."""
    ws, W = build_both("truncated", 4, depth=6)
    B, L = 66000, 3
    X = make_path("iid", 41, B, L, 4)
    G = make_grad_coeffs(42, B, ws.size)
    sample = [0, 1, 63, 64, 4095, 65535, 65536, B - 1]
    check_parity(ws, W, "truncated", 6, X, G, sample=sample, what="B=66000")


@pytest.mark.parametrize("d,depth,B", [(8, 5, 60000), (4, 6, 400000)])
def test_more_than_2_to_the_31_coefficients(d, depth, B):
    """Row offsets in 64 bits: 60,000 paths of the (8, 5) truncation are 2.25e9 coefficients (9 GB per array), and so
    are 400,000 paths of the (4, 6) truncation, which the run-time specialised kernels serve (lanes = paths).
    Sampled paths against the oracle, among them the row in which the element index passes 2^31 and the last one.
    The cotangent is drawn on the device (a seeded input; 2e9 normals would take the host half a minute)."""
    import torch
    ws, W = build_both("truncated", d, depth=depth)
    L = 2
    assert B * ws.size > 2**31
    X = make_path("iid", 43, B, L, d)
    xp = torch.from_numpy(X).cuda()
    gen = torch.Generator(device="cuda").manual_seed(44)
    G = torch.randn((B, ws.size), device="cuda", dtype=torch.float32, generator=gen)
    coeffs = S.sig_forward(ws, xp)
    gp = S.sig_backward(ws, xp, coeffs, G)
    torch.cuda.synchronize()
    edge = 2**31 // ws.size
    idx = np.array([0, 1, 4095, edge - 1, edge, edge + 1, B - 2, B - 1])
    sel = torch.from_numpy(idx).cuda()
    c, g, gg = coeffs[sel].cpu().numpy(), gp[sel].cpu().numpy(), G[sel].cpu().numpy()
    del coeffs, G
    Xs = np.ascontiguousarray(X[idx])
    lengths = np.array([len(w) for w in W])
    for n, e in O.level_errors(c, O.forward_dense(Xs, depth), lengths).items():
        assert e <= FWD_TOL, (n, e)
    gerr = O.grad_errors(g, O.backward_dense(Xs, depth, gg.astype(np.float64)))
    assert gerr.max() <= BWD_TOL, gerr
    assert torch.isfinite(gp).all()


@pytest.mark.parametrize("d,depth,B,L,levels", [
    (6, 5, 3, 21, 2),     # two levels per lane, 216 words of length 3: three full wavefronts and a ragged one
    (6, 5, 2, 13, 1),     # one level per lane: 1,296 lanes; the first chain letter runs over 216 of them
    (3, 6, 5, 33, 2),     # 81 lanes per path
    (3, 6, 2, 20, 1),     # 243 lanes
    (2, 7, 4, 9, 2),      # half a wavefront per path
    (7, 4, 2, 17, 2),     # 49 lanes
    (7, 4, 2, 17, 1),     # 343 lanes
    (5, 3, 6, 8, 2),      # 5 lanes per path (forced: the launcher would take lanes = paths)
    (10, 4, 2, 19, 2),    # 100 lanes with 110 coefficients each, tiles of 6 segments
    (10, 4, 1, 25, 1),    # 1,000 lanes
    (9, 4, 3, 1, 1),      # a single segment
    (12, 3, 2, 11, 1),    # 144 lanes, tiles of 5 segments
    (12, 4, 1, 7, 1),     # the first chain letter changes inside some wavefronts (runs of 144 lanes)
    (6, 6, 1, 6, 2),      # runs of 216, 36, 6 and 1 lanes
    (3, 8, 2, 10, 2),     # six chain letters, two of them with runs of 64 lanes or more
    (40, 3, 1, 5, 1),     # tiles of one segment, 65,640 coefficients from a single path
])
def test_truncations_with_lanes_as_words(d, depth, B, L, levels, monkeypatch):
    """Full truncations that have no register-resident kernel of their own: the run-time compiled kernels with a
    word per lane, in both of their forms (the d leaves, or the d children and d^2 leaves, below the lane's word),
    every coefficient and the whole gradient against the oracle."""
    monkeypatch.setenv("SIG_LANES", "1")
    monkeypatch.setenv("SIG_LANES_LEVELS", str(levels))
    ws, W = build_both("truncated", d, depth=depth)
    assert ws.kernel_name(False, B, L + 1) == "sig_fwd_lanes" and ws.kernel_name(True, B, L + 1) == "sig_bwd_lanes"
    assert f"#define R {levels}\n" in ws.jit_source(False, B) and f"#define R {levels}\n" in ws.jit_source(True, B)
    X = make_path("iid", 71 + d, B, L, d)
    G = make_grad_coeffs(72 + d, B, ws.size)
    check_parity(ws, W, "truncated", depth, X, G, what=f"lanes = words, d={d} N={depth}, {levels} levels per lane")


def test_lanes_as_words_on_a_long_path():
    """5,000 segments through the word-per-lane kernels: many staging tiles, and the reconstruction of the
    backward pass over a long walk (within the gradient tolerance, as for the 4,096 segments of c5)."""
    ws, W = build_both("truncated", 6, depth=4)
    B, L = 2, 5000
    assert ws.kernel_name(True, B, L + 1) == "sig_bwd_lanes"
    X = make_path("iid", 91, B, L, 6)
    G = make_grad_coeffs(92, B, ws.size)
    check_parity(ws, W, "truncated", 4, X, G, what="lanes = words, 5,000 segments")


def test_lanes_as_words_on_random_shapes(monkeypatch):
    """Sixteen seeded random shapes (2..20 letters, depth 2..6, up to 30,000 words, 1..5 paths of 1..40 segments),
    alternating between the two forms of the word-per-lane kernels where both exist."""
    rng = np.random.default_rng(2024)
    monkeypatch.setenv("SIG_LANES", "1")
    done = 0
    while done < 16:
        d, depth = int(rng.integers(2, 21)), int(rng.integers(2, 7))
        if sum(d ** n for n in range(1, depth + 1)) > 30000 or (d, depth) in ((4, 6), (8, 5), (16, 4)):
            continue
        B, L = int(rng.integers(1, 6)), int(rng.integers(1, 41))
        monkeypatch.setenv("SIG_LANES_LEVELS", str(1 + done % 2))
        ws, W = build_both("truncated", d, depth=depth)
        assert ws.kernel_name(True, B, L + 1) == "sig_bwd_lanes"
        X = make_path("iid", 300 + done, B, L, d)
        G = make_grad_coeffs(400 + done, B, ws.size)
        check_parity(ws, W, "truncated", depth, X, G, what=f"random shape {done}: d={d} N={depth} B={B} L={L}")
        done += 1


def test_lanes_as_words_and_lanes_as_paths_agree(monkeypatch):
    """The two run-time compiled forms of one truncation on the same inputs (each is compared with the oracle
    elsewhere; this pins the switch between them)."""
    import torch
    d, depth, B, L = 6, 4, 70, 40
    X = torch.from_numpy(make_path("iid", 81, B, L, d)).cuda()
    out = {}
    for form in ("0", "1"):
        monkeypatch.setenv("SIG_LANES", form)
        ws = S.sig_wordset_build_truncated(d, depth)
        ws.upload("cuda:0")
        assert ws.kernel_name(False, B, L + 1) == ("sig_fwd_lanes" if form == "1" else "sig_fwd_jit")
        G = torch.from_numpy(make_grad_coeffs(82, B, ws.size)).cuda()
        c = S.sig_forward(ws, X)
        g = S.sig_backward(ws, X, c, G)
        out[form] = (c.cpu().numpy(), g.cpu().numpy())
    np.testing.assert_allclose(out["0"][0], out["1"][0], rtol=2e-4, atol=1e-6)
    np.testing.assert_allclose(out["0"][1], out["1"][1], rtol=1e-3, atol=1e-4)


def test_graph_induced_word_set():
    edges = [(0, 1), (0, 2), (1, 3), (2, 3), (3, 4), (3, 5), (1, 5), (4, 5), (2, 4)]
    ws = S.sig_wordset_build_graph(6, edges, 5)
    ws.upload("cuda:0")
    W = O.graph_words(6, edges, 5)
    assert ws.size == len(W)
    X = make_path("iid", 61, 70, 33, 6)
    G = make_grad_coeffs(62, 70, ws.size)
    check_parity(ws, W, "words", None, X, G, what="graph-induced set")


def test_leadlag_transform_and_sparse_word_set():
    import torch
    d, depth, B, n = 3, 4, 9, 12
    X = make_path("iid", 63, B, n - 1, d)
    xp = torch.from_numpy(X).cuda()
    yp = S.sig_leadlag_transform(xp)
    Y = O.leadlag_transform(X)
    assert np.array_equal(yp.cpu().numpy(), Y)                       # copies only: exact
    # its adjoint against the transpose of the (linear) oracle transform, applied to a random cotangent
    Gy = np.random.default_rng(64).standard_normal(Y.shape).astype(np.float32)
    gx = S.sig_leadlag_backward(torch.from_numpy(Gy).cuda()).cpu().numpy()
    ref = np.zeros(X.shape, dtype=np.float64)
    ref += Gy[:, 0::2, :d] + Gy[:, 0::2, d:]
    ref[:, :-1] += Gy[:, 1::2, :d]
    ref[:, 1:] += Gy[:, 1::2, d:]
    np.testing.assert_allclose(gx, ref, rtol=1e-6, atol=1e-6)
    # signatures of the lead-lag path on the sparse set
    ws = S.sig_wordset_build_leadlag_sparse(d, depth)
    ws.upload("cuda:0")
    W = O.prefix_closure(O.leadlag_sparse_words(d, depth))
    assert ws.size == len(W)
    G = make_grad_coeffs(65, B, ws.size)
    check_parity(ws, W, "words", None, Y, G, what="sparse lead-lag set")


WINDOW_SETS = [
    ("truncated", dict(d=3, depth=4)),
    ("truncated", dict(d=4, depth=6)),
    ("truncated", dict(d=5, depth=4)),
    ("truncated", dict(d=6, depth=4)),           # a word per lane: 36 words of length 2
    ("truncated", dict(d=3, depth=6)),           # a word per lane: 81 words of length 4, two wavefronts per row
    ("anisotropic", dict(d=4, weights=(1.0, 1.0, 2.0, 3.0), cutoff=5.0)),
    ("words", dict(d=6, n_words=500, max_len=5)),
]


# table_driven: the fallback kernels, whose windows are gathered into padded sub-paths and scattered back
@pytest.mark.parametrize("case,B,table_driven",
                         [(c, B, False) for c in range(len(WINDOW_SETS)) for B in (5, 13)] +
                         [(c, 5, True) for c, (kind, kw) in enumerate(WINDOW_SETS) if (kw["d"], kw.get("depth")) != (4, 6)])
def test_windows(case, B, table_driven):
    """Signatures over user-given windows (expanding, sliding, overlapping, single-segment, empty, whole path) against
    one oracle evaluation per window, forward and backward."""
    import torch
    kind, kw = WINDOW_SETS[case]
    d = kw["d"]
    words = random_prefix_closed_words(400 + case, d, kw["n_words"], kw["max_len"]) if kind == "words" else None
    ws, W = build_both(kind, d, depth=kw.get("depth"), weights=kw.get("weights"), cutoff=kw.get("cutoff"), words=words)
    if table_driven:
        ws.set_option("no_jit", 1)                 # (d = 4, depth 6 has a precompiled kernel and is left out above)
        assert ws.kernel_name(True, B * 11, 41) == "bwd_generic_kernel"
    if not table_driven and kind == "truncated" and (d, kw["depth"]) in ((6, 4), (3, 6)):
        assert ws.kernel_name(True, B * 11, 41) == "sig_bwd_lanes"
    L = 40                      # B = 13: 143 (path, window) rows, more than two wavefronts of rows for the lane = row kernels
    X = make_path("iid", 410 + case, B, L, d)
    windows = [(0, L), (0, 1), (0, 7), (0, 23), (5, 15), (10, 20), (15, 25), (39, 40), (17, 17), (3, 38), (5, 15)]
    K = len(windows)
    G = make_grad_coeffs(420 + case, B * K, ws.size).reshape(B, K, ws.size)
    xp = torch.from_numpy(X).cuda()
    coeffs = S.sig_forward_windows(ws, xp, windows)
    gp = S.sig_backward_windows(ws, xp, windows, coeffs, torch.from_numpy(G).cuda())
    torch.cuda.synchronize()
    coeffs, gp = coeffs.cpu().numpy(), gp.cpu().numpy()
    ref = O.forward_windows(X, W, windows)
    lengths = np.array([len(w) for w in W])
    for k, (l, r) in enumerate(windows):
        if l == r:
            assert np.all(coeffs[:, k] == 0.0)
            continue
        for n, e in O.level_errors(coeffs[:, k], ref[:, k], lengths).items():
            assert e <= FWD_TOL, f"window {k} level {n}: {e:.3e}"
    gref = O.backward_windows(X, W, windows, G.astype(np.float64))
    assert O.grad_errors(gp, gref).max() <= BWD_TOL


@pytest.mark.parametrize("d,depth,B,L", [(2, 6, 7, 20), (3, 4, 66, 15), (4, 5, 3, 9), (5, 1, 2, 4), (4, 6, 5, 33)])
def test_log_signature(d, depth, B, L):
    """Log-signature in Lyndon-word coordinates: signature on the reduced word set, then the tensor logarithm word by
    word, against the oracle's dense tensor logarithm of the full truncated signature."""
    import torch
    ws = S.sig_wordset_build_logsig(d, depth)
    ws.upload("cuda:0")
    X = make_path("iid", 500 + d, B, L, d)
    xp = torch.from_numpy(X).cuda()
    coeffs = S.sig_forward(ws, xp)
    lg = S.sig_logsig_forward(ws, coeffs).cpu().numpy()
    ref = O.logsig_from_path(X, depth)
    lyn = O.lyndon_words(d, depth)
    assert lg.shape == ref.shape == (B, len(lyn))
    lengths = np.array([len(w) for w in lyn])
    for n, e in O.level_errors(lg, ref, lengths).items():
        assert e <= FWD_TOL, f"log-signature level {n}: {e:.3e}"


@pytest.mark.parametrize("two_kernels", [False, True])
def test_log_signature_gradient(monkeypatch, two_kernels):
    """d <G, logsig(X)> / dX through sig_logsig_backward and sig_backward against central differences of the oracle;
    sig_logsig_backward in its one-kernel form (gradient row summed in LDS) and in the form for rows that do not fit
    there (contributions written out, then gathered per word)."""
    import torch
    if two_kernels:
        monkeypatch.setenv("SIG_LOGSIG_GATHER", "1")
    else:
        monkeypatch.delenv("SIG_LOGSIG_GATHER", raising=False)
    d, depth, B, L = 3, 4, 2, 5
    ws = S.sig_wordset_build_logsig(d, depth)
    ws.upload("cuda:0")
    # points on a grid of 2^-6, so that X +- h is exact in fp32 (the oracle consumes fp32 paths)
    X = (np.round(make_path("iid", 510, B, L, d) * 64.0) / 64.0).astype(np.float32)
    G = np.random.default_rng(511).standard_normal((B, int(S.load_library().sig_wordset_n_lyndon(ws._h)))).astype(np.float32)
    xp = torch.from_numpy(X).cuda()
    coeffs = S.sig_forward(ws, xp)
    gc = S.sig_logsig_backward(ws, coeffs, torch.from_numpy(G).cuda())
    gp = S.sig_backward(ws, xp, coeffs, gc).cpu().numpy()
    Xd = X.astype(np.float64)
    fun = lambda Y: float((O.logsig_from_path(Y, depth) * G).sum())
    num = np.zeros_like(Xd)
    h = 2.0 ** -10
    for idx in np.ndindex(*Xd.shape):
        Yp, Ym = Xd.copy(), Xd.copy()
        Yp[idx] += h
        Ym[idx] -= h
        num[idx] = (fun(Yp) - fun(Ym)) / (2 * h)
    assert O.grad_errors(gp, num).max() <= BWD_TOL


@pytest.mark.parametrize("kind,d,depth,B,L", [("truncated", 4, 6, 9, 70), ("truncated", 8, 5, 2, 24), ("words", 5, 4, 70, 19),
                                              ("truncated", 6, 4, 5, 31)])
def test_step_captured_in_a_graph(kind, d, depth, B, L):
    """Forward + backward recorded into a HIP graph (the library enqueues kernels only: no allocation, no memset) and
    replayed on new inputs, with eager calls and synchronisations between the replays; every replay must reproduce
    the eager results, and the first one the oracle's."""
    import torch
    from sig_workloads import random_prefix_closed_words
    words = random_prefix_closed_words(1699, d, 200, depth) if kind == "words" else None
    ws, W = build_both(kind, d, depth=depth, words=words)
    lib = S.load_library()
    X0 = make_path("iid", 1700, B, L, d)
    G0 = make_grad_coeffs(1701, B, ws.size)
    xp = torch.from_numpy(X0).cuda()
    grad = torch.from_numpy(G0).cuda()
    coeffs = torch.empty((B, ws.size), dtype=torch.float32, device="cuda")
    gpath = torch.empty((B, L + 1, d), dtype=torch.float32, device="cuda")
    wf = torch.empty(max(int(lib.sig_forward_workspace_bytes(ws._h, B, L + 1)), 256), dtype=torch.uint8, device="cuda")
    wb = torch.empty(max(int(lib.sig_backward_workspace_bytes(ws._h, B, L + 1)), 256), dtype=torch.uint8, device="cuda")

    def step():
        S.sig_forward(ws, xp, out=coeffs, workspace=wf)
        S.sig_backward(ws, xp, coeffs, grad, out=gpath, workspace=wb)

    step()                                   # compiles / sets kernel attributes outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    lengths = np.array([len(w) for w in W])
    for rep in range(3):
        X = make_path("iid", 1710 + rep, B, L, d)
        G = make_grad_coeffs(1720 + rep, B, ws.size)
        xp.copy_(torch.from_numpy(X).cuda())
        grad.copy_(torch.from_numpy(G).cuda())
        coeffs.zero_()
        gpath.zero_()
        graph.replay()
        torch.cuda.synchronize()
        c_graph, g_graph = coeffs.cpu().numpy(), gpath.cpu().numpy()
        c_eager = S.sig_forward(ws, xp)
        g_eager = S.sig_backward(ws, xp, c_eager, grad)
        torch.cuda.synchronize()
        assert np.array_equal(c_graph, c_eager.cpu().numpy()), f"replay {rep}: forward differs from the eager call"
        assert O.grad_errors(g_graph, g_eager.cpu().numpy().astype(np.float64)).max() <= 1e-5, f"replay {rep}"
        if rep == 0:
            for n, e in O.level_errors(c_graph, O.forward_words(X, W), lengths).items():
                assert e <= FWD_TOL, (n, e)
            assert O.grad_errors(g_graph, O.backward_words(X, W, G.astype(np.float64))).max() <= BWD_TOL


@pytest.mark.parametrize("kind,d,depth,B,L", [("anisotropic", 3, None, 5, 200), ("anisotropic", 3, None, 3, 130), ("truncated", 8, 5, 2, 200)])
def test_checkpointed_step_captured_in_a_graph(kind, d, depth, B, L):
    """The pair of calls that keeps the time-chunk signatures, recorded into a HIP graph with its checkpoint and
    workspaces (kernels only: the clearing is a kernel, the products and boundary adjoints are kernels) and replayed
    on new inputs with eager work between the replays."""
    import torch
    ws, W = build_both(kind, d, depth=depth, weights=(1.0, 1.25, 1.5), cutoff=4.5)
    if kind == "anisotropic":
        ws.set_option("ckpt_chunks", 3 if L >= 192 else 2)
    lib = S.load_library()
    nck = int(lib.sig_checkpoint_bytes(ws._h, B, L + 1))
    assert nck > 0
    xp = torch.from_numpy(make_path("iid", 1800, B, L, d)).cuda()
    grad = torch.from_numpy(make_grad_coeffs(1801, B, ws.size)).cuda()
    coeffs = torch.empty((B, ws.size), dtype=torch.float32, device="cuda")
    gpath = torch.empty((B, L + 1, d), dtype=torch.float32, device="cuda")
    ck = torch.empty(nck, dtype=torch.uint8, device="cuda")
    wf = torch.empty(max(int(lib.sig_forward_checkpointed_workspace_bytes(ws._h, B, L + 1)), 256), dtype=torch.uint8, device="cuda")
    wb = torch.empty(max(int(lib.sig_backward_checkpointed_workspace_bytes(ws._h, B, L + 1)), 256), dtype=torch.uint8, device="cuda")

    def step():
        S.sig_forward_checkpointed(ws, xp, out=coeffs, checkpoint=ck, workspace=wf)
        S.sig_backward_checkpointed(ws, xp, coeffs, grad, ck, out=gpath, workspace=wb)

    step()                                   # compiles / sets kernel attributes outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    lengths = np.array([len(w) for w in W])
    for rep in range(3):
        X = make_path("iid", 1810 + rep, B, L, d)
        G = make_grad_coeffs(1820 + rep, B, ws.size)
        xp.copy_(torch.from_numpy(X).cuda())
        grad.copy_(torch.from_numpy(G).cuda())
        coeffs.zero_()
        gpath.fill_(7.0)
        ck.zero_()
        graph.replay()
        torch.cuda.synchronize()
        c_graph, g_graph = coeffs.cpu().numpy(), gpath.cpu().numpy()
        c_eager, ck_eager = S.sig_forward_checkpointed(ws, xp)
        g_eager = S.sig_backward_checkpointed(ws, xp, c_eager, grad, ck_eager)
        torch.cuda.synchronize()
        assert np.array_equal(c_graph, c_eager.cpu().numpy()), f"replay {rep}: forward differs from the eager call"
        assert O.grad_errors(g_graph, g_eager.cpu().numpy().astype(np.float64)).max() <= 1e-5, f"replay {rep}"
        if rep == 0:
            ref = O.forward_dense(X, depth) if kind == "truncated" else O.forward_words(X, W)
            for n, e in O.level_errors(c_graph, ref, lengths).items():
                assert e <= FWD_TOL, (n, e)
            gref = O.backward_dense(X, depth, G.astype(np.float64)) if kind == "truncated" else O.backward_words(X, W, G.astype(np.float64))
            assert O.grad_errors(g_graph, gref).max() <= BWD_TOL


def test_code_object_from_the_disk_cache_runs(tmp_path, monkeypatch):
    """A kernel loaded from SIG_JIT_CACHE instead of compiled gives the results of the compiled one, bit for bit."""
    import torch
    monkeypatch.setenv("SIG_JIT_CACHE", str(tmp_path))
    words = random_prefix_closed_words(77, 5, 150, 4)
    X = torch.from_numpy(make_path("iid", 78, 9, 23, 5)).cuda()
    res = []
    for _ in range(2):
        ws = S.sig_wordset_build(5, words)
        ws.upload("cuda:0")
        G = torch.from_numpy(make_grad_coeffs(79, 9, ws.size)).cuda()
        c = S.sig_forward(ws, X)
        g = S.sig_backward(ws, X, c, G)
        res.append((c.cpu().numpy(), g.cpu().numpy()))
    import os
    assert len(os.listdir(tmp_path)) == 2                         # forward and backward kernel, written once
    assert np.array_equal(res[0][0], res[1][0])
    np.testing.assert_allclose(res[0][1], res[1][1], rtol=1e-5, atol=1e-6)      # atomics: order of additions
    ws2, W = build_both("words", 5, words=words)
    check_parity(ws2, W, "words", None, make_path("iid", 78, 9, 23, 5), make_grad_coeffs(79, 9, ws2.size), what="cached kernels")


def test_one_point_paths_give_zero():
    import torch
    ws, W = build_both("truncated", 3, depth=3)
    X = np.random.default_rng(0).standard_normal((5, 1, 3)).astype(np.float32)
    G = make_grad_coeffs(1, 5, ws.size)
    coeffs, gp = gpu_forward_backward(ws, X, G)
    assert coeffs.shape == (5, ws.size) and np.all(coeffs == 0.0)
    assert gp.shape == (5, 1, 3) and np.all(gp == 0.0)


def test_empty_batch_is_a_noop():
    import torch
    ws, W = build_both("truncated", 3, depth=3)
    xp = torch.zeros((0, 4, 3), dtype=torch.float32, device="cuda")
    out = S.sig_forward(ws, xp)
    assert tuple(out.shape) == (0, ws.size)
    gp = S.sig_backward(ws, xp, out, out.clone())
    assert tuple(gp.shape) == (0, 4, 3)
    torch.cuda.synchronize()


def test_repeated_points_change_nothing():
    ws, W = build_both("truncated", 3, depth=4)
    X = make_path("iid", 5, 4, 12, 3)
    Xr = np.ascontiguousarray(np.insert(X, 6, X[:, 6], axis=1))
    a, _ = gpu_forward_backward(ws, X, None)
    b, _ = gpu_forward_backward(ws, Xr, None)
    assert np.array_equal(a, b)        # exp(0) = 1: the extra segment adds exact zeros


def test_forward_is_deterministic_and_outputs_fully_overwritten():
    import torch
    wl = WORKLOADS["c1"]
    ws, W = build_for_workload(wl)
    X = workload_path(wl)
    xp = torch.from_numpy(X).cuda()
    out1 = torch.full((wl.B, ws.size), float("nan"), device="cuda")
    S.sig_forward(ws, xp, out=out1)
    out2 = S.sig_forward(ws, xp)
    torch.cuda.synchronize()
    assert torch.equal(out1, out2)
    g = torch.from_numpy(make_grad_coeffs(wl.seed, wl.B, ws.size)).cuda()
    gp = torch.full((wl.B, wl.L + 1, wl.d), float("nan"), device="cuda")
    S.sig_backward(ws, xp, out1, g, out=gp)
    torch.cuda.synchronize()
    assert torch.isfinite(gp).all()


def test_gradient_against_finite_differences_of_the_oracle_forward():
    # the benchmark spec of the gradient tolerance: fp64 central differences, 1e-3 relative
    wl = WORKLOADS["c1"]
    ws, W = build_for_workload(wl)
    B = 4
    X = workload_path(wl)[:B].astype(np.float64)
    X = np.round(X * 128) / 128                      # +-2^-12 steps stay exact in fp32
    G = make_grad_coeffs(wl.seed, B, ws.size)
    _, gp = gpu_forward_backward(ws, X.astype(np.float32), G)
    h = 2.0 ** -12
    rng = np.random.default_rng(0)
    fun = lambda Y: (O.forward_dense(Y.astype(np.float32), wl.depth) * G.astype(np.float64)).sum(axis=1)
    for _ in range(6):
        V = np.sign(rng.standard_normal(X.shape))    # +-1 directions keep the perturbed points on the grid
        num = (fun(X + h * V) - fun(X - h * V)) / (2 * h)
        ana = (gp.astype(np.float64) * V).reshape(B, -1).sum(axis=1)
        scale = np.abs(gp).reshape(B, -1).sum(axis=1)
        assert np.all(np.abs(num - ana) <= 1e-3 * scale)


def test_projection_equals_gather_of_truncation():
    # a word-projected coefficient is the same number as that word's coefficient in the full truncation
    d, depth = 4, 5
    words = random_prefix_closed_words(9, d, 200, depth)
    wsp, Wp = build_both("words", d, words=words)
    wst, Wt = build_both("truncated", d, depth=depth)
    X = make_path("iid", 77, 20, 30, d)
    a, _ = gpu_forward_backward(wsp, X, None)
    b, _ = gpu_forward_backward(wst, X, None)
    index = {w: k for k, w in enumerate(Wt)}
    pick = np.array([index[w] for w in Wp])
    ref = O.forward_dense(X, depth)[:, pick]
    lengths = np.array([len(w) for w in Wp])
    assert max(O.level_errors(a, ref, lengths).values()) <= FWD_TOL
    np.testing.assert_allclose(a, b[:, pick], rtol=2e-5, atol=1e-7)
    assert np.array_equal(wsp.user_index, np.array([{w: k for k, w in enumerate(Wp)}[w] for w in words]))


# full-size workloads in the launch configuration the benchmark times; the oracle is run on a sample
# of paths (paths are independent, so a sampled path is checked exactly as in a full comparison)
FULL = {
    "c1": None,                       # all 32 paths
    "c2": [0, 1, 63, 64, 127, 128, 200, 255],
    "c3": [0, 63, 64, 127],
    "c4a": [0, 63, 64, 300, 511],
    "c4b": [0, 63, 64, 300, 511],
    "c5": [0, 63],
}


# (name, checkpointed): the benchmark times the checkpointed pair of calls where the library offers it (c3, c4a, c5)
# and the plain pair beside it
@pytest.mark.parametrize("name,checkpointed", [(n, False) for n in FULL] + [("c3", True), ("c4a", True), ("c5", True)])
def test_full_size_workloads(name, checkpointed):
    wl = WORKLOADS[name]
    ws, W = build_for_workload(wl)
    if checkpointed:
        assert S.load_library().sig_checkpoint_bytes(ws._h, wl.B, wl.L + 1) > 0
    X = workload_path(wl)
    G = make_grad_coeffs(wl.seed, wl.B, ws.size)
    if name == "c5":
        O.set_threads(2)              # the oracle's backward keeps every intermediate signature: 2.3 GB per path
    try:
        errs, gerr = check_parity(ws, W, wl.kind, wl.depth, X, G, sample=FULL[name], what=name, checkpointed=checkpointed)
    finally:
        O.set_threads(16)
    print(f"{name}: forward level errors {errs}; gradient error max {gerr.max():.3e}")
