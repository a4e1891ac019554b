"""Host-side checks of the C-ABI library: exported symbols, word-set tables (bit-exact against the
oracle's independent Python builder and the closed forms of Appendix A), error codes, and the launch
plans (every word owned once; an fp64 model of the unit programs reproduces the oracle)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2602_24066_amd as S
from oracle import sig_oracle as O
from sig_workloads import make_path, random_prefix_closed_words
from tests import plan_model

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(sig_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(S.lib_path())
    names = declared_functions()
    assert len(names) >= 25
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/*.h but not exported"


def test_compiled_kernels_are_checked_against_their_launch_shape():
    """What a loaded code object declares decides whether it may be dispatched (the check of jit_load)."""
    ok = S.load_library().sig_jit_launch_shape_ok
    assert ok(4, 256, 62 * 1024, 153) == 1              # the shapes in use: four wavefronts, static LDS under 64 KB
    assert ok(4, 256, 64 * 1024, 256) == 1
    assert ok(8, 512, 112128, 146) == 0                 # eight wavefronts with 112 KB of static LDS: the rejected dispatch
    assert ok(4, 256, 64 * 1024 + 4, 100) == 0
    assert ok(8, 256, 32 * 1024, 100) == 0              # more threads than the kernel declares
    assert ok(8, 1024, 32 * 1024, 256) == 1 and ok(8, 1024, 32 * 1024, 257) == 0   # two wavefronts share a SIMD's 512 registers
    assert ok(0, 256, 0, 10) == 0


def test_boundary_from_plain_c(tmp_path):
    """include/sig.h is a C header: a C99 program compiled with gcc links against the library and calls it."""
    import shutil, subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    here = os.path.dirname(os.path.abspath(__file__))
    root = os.path.dirname(here)
    lib = S.lib_path()
    exe = str(tmp_path / "abi_smoke")
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(root, "include"),
                    os.path.join(here, "c_abi", "abi_smoke.c"), "-o", exe, lib, "-Wl,-rpath," + os.path.dirname(lib)], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split("\n")
    assert out[0].split() == ["120", "3", "4", str(S.sig_wordset_build_truncated(3, 4).min_fma_per_step)]
    assert out[1].startswith("-1 ")


def test_strerror_and_version():
    lib = S.load_library()
    assert lib.sig_strerror(0) == b"success"
    for code in range(-9, 0):
        assert lib.sig_strerror(code) not in (b"", b"unknown error")
    assert lib.sig_strerror(-99) == b"unknown error"
    assert b"sig" in lib.sig_version()


@pytest.mark.parametrize("d,N", [(1, 5), (2, 4), (3, 4), (4, 6), (6, 3), (8, 5), (16, 4)])
def test_truncated_tables_bit_exact(d, N):
    ws = S.sig_wordset_build_truncated(d, N)
    assert ws.size == sum(d ** n for n in range(1, N + 1))
    assert ws.dim == d and ws.max_len == N
    # closed forms of Appendix A
    ls = [0, 0]
    for n in range(1, N + 1):
        ls.append(ls[-1] + d ** n)
    assert list(ws.level_start) == ls
    par, let = ws.parent, ws.letter
    for n in range(1, N + 1):
        phi = np.arange(d ** n)
        assert np.array_equal(let[ls[n]:ls[n + 1]], phi % d)
        if n == 1:
            assert np.all(par[ls[1]:ls[2]] == -1)
        else:
            assert np.array_equal(par[ls[n]:ls[n + 1]], ls[n - 1] + phi // d)
    if ws.size < 50000:
        t = O.word_tables(O.truncated_words(d, N))
        assert np.array_equal(par, t["parent"]) and np.array_equal(let, t["letter"])
        assert np.array_equal(ws.level_start, t["level_start"])
    assert ws.min_fma_per_step == sum(d ** k for n in range(1, N + 1) for k in range(1, n + 1))


def test_paper_sizes():
    for d, N, size in [(6, 2, 42), (6, 3, 258), (6, 4, 1554), (6, 5, 9330), (6, 6, 55986), (4, 6, 5460),
                       (10, 4, 11110), (8, 3, 584), (8, 6, 299592)]:
        assert S.sig_wordset_build_truncated(d, N).size == size


@pytest.mark.parametrize("d,gam,r", [(3, (1.0, 2.0, 1.5), 4.0), (6, (1, 1, 2, 2, 3, 3), 8.0), (2, (0.3, 0.7), 2.0),
                                     (4, (1, 1, 1, 1), 3.0)])
def test_anisotropic_tables_bit_exact(d, gam, r):
    ws = S.sig_wordset_build_anisotropic(d, gam, r)
    W = O.anisotropic_words(d, gam, r)
    t = O.word_tables(W)
    assert ws.size == len(W)
    assert np.array_equal(ws.parent, t["parent"])
    assert np.array_equal(ws.letter, t["letter"])
    assert np.array_equal(ws.level_start, t["level_start"])


def test_anisotropic_unit_weights_is_truncation():
    a = S.sig_wordset_build_anisotropic(3, (1.0, 1.0, 1.0), 4.0)
    b = S.sig_wordset_build_truncated(3, 4)
    assert np.array_equal(a.parent, b.parent) and np.array_equal(a.letter, b.letter)
    assert np.array_equal(a.level_start, b.level_start)
    assert S.sig_wordset_build_anisotropic(6, (1, 1, 2, 2, 3, 3), 8.0).size == 5754


@pytest.mark.parametrize("seed,d,n,maxlen", [(0, 3, 50, 4), (1, 10, 2000, 6), (2, 2, 30, 7), (3, 5, 1, 1)])
def test_list_tables_bit_exact(seed, d, n, maxlen):
    words = random_prefix_closed_words(seed, d, n, maxlen)
    # hand over a sparse, shuffled subset with duplicates: the builder must close and sort it
    rng = np.random.default_rng(seed)
    pick = [words[i] for i in rng.permutation(len(words))[: max(1, len(words) // 2)]]
    pick = pick + pick[:3]
    ws = S.sig_wordset_build(d, pick)
    C = O.prefix_closure(pick)
    t = O.word_tables(C, pick)
    assert ws.size == len(C)
    assert np.array_equal(ws.parent, t["parent"])
    assert np.array_equal(ws.letter, t["letter"])
    assert np.array_equal(ws.level_start, t["level_start"])
    assert np.array_equal(ws.user_index, t["user_index"])
    # structural properties: parents precede children; parent/letter chain spells the word
    par, let = ws.parent, ws.letter
    assert np.all(par < np.arange(ws.size))
    for k in rng.integers(0, ws.size, size=min(ws.size, 50)):
        rec, q = [], int(k)
        while q != -1:
            rec.append(int(let[q]))
            q = int(par[q])
        assert tuple(reversed(rec)) == C[int(k)]


def test_error_codes():
    lib = S.load_library()
    h = ctypes.c_void_p()
    B = ctypes.byref(h)
    assert lib.sig_wordset_build_truncated(0, 3, B) == -1
    assert lib.sig_wordset_build_truncated(3, 0, B) == -1
    assert lib.sig_wordset_build_truncated(3, 3, None) == -1
    assert lib.sig_wordset_build_truncated(2, 40, B) == -7
    assert lib.sig_wordset_build_truncated(10, 12, B) == -7          # 10^12 words
    w = np.array([1.0, 0.0], dtype=np.float64)
    assert lib.sig_wordset_build_anisotropic(2, w.ctypes.data, 3.0, B) == -1      # weight must be > 0
    w = np.array([1.0, -1.0], dtype=np.float64)
    assert lib.sig_wordset_build_anisotropic(2, w.ctypes.data, 3.0, B) == -1
    w = np.array([1.0, 2.0], dtype=np.float64)
    assert lib.sig_wordset_build_anisotropic(2, None, 3.0, B) == -1
    assert lib.sig_wordset_build_anisotropic(2, w.ctypes.data, float("nan"), B) == -1
    assert lib.sig_wordset_build_anisotropic(2, w.ctypes.data, 0.5, B) == -3      # nothing admissible
    assert lib.sig_wordset_build_anisotropic(2, w.ctypes.data, 100.0, B) == -7    # words longer than the format allows
    letters = np.array([0, 1, 5], dtype=np.int32)
    offs = np.array([0, 2, 3], dtype=np.int64)
    assert lib.sig_wordset_build(3, letters.ctypes.data, offs.ctypes.data, 2, B) == -2   # letter 5 >= d
    letters = np.array([0, 1, 2], dtype=np.int32)
    offs = np.array([0, 2, 2, 3], dtype=np.int64)
    assert lib.sig_wordset_build(3, letters.ctypes.data, offs.ctypes.data, 3, B) == -3   # empty word
    offs = np.array([0, 2, 1], dtype=np.int64)
    assert lib.sig_wordset_build(3, letters.ctypes.data, offs.ctypes.data, 2, B) == -1   # decreasing offsets
    offs = np.array([1, 2, 3], dtype=np.int64)
    assert lib.sig_wordset_build(3, letters.ctypes.data, offs.ctypes.data, 2, B) == -1   # offsets[0] != 0
    assert lib.sig_wordset_build(3, letters.ctypes.data, offs.ctypes.data, 0, B) == -3   # empty list
    assert lib.sig_wordset_build(3, letters.ctypes.data, None, 2, B) == -1
    assert h.value is None
    # forward / backward argument checks that need no device
    ws = S.sig_wordset_build_truncated(2, 3)
    assert lib.sig_forward(None, None, 1, 2, None, None, 0, None) == -1
    assert lib.sig_forward(ws._h, None, 1, 2, None, None, 0, None) == -1
    assert lib.sig_forward(ws._h, ctypes.c_void_p(256), -1, 2, None, None, 0, None) == -1
    assert lib.sig_forward(ws._h, ctypes.c_void_p(256), 1, 0, None, None, 0, None) == -1
    assert lib.sig_forward(ws._h, ctypes.c_void_p(256), 1, 2, ctypes.c_void_p(256), None, 0, None) == -8   # not uploaded
    assert lib.sig_wordset_upload(ws._h, None, 0, None) == -1
    assert lib.sig_wordset_upload(ws._h, ctypes.c_void_p(256), 1, None) == -5
    assert lib.sig_wordset_upload(ws._h, ctypes.c_void_p(260), 1 << 20, None) == -1                        # misaligned
    deep = S.sig_wordset_build_truncated(2, 14)
    assert lib.sig_forward(deep._h, ctypes.c_void_p(256), 1, 2, ctypes.c_void_p(256), None, 0, None) == -9
    gdx = 4 * 10 * 2 * 4 + (-(4 * 10 * 2 * 4)) % 256          # dLoss/d dX: B * L * d floats, rounded up to 256 bytes
    ws.set_option("no_jit", 1)
    assert ws.get_option("no_jit") == 1
    assert lib.sig_backward_workspace_bytes(ws._h, 4, 11) == gdx
    assert lib.sig_forward_workspace_bytes(ws._h, 4, 11) == 0
    ws.set_option("no_jit", 0)
    assert lib.sig_wordset_set_option(ws._h, b"no_such_knob", 1) == -1
    assert lib.sig_wordset_set_option(None, b"no_jit", 1) == -1
    # the entry point that allocates nothing: same argument checks, before anything touches a device
    assert lib.sig_backward_static(None, None, None, None, 1, 2, None, None) == -1
    assert lib.sig_backward_static(ws._h, ctypes.c_void_p(256), ctypes.c_void_p(256), ctypes.c_void_p(256), 1, 2,
                                   ctypes.c_void_p(256), None) == -8                                        # not uploaded
    # with run-time specialisation: the transposed increments in addition (padded to whole tiles of segments)
    nb = lib.sig_backward_workspace_bytes(ws._h, 4, 11)
    nf = lib.sig_forward_workspace_bytes(ws._h, 4, 11)
    assert nf > 0 and nf % 256 == 0 and nb % 256 == 0 and nb >= gdx + 4 * 10 * 2 * 64
    assert lib.sig_backward_workspace_bytes(ws._h, 4, 1) == 0
    lib.sig_wordset_free(None)


def _sets():
    yield "trunc(2,4)", S.sig_wordset_build_truncated(2, 4), O.truncated_words(2, 4), 2
    yield "trunc(4,5)", S.sig_wordset_build_truncated(4, 5), O.truncated_words(4, 5), 4
    yield "aniso", S.sig_wordset_build_anisotropic(3, (1.0, 2.0, 1.5), 6.0), O.anisotropic_words(3, (1.0, 2.0, 1.5), 6.0), 3
    words = random_prefix_closed_words(5, 5, 700, 6)
    yield "random", S.sig_wordset_build(5, words), O.prefix_closure(words), 5


def _all_plans(ws, backward):
    """Static variants (table-driven kernels) and balanced plans (specialised kernels) for several batch sizes."""
    for v in range(ws.plan_count(backward)):
        yield f"v{v}", ws.plan(backward, v), (56 if backward else 112)
    for B in (1, 64, 512, 5000, 200000):
        yield f"balanced B={B}", ws.jit_plan(backward, B), (160 if backward else 320)


@pytest.mark.parametrize("backward", [False, True])
def test_plans_cover_every_word_exactly_once(backward):
    for name, ws, W, d in _sets():
        for v, p, slot_limit in _all_plans(ws, backward):
            owned = p["slot_word"][p["slot_word"] >= 0]
            assert np.array_equal(np.sort(owned), np.arange(ws.size)), (name, v)
            # programs: slots = number of non-LEAVE ops; ENTER/LEAVE balanced; levels consistent with the tables
            for (op_off, n_ops, slot_off, n_slots) in p["units"]:
                prog = [plan_model.decode(o) for o in p["ops"][op_off:op_off + n_ops]]
                sw = p["slot_word"][slot_off:slot_off + n_slots]
                assert sum(1 for o in prog if o[3] != plan_model.LEAVE) == n_slots
                assert n_slots <= slot_limit
                r, stack = 0, []
                for letter, level, h, kind in prog:
                    if kind == plan_model.LEAVE:
                        assert backward and stack and stack[-1] == (letter, level, h)
                        stack.pop()
                        continue
                    w = int(sw[r]); w = w if w >= 0 else ~w
                    assert W[w][-1] == letter and len(W[w]) == level
                    if not backward:
                        stack = stack[: level - 1]      # without LEAVE ops the open chain is implied by the levels
                    assert len(stack) == level - 1          # parent chain is open
                    if level > 1:
                        assert stack[-1][2] >= h + 1        # the parent carries one more target length
                    if kind == plan_model.ENTER:
                        assert h >= 1
                        stack.append((letter, level, h))
                    else:
                        assert h == 0
                    r += 1
                if backward:
                    assert not stack


def test_plan_model_forward_matches_oracle():
    for name, ws, W, d in _sets():
        X = make_path("iid", 3, 3, 9, d)
        ref = O.forward_words(X, W)
        for v, p, _ in _all_plans(ws, False):
            out, written = plan_model.forward(p, X, ws.size)
            assert np.all(written == 1)
            np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-14, err_msg=f"{name} {v}")


def test_plan_model_backward_matches_oracle():
    for name, ws, W, d in _sets():
        X = make_path("iid", 4, 2, 7, d)
        G = np.random.default_rng(0).standard_normal((2, ws.size))
        coeffs = O.forward_words(X, W)
        ref = O.backward_words(X, W, G)
        for v, p, _ in _all_plans(ws, True):
            gp = plan_model.backward(p, X, coeffs, G)
            np.testing.assert_allclose(gp, ref, rtol=1e-9, atol=1e-11, err_msg=f"{name} {v}")


def test_fma_counts():
    for d, N, fmin in [(4, 6, 7272), (8, 5, 42792), (16, 4, 74560), (2, 4, 52)]:
        assert S.sig_wordset_build_truncated(d, N).min_fma_per_step == fmin
    assert S.sig_wordset_build_anisotropic(6, (1, 1, 2, 2, 3, 3), 8.0).min_fma_per_step == 8742
    ws = S.sig_wordset_build_truncated(4, 6)
    for v, p, _ in _all_plans(ws, False):
        assert p["fma_per_step"] == sum(plan_model.decode(o)[2] + 1 for o in p["ops"])
        assert p["fma_per_step"] >= ws.min_fma_per_step


def test_balanced_plans_are_balanced():
    """Units of a balanced plan have nearly equal cost: no unit is cheaper than the costliest one by more than one
    word's worth of multiply-adds plus the ancestor chain (the last unit takes what is left)."""
    ws = S.sig_wordset_build_anisotropic(6, (1, 1, 2, 2, 3, 3), 8.0)
    p = ws.jit_plan(False, 512)
    cost = []
    for (op_off, n_ops, slot_off, n_slots) in p["units"]:
        cost.append(sum(plan_model.decode(o)[2] + 1 for o in p["ops"][op_off:op_off + n_ops]))
    cost = np.array(cost)
    assert 0.9 * len(cost) <= 4 * ((2048 // 8 + 3) // 4) and len(cost) <= 4 * ((2048 // 8 + 3) // 4)
    assert cost.max() - np.sort(cost)[1] <= 8 * 9 // 2 + 8
    assert p["fma_per_step"] <= 1.6 * ws.min_fma_per_step


def test_runtime_compilation_without_a_device():
    """hiprtc needs no GPU: the specialised kernels of a small word set compile, and the generated source holds one
    body per work unit of the balanced plan."""
    ws = S.sig_wordset_build(5, random_prefix_closed_words(9, 5, 200, 5))
    for backward in (False, True):
        plan = ws.jit_plan(backward, 128)
        src = ws.jit_source(backward, 128)
        name = "bwd_unit_" if backward else "fwd_unit_"
        assert src.count("void " + name) == len(plan["units"])
        assert ("sig_bwd_jit" if backward else "sig_fwd_jit") in src
        assert ws.jit_prepare(backward, 128) == 0
    full = S.sig_wordset_build_truncated(4, 6)                  # served by a precompiled kernel instead
    assert full.jit_prepare(False, 128) == -9
    # truncations of other shapes: one fixed source with the shape as macros, a word per lane; two levels below the
    # lane's word for large batches, one for small ones (more, shorter wavefronts) and for large alphabets
    for d, depth, B, levels in [(6, 5, 4096, 2), (6, 5, 32, 1), (10, 4, 4096, 2), (10, 4, 1, 1), (12, 3, 4096, 1),
                                (40, 3, 64, 1)]:
        ws = S.sig_wordset_build_truncated(d, depth)
        for backward in (False, True):
            src = ws.jit_source(backward, B)
            assert f"#define D {d}\n#define N {depth}\n#define R {levels}\n" in src
            assert ("sig_bwd_lanes" if backward else "sig_fwd_lanes") in src
            assert ws.jit_prepare(backward, B) == 0


def test_code_object_cache_on_disk(tmp_path, monkeypatch):
    """SIG_JIT_CACHE: the first compilation stores the code object, a fresh word-set object of the same set loads it
    (no compiler run: the log says where it came from); another word set gets another file."""
    import time
    monkeypatch.setenv("SIG_JIT_CACHE", str(tmp_path))
    lib = S.load_library()
    words = random_prefix_closed_words(31, 4, 120, 5)
    a = S.sig_wordset_build(4, words)
    assert a.jit_prepare(False, 64) == 0
    files = sorted(os.listdir(tmp_path))
    assert len(files) == 1 and files[0].startswith("sig_gfx950_") and files[0].endswith(".hsaco")
    stamp = os.path.getmtime(os.path.join(tmp_path, files[0]))
    b = S.sig_wordset_build(4, words)
    t0 = time.perf_counter()
    assert b.jit_prepare(False, 64) == 0
    assert time.perf_counter() - t0 < 0.2
    assert sorted(os.listdir(tmp_path)) == files and os.path.getmtime(os.path.join(tmp_path, files[0])) == stamp
    assert a.jit_prepare(True, 64) == 0                           # the backward kernel: a second file
    assert len(os.listdir(tmp_path)) == 2
    c = S.sig_wordset_build_truncated(6, 4)                       # word-per-lane source of another shape: a third
    assert c.jit_prepare(False, 8) == 0
    assert len(os.listdir(tmp_path)) == 3
    # a directory that does not exist: compilation still succeeds, nothing is written
    monkeypatch.setenv("SIG_JIT_CACHE", str(tmp_path / "missing"))
    d = S.sig_wordset_build(4, words)
    assert d.jit_prepare(False, 64) == 0
    assert not os.path.exists(tmp_path / "missing")
    del lib


def test_time_chunk_workspace():
    """Few long paths of a full truncation are cut into time chunks: the forward workspace holds the chunk
    signatures (and the partial products when four or more signatures too large for LDS are multiplied pair by pair);
    many paths, or short ones, need none."""
    lib = S.load_library()
    ws = S.sig_wordset_build_truncated(4, 6)
    rows = 2 * 4                                               # B = 2 paths, L = 1024 -> 4 chunks of 256 segments
    per_array = (4 * rows * ws.size + 255) // 256 * 256
    assert lib.sig_forward_workspace_bytes(ws._h, 2, 1025) == per_array
    ws85 = S.sig_wordset_build_truncated(8, 5)
    per85 = (4 * 2 * 4 * ws85.size + 255) // 256 * 256        # 2 paths, 4 chunks of 256 segments
    assert lib.sig_forward_workspace_bytes(ws85._h, 2, 1025) == 2 * per85
    assert lib.sig_forward_workspace_bytes(ws85._h, 128, 1025) == (4 * 128 * 2 * ws85.size + 255) // 256 * 256   # two chunks
    # checkpointed form: offered where the backward kernel of the shape would leave SIMDs with a single wavefront
    assert lib.sig_checkpoint_bytes(ws85._h, 128, 1025) == (4 * 128 * 2 * ws85.size + 255) // 256 * 256
    assert lib.sig_checkpoint_bytes(ws85._h, 1024, 1025) == 0 and lib.sig_checkpoint_bytes(ws85._h, 128, 100) == 0
    assert lib.sig_checkpoint_bytes(ws._h, 2, 1025) == 0
    # its backward workspace: increment gradients and one boundary adjoint per chunk but the last
    gdx85 = (4 * 128 * 1024 * 8 + 255) // 256 * 256
    assert lib.sig_backward_checkpointed_workspace_bytes(ws85._h, 128, 1025) == gdx85 + (4 * 128 * 1 * ws85.size + 255) // 256 * 256
    assert lib.sig_backward_checkpointed_workspace_bytes(ws._h, 2, 1025) == lib.sig_backward_workspace_bytes(ws._h, 2, 1025)
    assert lib.sig_forward_workspace_bytes(ws._h, 2, 300) == 0
    assert lib.sig_forward_workspace_bytes(ws._h, 4096, 1025) == 0
    gdx = (4 * 2 * 1024 * 4 + 255) // 256 * 256
    assert lib.sig_backward_workspace_bytes(ws._h, 2, 1025) == gdx       # backward is not chunked by itself


def _no_repeat_words(d, n):
    """Words of up to n letters in which no letter follows itself: closed under prefixes and suffixes."""
    out, level = [], [(i,) for i in range(d)]
    for _ in range(n):
        out += level
        level = [w + (i,) for w in level for i in range(d) if i != w[-1]]
    return out


@pytest.mark.parametrize("case", ["anisotropic", "anisotropic-c4", "no-repeat list", "random list", "truncation"])
def test_suffix_tables(case):
    """Sets closed under suffixes carry, for every word, the indices of the word without its first m letters; the
    table is checked against the words written out as tuples.  Sets that lack a suffix, and full truncations (which
    have product kernels of their own), carry none."""
    if case == "anisotropic":
        ws, words = S.sig_wordset_build_anisotropic(3, (1.0, 2.0, 1.5), 4.0), O.anisotropic_words(3, (1.0, 2.0, 1.5), 4.0)
    elif case == "anisotropic-c4":
        ws, words = S.sig_wordset_build_anisotropic(6, (1, 1, 2, 2, 3, 3), 8.0), O.anisotropic_words(6, (1, 1, 2, 2, 3, 3), 8.0)
    elif case == "no-repeat list":
        given = _no_repeat_words(3, 5)
        ws, words = S.sig_wordset_build(3, given), O.prefix_closure(given)
    elif case == "random list":
        given = random_prefix_closed_words(7, 4, 60, 5)
        ws, words = S.sig_wordset_build(4, given), O.prefix_closure(given)
        index = {tuple(w): k for k, w in enumerate(words)}
        assert any(tuple(w[1:]) not in index for w in words if len(w) > 1)      # the case is what it says
        assert not ws.suffix_closed and ws.tail_table() is None
        assert S.load_library().sig_checkpoint_bytes(ws._h, 64, 513) == 0
        return
    else:
        ws = S.sig_wordset_build_truncated(3, 4)
        assert not ws.suffix_closed and ws.tail_table() is None
        return
    assert ws.suffix_closed
    index = {tuple(w): k for k, w in enumerate(words)}
    tab, off = ws.tail_table()
    ls = ws.level_start
    seen = 0
    for k, w in enumerate(words):
        n = len(w)
        cnt = int(ls[n + 1] - ls[n])
        for m in range(1, n):
            assert tab[off[n] + (m - 1) * cnt + (k - ls[n])] == index[tuple(w[m:])]
            seen += 1
    assert seen == sum(len(w) - 1 for w in words) and seen > 0
    # the checkpointed calls offer time chunks for such a set: up to 2,048 rows, chunks of at least 256 segments (128 for few rows)
    lib = S.load_library()
    per_row = 4 * ws.size
    assert lib.sig_checkpoint_bytes(ws._h, 128, 513) == (per_row * 128 * 4 + 255) // 256 * 256
    assert lib.sig_checkpoint_bytes(ws._h, 512, 513) == (per_row * 512 * 2 + 255) // 256 * 256
    assert lib.sig_checkpoint_bytes(ws._h, 1024, 513) == (per_row * 1024 * 2 + 255) // 256 * 256
    assert lib.sig_checkpoint_bytes(ws._h, 2048, 513) == 0 and lib.sig_checkpoint_bytes(ws._h, 512, 101) == 0
    assert lib.sig_checkpoint_bytes(ws._h, 5, 201) == 0
    assert lib.sig_checkpoint_bytes(ws._h, 5, 257) == (per_row * 5 * 2 + 255) // 256 * 256
    assert lib.sig_checkpoint_chunks(ws._h, 5, 257) == 2 and lib.sig_checkpoint_chunks(ws._h, 2048, 513) == 1
    assert lib.sig_checkpoint_chunks(ws._h, 64, 4097) == 8 and lib.sig_checkpoint_chunks(ws._h, 128, 2049) == 8
    assert lib.sig_checkpoint_chunks(ws._h, 512, 2049) == 4 and lib.sig_checkpoint_chunks(ws._h, 256, 1025) == 4
    ws.set_option("ckpt_chunks", 3)
    assert lib.sig_checkpoint_chunks(ws._h, 5, 201) == 3 and lib.sig_checkpoint_chunks(ws._h, 5, 150) == 2
    ws.set_option("ckpt_chunks", 0)
    if case == "anisotropic":                                                  # the kernels of the B * C rows, ahead of time
        assert ws.jit_prepare(False, 5 * 2) == 0 and ws.jit_prepare(True, 5 * 2) == 0
    # sig_forward takes the same chunks with the chunk signatures in its workspace
    assert (lib.sig_forward_checkpointed_workspace_bytes(ws._h, 512, 513) + lib.sig_checkpoint_bytes(ws._h, 512, 513)
            >= lib.sig_forward_workspace_bytes(ws._h, 512, 513) > lib.sig_checkpoint_bytes(ws._h, 512, 513))
    assert lib.sig_backward_checkpointed_workspace_bytes(ws._h, 512, 513) >= lib.sig_backward_workspace_bytes(ws._h, 512, 513)
    ws.set_option("no_jit", 1)                                                 # the table-driven kernels take whole paths
    assert lib.sig_checkpoint_bytes(ws._h, 512, 513) == 0
    if case == "anisotropic-c4":
        # a suffix-closed set too large for three signatures in LDS (16,802 words) takes whole paths as well
        big = S.sig_wordset_build_anisotropic(6, (1, 1, 2, 2, 3, 3), 9.0)
        assert big.size == 16802 and big.suffix_closed and big.term_tables() is not None
        assert lib.sig_checkpoint_bytes(big._h, 64, 4097) == 0 and lib.sig_checkpoint_chunks(big._h, 64, 4097) == 1


@pytest.mark.parametrize("case", ["anisotropic", "no-repeat list"])
def test_term_tables_reproduce_chens_relation(case):
    """The term tables the chunk kernels read, applied in numpy to oracle signatures of two pieces of a path, give the
    oracle signature of the whole path (eq. 2 restricted to the set); the prefix-sorted copy of the terms gives the
    derivative of <g, a (x) q> with respect to a (Proposition 4.1 at a chunk boundary)."""
    if case == "anisotropic":
        d = 3
        ws, words = S.sig_wordset_build_anisotropic(d, (1.0, 1.25, 1.5), 4.5), O.anisotropic_words(d, (1.0, 1.25, 1.5), 4.5)
    else:
        d = 3
        given = _no_repeat_words(d, 5)
        ws, words = S.sig_wordset_build(d, given), O.prefix_closure(given)
    n = len(words)
    prod, adj, key = ws.term_tables()
    ls, (_, tail_off) = ws.level_start, ws.tail_table()
    lengths = ws.lengths
    assert len(adj) % 256 == 0 and (key[np.count_nonzero(key < n):] == n).all() and (np.diff(key.astype(np.int64)) >= 0).all()
    assert np.count_nonzero(key < n) == int((lengths - 1).sum())

    def product(a, b):
        out = a + b
        for k in range(n):
            ln = int(lengths[k])
            cnt = int(ls[ln + 1] - ls[ln])
            for m in range(ln - 1):
                pr = int(prod[tail_off[ln] + m * cnt + (k - ls[ln])])
                out[k] += a[pr & 0xffff] * b[pr >> 16]
        return out

    X = make_path("iid", 77, 1, 40, d).astype(np.float64)
    X = X.astype(np.float32)
    a = O.forward_words(np.ascontiguousarray(X[:, :16]), words)[0]
    b = O.forward_words(np.ascontiguousarray(X[:, 15:]), words)[0]
    whole = O.forward_words(X, words)[0]
    np.testing.assert_allclose(product(a, b), whole, rtol=1e-10, atol=1e-12)
    # not commutative: the tables hold prefix and suffix in this order
    assert np.abs(product(b, a) - whole).max() > 1e-6
    rng = np.random.default_rng(5)
    g, a2 = rng.standard_normal(n), rng.standard_normal(n)
    abar = g.copy()
    for t in range(len(adj)):
        if key[t] < n:
            abar[key[t]] += g[adj[t] & 0xffff] * b[adj[t] >> 16]
    lhs = float(abar @ (a - a2))
    rhs = float(g @ (product(a, b) - product(a2, b)))
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(rhs))


GRAPHS = [
    (4, [(a, b) for a in range(4) for b in range(4)], 4),                      # complete graph with loops: the truncation
    (5, [(i, i + 1) for i in range(4)], 5),                                    # a chain
    (6, [(0, 1), (0, 2), (1, 3), (2, 3), (3, 4), (3, 5), (1, 5)], 6),           # a DAG
    (3, [(0, 1), (1, 0), (1, 2), (2, 2)], 5),                                  # cycles and a loop are accepted too
    (4, [], 3),                                                                # no edges: single letters only
]


@pytest.mark.parametrize("case", range(len(GRAPHS)))
def test_graph_tables_bit_exact(case):
    d, edges, depth = GRAPHS[case]
    ws = S.sig_wordset_build_graph(d, edges, depth)
    W = O.graph_words(d, edges, depth)
    t = O.word_tables(W)
    parent, letter, level_start = t["parent"], t["letter"], t["level_start"]
    assert ws.size == len(W)
    assert np.array_equal(ws.parent, parent) and np.array_equal(ws.letter, letter)
    assert np.array_equal(ws.level_start, level_start)
    assert np.array_equal(ws.user_index, np.arange(len(W)))                     # generated in canonical order already
    if case == 0:
        full = S.sig_wordset_build_truncated(4, 4)
        assert np.array_equal(ws.parent, full.parent) and np.array_equal(ws.letter, full.letter)
    if case == 1:
        assert ws.size == sum(5 - n + 1 for n in range(1, 6))                   # runs i, i+1, .., i+n-1


def test_graph_and_leadlag_error_codes():
    lib = S.load_library()
    h = ctypes.c_void_p()
    bad = np.array([[0, 7]], dtype=np.int32)
    assert lib.sig_wordset_build_graph(3, bad.ctypes.data, 1, 2, ctypes.byref(h)) == -2
    assert lib.sig_wordset_build_graph(3, None, 0, 0, ctypes.byref(h)) == -1
    assert lib.sig_wordset_build_graph(3, None, 1, 2, ctypes.byref(h)) == -1
    assert lib.sig_wordset_build_leadlag_sparse(0, 3, ctypes.byref(h)) == -1
    assert lib.sig_wordset_build_leadlag_sparse(2, 0, ctypes.byref(h)) == -1
    assert lib.sig_wordset_build_leadlag_sparse(2, 40, ctypes.byref(h)) == -7


@pytest.mark.parametrize("d,depth", [(1, 5), (2, 5), (3, 4), (5, 4)])
def test_leadlag_sparse_tables_bit_exact(d, depth):
    ws = S.sig_wordset_build_leadlag_sparse(d, depth)
    words = O.leadlag_sparse_words(d, depth)
    W = O.prefix_closure(words)
    t = O.word_tables(W)
    parent, letter, level_start = t["parent"], t["letter"], t["level_start"]
    assert ws.dim == 2 * d and ws.size == len(W)
    assert np.array_equal(ws.parent, parent) and np.array_equal(ws.letter, letter)
    assert np.array_equal(ws.level_start, level_start)
    assert [W[i] for i in np.unique(ws.user_index)] == words                   # exactly the generated words
    if (d, depth) == (5, 4):
        assert len(words) == 1685 and len(W) == 1860


@pytest.mark.parametrize("d,depth", [(2, 1), (2, 6), (3, 4), (4, 5), (5, 2)])
def test_logsig_word_set_bit_exact(d, depth):
    ws = S.sig_wordset_build_logsig(d, depth)
    W = O.logsig_word_set(d, depth)
    t = O.word_tables(W)
    assert ws.size == len(W) and ws.max_len == depth
    assert np.array_equal(ws.parent, t["parent"]) and np.array_equal(ws.letter, t["letter"])
    assert np.array_equal(ws.level_start, t["level_start"])
    lyn = O.lyndon_words(d, depth)
    assert int(S.load_library().sig_wordset_n_lyndon(ws._h)) == len(lyn)
    assert [W[i] for i in ws.user_index] == lyn
    assert int(S.load_library().sig_wordset_n_lyndon(S.sig_wordset_build_truncated(2, 3)._h)) == 0


def test_logsig_word_set_on_a_shape_with_a_truncated_kernel():
    """(4, 6) has kernels for the full truncation: the log-signature set is that truncation, the Lyndon words are
    located in it."""
    ws = S.sig_wordset_build_logsig(4, 6)
    W = O.truncated_words(4, 6)
    assert ws.size == len(W) == 5460
    lyn = O.lyndon_words(4, 6)
    assert int(S.load_library().sig_wordset_n_lyndon(ws._h)) == len(lyn) == 964
    assert [W[i] for i in ws.user_index] == lyn
    assert ws.kernel_name(False, 256, 256) == "trunc_tails_fwd_kernel"


# ---- which kernel a batch would launch (host logic only: no device call is made) ---------------------------
def test_kernel_selection_for_full_truncations(monkeypatch):
    for k in ("SIG_FWD_TAILS", "SIG_BWD_TAILS", "SIG_CHUNKS", "SIG_NO_JIT", "SIG_LANES", "SIG_LANES_LEVELS"):
        monkeypatch.delenv(k, raising=False)
    ws46 = S.sig_wordset_build_truncated(4, 6)
    # d = 4: the one-wavefront-per-row layout for every batch size of the forward except few, long paths
    assert ws46.kernel_name(False, 256, 256) == "trunc_tails_fwd_kernel"
    assert ws46.kernel_name(False, 5000, 64) == "trunc_tails_fwd_kernel"
    assert ws46.kernel_name(False, 64, 2049) == "trunc_mfma_fwd_kernel"
    assert ws46.kernel_name(False, 64, 9) == "trunc_mfma_fwd_kernel"          # too short for two chunks of 8 segments
    assert ws46.kernel_name(True, 256, 256) == "trunc_tails_bwd_kernel"
    assert ws46.kernel_name(True, 4000, 40) == "trunc_tails_bwd_kernel"
    ws46.set_option("fwd_tails", 0)
    ws46.set_option("bwd_tails", 0)
    assert ws46.kernel_name(False, 256, 256) == "trunc_mfma_fwd_kernel"
    assert ws46.kernel_name(True, 256, 256) == "trunc_node_bwd_kernel"
    ws46.set_option("fwd_tails", -1)
    ws46.set_option("bwd_tails", -1)
    ws46.set_option("chunks", 4)                                                # asks for chunk arrays in HBM
    assert ws46.kernel_name(False, 256, 256) == "trunc_mfma_fwd_kernel"
    ws46.set_option("chunks", 0)
    # the knobs are read from the environment once, when a set is built; a set built earlier does not see a change
    monkeypatch.setenv("SIG_FWD_TAILS", "0")
    assert ws46.kernel_name(False, 256, 256) == "trunc_tails_fwd_kernel"
    assert S.sig_wordset_build_truncated(4, 6).kernel_name(False, 256, 256) == "trunc_mfma_fwd_kernel"
    monkeypatch.delenv("SIG_FWD_TAILS")
    # the other instantiated shapes, and a truncation without one
    assert S.sig_wordset_build_truncated(8, 5).kernel_name(True, 128, 1025) == "trunc_node_bwd_kernel"
    assert S.sig_wordset_build_truncated(16, 4).kernel_name(True, 64, 4097) == "trunc_mfma_bwd_kernel"
    assert S.sig_wordset_build_truncated(16, 4).kernel_name(False, 64, 4097) == "trunc_mfma_fwd_kernel"
    # other truncations: a word per lane when the words of length N - 2 (N - 1 beyond 8 letters) fill half a
    # wavefront, else a path per lane
    assert S.sig_wordset_build_truncated(3, 4).kernel_name(False, 64, 65) == "sig_fwd_jit"
    assert S.sig_wordset_build_truncated(6, 5).kernel_name(False, 32, 100) == "sig_fwd_lanes"
    assert S.sig_wordset_build_truncated(10, 4).kernel_name(True, 1, 200) == "sig_bwd_lanes"
    monkeypatch.setenv("SIG_LANES", "0")
    assert S.sig_wordset_build_truncated(6, 5).kernel_name(False, 32, 100) == "sig_fwd_jit"
    monkeypatch.delenv("SIG_LANES")
    # batches beyond the row limit of the register-resident kernels take the run-time compiled ones
    assert ws46.kernel_name(False, 70000, 17) == "sig_fwd_lanes"
