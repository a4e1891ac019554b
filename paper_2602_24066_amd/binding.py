"""ctypes binding of the C ABI (include/sig.h).  Argument marshalling only.

torch is used for device memory and streams; numpy for host tables.  torch is imported lazily so
that the host-only parts (word-set tables, plans) work where no GPU stack is needed.
"""
from __future__ import annotations

import ctypes
import os
from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsig_mi355x.so")
_lib = None

SIG_OK = 0


class SigError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = load_library().sig_strerror(code).decode()
        if code == -6:
            msg += f" (hipError {load_library().sig_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libsig_mi355x.so; raises if it has not been built (python -m paper_2602_24066_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2602_24066_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    c_int, c_i64, c_sz, c_p, c_dbl = ctypes.c_int, ctypes.c_int64, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_double
    PP = ctypes.POINTER(ctypes.c_void_p)

    def sig(name, restype, argtypes):
        f = getattr(lib, name)
        f.restype = restype
        f.argtypes = argtypes

    sig("sig_wordset_build_truncated", c_int, [c_int, c_int, PP])
    sig("sig_wordset_build_anisotropic", c_int, [c_int, c_p, c_dbl, PP])
    sig("sig_wordset_build", c_int, [c_int, c_p, c_p, c_i64, PP])
    sig("sig_forward_windows_workspace_bytes", c_sz, [c_p, c_i64, c_i64, c_i64, c_i64])
    sig("sig_backward_windows_workspace_bytes", c_sz, [c_p, c_i64, c_i64, c_i64, c_i64])
    sig("sig_forward_windows", c_int, [c_p, c_p, c_i64, c_i64, c_p, c_i64, c_i64, c_p, c_p, c_sz, c_p])
    sig("sig_backward_windows", c_int, [c_p, c_p, c_p, c_p, c_i64, c_i64, c_p, c_i64, c_i64, c_p, c_p, c_sz, c_p])
    sig("sig_wordset_build_logsig", c_int, [c_int, c_int, PP])
    sig("sig_wordset_n_lyndon", c_i64, [c_p])
    sig("sig_logsig_forward", c_int, [c_p, c_p, c_i64, c_p, c_p])
    sig("sig_logsig_backward_workspace_bytes", c_sz, [c_p, c_i64])
    sig("sig_logsig_backward", c_int, [c_p, c_p, c_p, c_i64, c_p, c_p, c_sz, c_p])
    sig("sig_wordset_build_graph", c_int, [c_int, c_p, c_i64, c_int, PP])
    sig("sig_wordset_build_leadlag_sparse", c_int, [c_int, c_int, PP])
    sig("sig_leadlag_transform", c_int, [c_p, c_i64, c_i64, c_int, c_p, c_p])
    sig("sig_leadlag_backward", c_int, [c_p, c_i64, c_i64, c_int, c_p, c_p])
    sig("sig_wordset_free", None, [c_p])
    sig("sig_wordset_size", c_i64, [c_p])
    sig("sig_wordset_dim", c_int, [c_p])
    sig("sig_wordset_max_len", c_int, [c_p])
    sig("sig_wordset_n_user", c_i64, [c_p])
    sig("sig_wordset_parent", c_p, [c_p])
    sig("sig_wordset_letter", c_p, [c_p])
    sig("sig_wordset_level_start", c_p, [c_p])
    sig("sig_wordset_user_index", c_p, [c_p])
    sig("sig_wordset_suffix_closed", c_int, [c_p])
    sig("sig_wordset_tail_table", c_p, [c_p, PP])
    sig("sig_wordset_term_tables", c_i64, [c_p, PP, PP, PP, ctypes.POINTER(c_i64)])
    sig("sig_wordset_min_fma_per_step", c_i64, [c_p])
    sig("sig_wordset_kernel_fma_per_step", c_i64, [c_p, c_int])
    sig("sig_wordset_plan_count", c_int, [c_p, c_int])
    sig("sig_wordset_plan_get", c_int, [c_p, c_int, c_int, PP, ctypes.POINTER(c_i64), PP, ctypes.POINTER(c_i64), PP,
                                         ctypes.POINTER(c_i64), ctypes.POINTER(c_i64)])
    sig("sig_wordset_jit_plan_get", c_int, [c_p, c_int, c_i64, PP, ctypes.POINTER(c_i64), PP, ctypes.POINTER(c_i64), PP,
                                             ctypes.POINTER(c_i64), ctypes.POINTER(c_i64)])
    sig("sig_wordset_jit_prepare", c_int, [c_p, c_int, c_i64])
    sig("sig_checkpoint_chunks", c_i64, [c_p, c_i64, c_i64])
    sig("sig_wordset_jit_source", c_sz, [c_p, c_int, c_i64, c_p, c_sz])
    sig("sig_wordset_device_bytes", c_sz, [c_p])
    sig("sig_wordset_upload", c_int, [c_p, c_p, c_sz, c_p])
    sig("sig_forward_workspace_bytes", c_sz, [c_p, c_i64, c_i64])
    sig("sig_backward_workspace_bytes", c_sz, [c_p, c_i64, c_i64])
    sig("sig_forward", c_int, [c_p, c_p, c_i64, c_i64, c_p, c_p, c_sz, c_p])
    sig("sig_backward", c_int, [c_p, c_p, c_p, c_p, c_i64, c_i64, c_p, c_p, c_sz, c_p])
    sig("sig_checkpoint_bytes", c_sz, [c_p, c_i64, c_i64])
    sig("sig_forward_checkpointed_workspace_bytes", c_sz, [c_p, c_i64, c_i64])
    sig("sig_backward_checkpointed_workspace_bytes", c_sz, [c_p, c_i64, c_i64])
    sig("sig_forward_checkpointed", c_int, [c_p, c_p, c_i64, c_i64, c_p, c_p, c_sz, c_p, c_sz, c_p])
    sig("sig_backward_checkpointed", c_int, [c_p, c_p, c_p, c_p, c_p, c_sz, c_i64, c_i64, c_p, c_p, c_sz, c_p])
    sig("sig_backward_residual", c_int, [c_p, c_p, c_p, c_p, c_i64, c_i64, c_p, c_p, c_p, c_sz, c_p])
    sig("sig_backward_static", c_int, [c_p, c_p, c_p, c_p, c_i64, c_i64, c_p, c_p])
    sig("sig_wordset_set_option", c_int, [c_p, ctypes.c_char_p, c_int])
    sig("sig_wordset_get_option", c_int, [c_p, ctypes.c_char_p, ctypes.POINTER(c_int)])
    sig("sig_profile_enable", c_int, [c_int])
    sig("sig_profile_read", c_int, [c_int, ctypes.POINTER(c_i64), ctypes.POINTER(c_dbl)])
    sig("sig_strerror", ctypes.c_char_p, [c_int])
    sig("sig_last_hip_error", c_int, [])
    sig("sig_version", ctypes.c_char_p, [])
    sig("sig_wordset_kernel_name", ctypes.c_char_p, [c_p, c_int])
    sig("sig_kernel_name", ctypes.c_char_p, [c_p, c_int, c_i64, c_i64])
    sig("sig_probe_fma", c_int, [c_p, c_sz, c_int, c_int, c_p])
    sig("sig_probe_issue", c_int, [c_p, c_sz, c_int, c_int, c_int, c_p])
    sig("sig_jit_launch_shape_ok", c_int, [c_int, c_int, c_int, c_int])
    _lib = lib
    return lib


def _check(rc: int, where: str):
    if rc != SIG_OK:
        raise SigError(rc, where)


def _np_from_ptr(ptr, n: int, dtype) -> np.ndarray:
    if n == 0 or not ptr:
        return np.zeros(0, dtype=dtype)
    buf = (ctypes.c_char * (n * np.dtype(dtype).itemsize)).from_address(ptr)
    return np.frombuffer(buf, dtype=dtype, count=n).copy()


class WordSet:
    """Owner of a sig_wordset handle plus (after upload) the device buffer holding its launch plan."""

    def __init__(self, handle: int):
        self._h = ctypes.c_void_p(handle)
        self._dev = None          # torch uint8 tensor keeping the device tables alive
        self._lib = load_library()

    def __del__(self):
        try:
            if getattr(self, "_h", None) is not None and self._h:
                self._lib.sig_wordset_free(self._h)
                self._h = None
        except Exception:
            pass

    # ---- host accessors
    @property
    def size(self) -> int:
        return int(self._lib.sig_wordset_size(self._h))

    @property
    def dim(self) -> int:
        return int(self._lib.sig_wordset_dim(self._h))

    @property
    def max_len(self) -> int:
        return int(self._lib.sig_wordset_max_len(self._h))

    @property
    def parent(self) -> np.ndarray:
        return _np_from_ptr(self._lib.sig_wordset_parent(self._h), self.size, np.int32)

    @property
    def letter(self) -> np.ndarray:
        return _np_from_ptr(self._lib.sig_wordset_letter(self._h), self.size, np.int32)

    @property
    def level_start(self) -> np.ndarray:
        return _np_from_ptr(self._lib.sig_wordset_level_start(self._h), self.max_len + 2, np.int32)

    @property
    def user_index(self) -> np.ndarray:
        n = int(self._lib.sig_wordset_n_user(self._h))
        return _np_from_ptr(self._lib.sig_wordset_user_index(self._h), n, np.int64)

    @property
    def suffix_closed(self) -> bool:
        return int(self._lib.sig_wordset_suffix_closed(self._h)) == 1

    def tail_table(self):
        """(tail_tab, tail_off) of a suffix-closed set, or None: see sig_wordset_tail_table."""
        off = ctypes.c_void_p()
        tab = self._lib.sig_wordset_tail_table(self._h, ctypes.byref(off))
        if not tab:
            return None
        tail_off = _np_from_ptr(off.value, self.max_len + 2, np.int32)
        ls = self.level_start
        total = sum((n - 1) * int(ls[n + 1] - ls[n]) for n in range(2, self.max_len + 1))
        return _np_from_ptr(tab, max(total, 1), np.int32), tail_off

    def term_tables(self):
        """(prod_pairs, adj_pairs, adj_key) of a suffix-closed set, or None: see sig_wordset_term_tables."""
        pp, ap, ak, n_adj = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_int64()
        n = int(self._lib.sig_wordset_term_tables(self._h, ctypes.byref(pp), ctypes.byref(ap), ctypes.byref(ak), ctypes.byref(n_adj)))
        if n < 0:
            return None
        return (_np_from_ptr(pp.value, n, np.uint32), _np_from_ptr(ap.value, n_adj.value, np.uint32),
                _np_from_ptr(ak.value, n_adj.value, np.uint32))

    @property
    def lengths(self) -> np.ndarray:
        ls = self.level_start
        out = np.zeros(self.size, dtype=np.int32)
        for n in range(1, self.max_len + 1):
            out[ls[n]:ls[n + 1]] = n
        return out

    @property
    def min_fma_per_step(self) -> int:
        return int(self._lib.sig_wordset_min_fma_per_step(self._h))

    def kernel_fma_per_step(self, backward: bool = False) -> int:
        return int(self._lib.sig_wordset_kernel_fma_per_step(self._h, int(backward)))

    def kernel_name(self, backward: bool = False, B: int = 0, n_points: int = 0) -> str:
        """Kernel family for this set; with B and n_points the main kernel that batch would launch."""
        if B > 0 and n_points > 1:
            return self._lib.sig_kernel_name(self._h, int(backward), B, n_points).decode()
        return self._lib.sig_wordset_kernel_name(self._h, int(backward)).decode()

    def set_option(self, name: str, value: int) -> None:
        """Launch-shape knob of this word set (see sig_wordset_set_option in include/sig.h)."""
        _check(self._lib.sig_wordset_set_option(self._h, name.encode(), int(value)), "sig_wordset_set_option")

    def get_option(self, name: str) -> int:
        v = ctypes.c_int()
        _check(self._lib.sig_wordset_get_option(self._h, name.encode(), ctypes.byref(v)), "sig_wordset_get_option")
        return int(v.value)

    def plan_count(self, backward: bool = False) -> int:
        return int(self._lib.sig_wordset_plan_count(self._h, int(backward)))

    def plan(self, backward: bool = False, variant: int = 0) -> dict:
        units, ops, slots = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        nu, no, ns, fma = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        _check(self._lib.sig_wordset_plan_get(self._h, int(backward), variant, ctypes.byref(units), ctypes.byref(nu),
                                              ctypes.byref(ops), ctypes.byref(no), ctypes.byref(slots), ctypes.byref(ns),
                                              ctypes.byref(fma)), "sig_wordset_plan_get")
        return {"units": _np_from_ptr(units.value, nu.value * 4, np.int32).reshape(-1, 4),
                "ops": _np_from_ptr(ops.value, no.value, np.uint32),
                "slot_word": _np_from_ptr(slots.value, ns.value, np.int32),
                "fma_per_step": int(fma.value)}

    def jit_plan(self, backward: bool, B: int) -> dict:
        """The balanced plan the specialised kernel for a batch of B paths is generated from (same format as plan)."""
        units, ops, slots = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        nu, no, ns, fma = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        _check(self._lib.sig_wordset_jit_plan_get(self._h, int(backward), B, ctypes.byref(units), ctypes.byref(nu),
                                                  ctypes.byref(ops), ctypes.byref(no), ctypes.byref(slots), ctypes.byref(ns),
                                                  ctypes.byref(fma)), "sig_wordset_jit_plan_get")
        return {"units": _np_from_ptr(units.value, nu.value * 4, np.int32).reshape(-1, 4),
                "ops": _np_from_ptr(ops.value, no.value, np.uint32),
                "slot_word": _np_from_ptr(slots.value, ns.value, np.int32),
                "fma_per_step": int(fma.value)}

    def jit_prepare(self, backward: bool, B: int) -> int:
        """Compiles the specialised kernel a batch of B paths would use; returns the library's status code."""
        return int(self._lib.sig_wordset_jit_prepare(self._h, int(backward), B))

    def jit_source(self, backward: bool, B: int) -> str:
        n = int(self._lib.sig_wordset_jit_source(self._h, int(backward), B, None, 0))
        buf = ctypes.create_string_buffer(n + 1)
        self._lib.sig_wordset_jit_source(self._h, int(backward), B, buf, n + 1)
        return buf.value.decode()

    # ---- device side
    def upload(self, device="cuda:0"):
        import torch
        nbytes = int(self._lib.sig_wordset_device_bytes(self._h))
        dev = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        off = (-dev.data_ptr()) % 256
        with torch.cuda.device(dev.device):
            stream = torch.cuda.current_stream().cuda_stream
            _check(self._lib.sig_wordset_upload(self._h, ctypes.c_void_p(dev.data_ptr() + off), nbytes,
                                                ctypes.c_void_p(stream)), "sig_wordset_upload")
            torch.cuda.current_stream().synchronize()
        self._dev = dev
        return self


def sig_wordset_build_truncated(d: int, depth: int) -> WordSet:
    h = ctypes.c_void_p()
    _check(load_library().sig_wordset_build_truncated(d, depth, ctypes.byref(h)), "sig_wordset_build_truncated")
    return WordSet(h.value)


def sig_wordset_build_anisotropic(d: int, weights: Sequence[float], cutoff: float) -> WordSet:
    w = np.ascontiguousarray(np.asarray(weights, dtype=np.float64))
    if w.shape != (d,):
        raise ValueError("weights must have d entries")
    h = ctypes.c_void_p()
    _check(load_library().sig_wordset_build_anisotropic(d, w.ctypes.data, float(cutoff), ctypes.byref(h)),
           "sig_wordset_build_anisotropic")
    return WordSet(h.value)


def sig_wordset_build(d: int, words: Iterable[Sequence[int]]) -> WordSet:
    words = [tuple(int(c) for c in w) for w in words]
    offsets = np.zeros(len(words) + 1, dtype=np.int64)
    for k, w in enumerate(words):
        offsets[k + 1] = offsets[k] + len(w)
    letters = np.fromiter((c for w in words for c in w), dtype=np.int32, count=int(offsets[-1]))
    if letters.size == 0:
        letters = np.zeros(1, dtype=np.int32)
    h = ctypes.c_void_p()
    _check(load_library().sig_wordset_build(d, letters.ctypes.data, offsets.ctypes.data, len(words), ctypes.byref(h)),
           "sig_wordset_build")
    return WordSet(h.value)


def sig_wordset_build_graph(d: int, edges: Iterable[Sequence[int]], depth: int) -> WordSet:
    """Words of length <= depth whose consecutive letters are joined by an edge (from, to)."""
    e = np.ascontiguousarray(np.array([tuple(int(c) for c in ed) for ed in edges], dtype=np.int32).reshape(-1, 2))
    h = ctypes.c_void_p()
    _check(load_library().sig_wordset_build_graph(d, e.ctypes.data if e.size else None, e.shape[0], depth, ctypes.byref(h)),
           "sig_wordset_build_graph")
    return WordSet(h.value)


def sig_wordset_build_leadlag_sparse(d: int, depth: int) -> WordSet:
    """Sparse lead-lag word set over 2 d letters (lag i -> letter i, lead i -> letter d + i)."""
    h = ctypes.c_void_p()
    _check(load_library().sig_wordset_build_leadlag_sparse(d, depth, ctypes.byref(h)), "sig_wordset_build_leadlag_sparse")
    return WordSet(h.value)


def sig_leadlag_transform(path, out=None):
    """path float32 CUDA [B, n, d] -> lead-lag path [B, 2 n - 1, 2 d]."""
    import torch
    if not path.is_cuda or path.dtype != torch.float32 or path.dim() != 3:
        raise ValueError("path must be a float32 CUDA tensor [B, n, d]")
    path = path.contiguous()
    B, P, d = path.shape
    if out is None:
        out = torch.empty((B, 2 * P - 1, 2 * d), dtype=torch.float32, device=path.device)
    with torch.cuda.device(path.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(load_library().sig_leadlag_transform(ctypes.c_void_p(path.data_ptr()), B, P, d, ctypes.c_void_p(out.data_ptr()),
                                                    ctypes.c_void_p(stream)), "sig_leadlag_transform")
    return out


def sig_leadlag_backward(grad_out, out=None):
    """Gradient of the lead-lag transform: [B, 2 n - 1, 2 d] -> [B, n, d]."""
    import torch
    if not grad_out.is_cuda or grad_out.dtype != torch.float32 or grad_out.dim() != 3:
        raise ValueError("grad_out must be a float32 CUDA tensor [B, 2 n - 1, 2 d]")
    grad_out = grad_out.contiguous()
    B, M, d2 = grad_out.shape
    if M % 2 != 1 or d2 % 2 != 0:
        raise ValueError("not the shape of a lead-lag path")
    P, d = (M + 1) // 2, d2 // 2
    if out is None:
        out = torch.empty((B, P, d), dtype=torch.float32, device=grad_out.device)
    with torch.cuda.device(grad_out.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(load_library().sig_leadlag_backward(ctypes.c_void_p(grad_out.data_ptr()), B, P, d, ctypes.c_void_p(out.data_ptr()),
                                                   ctypes.c_void_p(stream)), "sig_leadlag_backward")
    return out


def sig_wordset_build_logsig(d: int, depth: int) -> WordSet:
    """Word set for log-signatures of the given depth (every word shorter than depth + the Lyndon words of length depth);
    user_index holds the columns of the Lyndon words."""
    h = ctypes.c_void_p()
    _check(load_library().sig_wordset_build_logsig(d, depth, ctypes.byref(h)), "sig_wordset_build_logsig")
    return WordSet(h.value)


def sig_logsig_forward(ws: WordSet, coeffs):
    """coeffs float32 CUDA [B, |W|] (from sig_forward on a log-signature word set) -> logsig [B, n_lyndon]."""
    import torch
    coeffs = coeffs.contiguous()
    B = coeffs.shape[0]
    lib = load_library()
    n = int(lib.sig_wordset_n_lyndon(ws._h))
    out = torch.empty((B, n), dtype=torch.float32, device=coeffs.device)
    with torch.cuda.device(coeffs.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(lib.sig_logsig_forward(ws._h, ctypes.c_void_p(coeffs.data_ptr()), B, ctypes.c_void_p(out.data_ptr()),
                                      ctypes.c_void_p(stream)), "sig_logsig_forward")
    return out


def sig_logsig_backward(ws: WordSet, coeffs, grad_logsig):
    """grad_logsig [B, n_lyndon] -> gradient with respect to the signature coefficients [B, |W|]."""
    import torch
    coeffs, grad_logsig = coeffs.contiguous(), grad_logsig.contiguous()
    B = coeffs.shape[0]
    lib = load_library()
    out = torch.empty_like(coeffs)
    nbytes = int(lib.sig_logsig_backward_workspace_bytes(ws._h, B))
    keep, wptr = _aligned_workspace(nbytes, coeffs.device)
    with torch.cuda.device(coeffs.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(lib.sig_logsig_backward(ws._h, ctypes.c_void_p(coeffs.data_ptr()), ctypes.c_void_p(grad_logsig.data_ptr()), B,
                                       ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(wptr), nbytes, ctypes.c_void_p(stream)),
               "sig_logsig_backward")
    if keep is not None:
        keep.record_stream(torch.cuda.current_stream(coeffs.device))
    return out


def _windows_tensor(windows, device):
    """(device int64 [K, 2] tensor, K, longest window in segments) from a sequence of (l, r) point-index pairs."""
    import torch
    w = np.ascontiguousarray(np.asarray(windows, dtype=np.int64).reshape(-1, 2))
    if w.shape[0] and (np.any(w[:, 0] < 0) or np.any(w[:, 1] < w[:, 0])):
        raise ValueError("windows must be pairs 0 <= l <= r")
    max_len = int((w[:, 1] - w[:, 0]).max()) if w.shape[0] else 0
    return torch.from_numpy(w).to(device), int(w.shape[0]), max_len


def sig_forward_windows(ws: WordSet, path, windows):
    """Signatures over windows: path float32 CUDA [B, n, d], windows (l, r) point indices -> coeffs [B, K, |W|]."""
    import torch
    if not path.is_cuda or path.dtype != torch.float32 or path.dim() != 3:
        raise ValueError("path must be a float32 CUDA tensor [B, n, d]")
    path = path.contiguous()
    B, P, d = path.shape
    if d != ws.dim:
        raise ValueError(f"path has {d} channels, word set was built for {ws.dim}")
    wt, K, max_len = _windows_tensor(windows, path.device)
    if K and int(np.asarray(windows).reshape(-1, 2)[:, 1].max()) >= P:
        raise ValueError("window end beyond the path")
    lib = load_library()
    out = torch.empty((B, K, ws.size), dtype=torch.float32, device=path.device)
    nbytes = int(lib.sig_forward_windows_workspace_bytes(ws._h, B, P, K, max_len))
    keep, wptr = _aligned_workspace(nbytes, path.device)
    with torch.cuda.device(path.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(lib.sig_forward_windows(ws._h, ctypes.c_void_p(path.data_ptr()), B, P, ctypes.c_void_p(wt.data_ptr()), K, max_len,
                                       ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(wptr), nbytes, ctypes.c_void_p(stream)),
               "sig_forward_windows")
    for t in (keep, wt):
        if t is not None:
            t.record_stream(torch.cuda.current_stream(path.device))
    return out


def sig_backward_windows(ws: WordSet, path, windows, coeffs, grad_coeffs):
    """Gradient with respect to the path of a loss on the windowed signatures: grad_coeffs [B, K, |W|] -> [B, n, d]."""
    import torch
    for name, t in (("path", path), ("coeffs", coeffs), ("grad_coeffs", grad_coeffs)):
        if not t.is_cuda or t.dtype != torch.float32:
            raise ValueError(f"{name} must be a float32 CUDA tensor")
    if path.dim() != 3 or path.shape[2] != ws.dim:
        raise ValueError(f"path must be [B, n, {ws.dim}]")
    path, coeffs, grad_coeffs = path.contiguous(), coeffs.contiguous(), grad_coeffs.contiguous()
    B, P, d = path.shape
    wt, K, max_len = _windows_tensor(windows, path.device)
    if K and int(np.asarray(windows).reshape(-1, 2)[:, 1].max()) >= P:
        raise ValueError("window end beyond the path")
    if tuple(coeffs.shape) != (B, K, ws.size) or tuple(grad_coeffs.shape) != (B, K, ws.size):
        raise ValueError("shape mismatch")
    lib = load_library()
    out = torch.empty((B, P, d), dtype=torch.float32, device=path.device)
    nbytes = int(lib.sig_backward_windows_workspace_bytes(ws._h, B, P, K, max_len))
    keep, wptr = _aligned_workspace(nbytes, path.device)
    with torch.cuda.device(path.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(lib.sig_backward_windows(ws._h, ctypes.c_void_p(path.data_ptr()), ctypes.c_void_p(coeffs.data_ptr()),
                                        ctypes.c_void_p(grad_coeffs.data_ptr()), B, P, ctypes.c_void_p(wt.data_ptr()), K, max_len,
                                        ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(wptr), nbytes, ctypes.c_void_p(stream)),
               "sig_backward_windows")
    for t in (keep, wt):
        if t is not None:
            t.record_stream(torch.cuda.current_stream(path.device))
    return out


class WindowPlan:
    """Windowed signatures with every buffer allocated once: the device copy of the window list, the outputs and
    the workspaces of sig_forward_windows / sig_backward_windows.  forward() and backward() only enqueue (for
    timing loops and HIP-graph capture); each call overwrites the buffers of the one before."""

    def __init__(self, ws: WordSet, path, windows):
        import torch
        if not path.is_cuda or path.dtype != torch.float32 or path.dim() != 3 or path.shape[2] != ws.dim:
            raise ValueError("path must be a float32 CUDA tensor [B, n, d] with the word set's d")
        self.ws, self.path = ws, path.contiguous()
        B, P, d = self.path.shape
        self.wt, self.K, self.max_len = _windows_tensor(windows, path.device)
        if self.K and int(np.asarray(windows).reshape(-1, 2)[:, 1].max()) >= P:
            raise ValueError("window end beyond the path")
        lib = load_library()
        self.coeffs = torch.empty((B, self.K, ws.size), dtype=torch.float32, device=path.device)
        self.grad_path = torch.empty((B, P, d), dtype=torch.float32, device=path.device)
        self.nf = int(lib.sig_forward_windows_workspace_bytes(ws._h, B, P, self.K, self.max_len))
        self.nb = int(lib.sig_backward_windows_workspace_bytes(ws._h, B, P, self.K, self.max_len))
        self._wf, self.wf = _aligned_workspace(self.nf, path.device)
        self._wb, self.wb = _aligned_workspace(self.nb, path.device)

    def forward(self):
        import torch
        B, P, _ = self.path.shape
        with torch.cuda.device(self.path.device):
            stream = torch.cuda.current_stream().cuda_stream
            _check(load_library().sig_forward_windows(
                self.ws._h, ctypes.c_void_p(self.path.data_ptr()), B, P, ctypes.c_void_p(self.wt.data_ptr()), self.K,
                self.max_len, ctypes.c_void_p(self.coeffs.data_ptr()), ctypes.c_void_p(self.wf), self.nf,
                ctypes.c_void_p(stream)), "sig_forward_windows")
        return self.coeffs

    def backward(self, grad_coeffs):
        import torch
        B, P, _ = self.path.shape
        if tuple(grad_coeffs.shape) != tuple(self.coeffs.shape) or grad_coeffs.dtype != torch.float32 or not grad_coeffs.is_cuda:
            raise ValueError("grad_coeffs must be a float32 CUDA tensor [B, K, |W|]")
        grad_coeffs = grad_coeffs.contiguous()
        with torch.cuda.device(self.path.device):
            stream = torch.cuda.current_stream().cuda_stream
            _check(load_library().sig_backward_windows(
                self.ws._h, ctypes.c_void_p(self.path.data_ptr()), ctypes.c_void_p(self.coeffs.data_ptr()),
                ctypes.c_void_p(grad_coeffs.data_ptr()), B, P, ctypes.c_void_p(self.wt.data_ptr()), self.K, self.max_len,
                ctypes.c_void_p(self.grad_path.data_ptr()), ctypes.c_void_p(self.wb), self.nb, ctypes.c_void_p(stream)),
                "sig_backward_windows")
        return self.grad_path


def _aligned_workspace(nbytes: int, device):
    import torch
    if nbytes == 0:
        return None, 0
    t = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
    return t, t.data_ptr() + ((-t.data_ptr()) % 256)


def sig_forward(ws: WordSet, path, out=None, workspace=None):
    """path: float32 CUDA tensor [B, L+1, d] -> coeffs float32 [B, |W|].  Enqueues on torch's current stream."""
    import torch
    if not path.is_cuda or path.dtype != torch.float32 or path.dim() != 3:
        raise ValueError("path must be a float32 CUDA tensor [B, L+1, d]")
    path = path.contiguous()
    B, P, d = path.shape
    if d != ws.dim:
        raise ValueError(f"path has {d} channels, word set was built for {ws.dim}")
    lib = load_library()
    if out is None:
        out = torch.empty((B, ws.size), dtype=torch.float32, device=path.device)
    nbytes = int(lib.sig_forward_workspace_bytes(ws._h, B, P))
    if workspace is None:
        keep, wptr = _aligned_workspace(nbytes, path.device)
    else:
        keep, wptr, nbytes = None, workspace.data_ptr(), workspace.numel() * workspace.element_size()   # the caller's to keep alive
    with torch.cuda.device(path.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(lib.sig_forward(ws._h, ctypes.c_void_p(path.data_ptr()), B, P, ctypes.c_void_p(out.data_ptr()),
                               ctypes.c_void_p(wptr), nbytes, ctypes.c_void_p(stream)), "sig_forward")
    if keep is not None:
        keep.record_stream(torch.cuda.current_stream(path.device))
    return out


def sig_backward(ws: WordSet, path, coeffs, grad_coeffs, out=None, workspace=None):
    """Returns grad_path float32 [B, L+1, d].  Enqueues on torch's current stream."""
    import torch
    for name, t in (("path", path), ("coeffs", coeffs), ("grad_coeffs", grad_coeffs)):
        if not t.is_cuda or t.dtype != torch.float32:
            raise ValueError(f"{name} must be a float32 CUDA tensor")
    path, coeffs, grad_coeffs = path.contiguous(), coeffs.contiguous(), grad_coeffs.contiguous()
    B, P, d = path.shape
    if d != ws.dim or tuple(coeffs.shape) != (B, ws.size) or tuple(grad_coeffs.shape) != (B, ws.size):
        raise ValueError("shape mismatch")
    lib = load_library()
    if out is None:
        out = torch.empty((B, P, d), dtype=torch.float32, device=path.device)
    nbytes = int(lib.sig_backward_workspace_bytes(ws._h, B, P))
    if workspace is None:
        keep, wptr = _aligned_workspace(nbytes, path.device)
    else:
        keep, wptr, nbytes = None, workspace.data_ptr(), workspace.numel() * workspace.element_size()   # the caller's to keep alive
    with torch.cuda.device(path.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(lib.sig_backward(ws._h, ctypes.c_void_p(path.data_ptr()), ctypes.c_void_p(coeffs.data_ptr()),
                                ctypes.c_void_p(grad_coeffs.data_ptr()), B, P, ctypes.c_void_p(out.data_ptr()),
                                ctypes.c_void_p(wptr), nbytes, ctypes.c_void_p(stream)), "sig_backward")
    if keep is not None:
        keep.record_stream(torch.cuda.current_stream(path.device))
    return out


def sig_backward_residual(ws: WordSet, path, coeffs, grad_coeffs):
    """(grad_path, residual [B]): sig_backward plus, per path, the largest absolute coefficient left when the terminal
    signature has been stepped back through all segments (zero in exact arithmetic)."""
    import torch
    path, coeffs, grad_coeffs = path.contiguous(), coeffs.contiguous(), grad_coeffs.contiguous()
    B, P, d = path.shape
    if d != ws.dim or tuple(coeffs.shape) != (B, ws.size) or tuple(grad_coeffs.shape) != (B, ws.size):
        raise ValueError("shape mismatch")
    lib = load_library()
    out = torch.empty((B, P, d), dtype=torch.float32, device=path.device)
    resid = torch.empty((B,), dtype=torch.float32, device=path.device)
    bt = ws.get_option("bwd_tails")
    ws.set_option("bwd_tails", 0)                 # workspace of the kernel that walks whole paths
    nbytes = int(lib.sig_backward_workspace_bytes(ws._h, B, P))
    ws.set_option("bwd_tails", bt)
    keep, wptr = _aligned_workspace(nbytes, path.device)
    with torch.cuda.device(path.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(lib.sig_backward_residual(ws._h, ctypes.c_void_p(path.data_ptr()), ctypes.c_void_p(coeffs.data_ptr()),
                                         ctypes.c_void_p(grad_coeffs.data_ptr()), B, P, ctypes.c_void_p(out.data_ptr()),
                                         ctypes.c_void_p(resid.data_ptr()), ctypes.c_void_p(wptr), nbytes,
                                         ctypes.c_void_p(stream)), "sig_backward_residual")
    if keep is not None:
        keep.record_stream(torch.cuda.current_stream(path.device))
    return out, resid


def sig_forward_checkpointed(ws: WordSet, path, out=None, checkpoint=None, workspace=None):
    """sig_forward that also leaves the time-chunk signatures in `checkpoint` for sig_backward_checkpointed.
    Returns (coeffs, checkpoint); checkpoint is a uint8 CUDA tensor (empty where the library takes no chunks)."""
    import torch
    if not path.is_cuda or path.dtype != torch.float32 or path.dim() != 3 or path.shape[2] != ws.dim:
        raise ValueError("path must be a float32 CUDA tensor [B, L+1, d] with the word set's d")
    path = path.contiguous()
    B, P, _ = path.shape
    lib = load_library()
    if out is None:
        out = torch.empty((B, ws.size), dtype=torch.float32, device=path.device)
    nck = int(lib.sig_checkpoint_bytes(ws._h, B, P))
    if checkpoint is None:
        checkpoint = torch.empty(nck, dtype=torch.uint8, device=path.device)
    nbytes = int(lib.sig_forward_checkpointed_workspace_bytes(ws._h, B, P))
    if workspace is None:
        keep, wptr = _aligned_workspace(nbytes, path.device)
    else:
        keep, wptr, nbytes = None, workspace.data_ptr(), workspace.numel() * workspace.element_size()
    with torch.cuda.device(path.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(lib.sig_forward_checkpointed(ws._h, ctypes.c_void_p(path.data_ptr()), B, P, ctypes.c_void_p(out.data_ptr()),
                                            ctypes.c_void_p(checkpoint.data_ptr() if checkpoint.numel() else 0),
                                            checkpoint.numel() * checkpoint.element_size(), ctypes.c_void_p(wptr), nbytes,
                                            ctypes.c_void_p(stream)), "sig_forward_checkpointed")
    if keep is not None:
        keep.record_stream(torch.cuda.current_stream(path.device))
    return out, checkpoint


def sig_backward_checkpointed(ws: WordSet, path, coeffs, grad_coeffs, checkpoint, out=None, workspace=None):
    """sig_backward over the time chunks sig_forward_checkpointed left in `checkpoint`."""
    import torch
    for name, t in (("path", path), ("coeffs", coeffs), ("grad_coeffs", grad_coeffs)):
        if not t.is_cuda or t.dtype != torch.float32:
            raise ValueError(f"{name} must be a float32 CUDA tensor")
    path, coeffs, grad_coeffs = path.contiguous(), coeffs.contiguous(), grad_coeffs.contiguous()
    B, P, d = path.shape
    if d != ws.dim or tuple(coeffs.shape) != (B, ws.size) or tuple(grad_coeffs.shape) != (B, ws.size):
        raise ValueError("shape mismatch")
    lib = load_library()
    if out is None:
        out = torch.empty((B, P, d), dtype=torch.float32, device=path.device)
    nbytes = int(lib.sig_backward_checkpointed_workspace_bytes(ws._h, B, P))
    if workspace is None:
        keep, wptr = _aligned_workspace(nbytes, path.device)
    else:
        keep, wptr, nbytes = None, workspace.data_ptr(), workspace.numel() * workspace.element_size()
    with torch.cuda.device(path.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(lib.sig_backward_checkpointed(ws._h, ctypes.c_void_p(path.data_ptr()), ctypes.c_void_p(coeffs.data_ptr()),
                                             ctypes.c_void_p(grad_coeffs.data_ptr()),
                                             ctypes.c_void_p(checkpoint.data_ptr() if checkpoint.numel() else 0),
                                             checkpoint.numel() * checkpoint.element_size(), B, P,
                                             ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(wptr), nbytes,
                                             ctypes.c_void_p(stream)), "sig_backward_checkpointed")
    if keep is not None:
        keep.record_stream(torch.cuda.current_stream(path.device))
    return out


SIG_STATIC_SCRATCH_BYTES = 32 << 20


def sig_backward_static(ws: WordSet, path, coeffs, grad_coeffs, out):
    """sig_backward without a workspace argument and without any allocation: the library's static device scratch
    serves as workspace.  `out` [B, L+1, d] is the caller's.  Enqueues on torch's current stream."""
    import torch
    for name, t in (("path", path), ("coeffs", coeffs), ("grad_coeffs", grad_coeffs), ("out", out)):
        if not t.is_cuda or t.dtype != torch.float32 or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous float32 CUDA tensor")
    B, P, d = path.shape
    if d != ws.dim or tuple(coeffs.shape) != (B, ws.size) or tuple(grad_coeffs.shape) != (B, ws.size) or tuple(out.shape) != (B, P, d):
        raise ValueError("shape mismatch")
    with torch.cuda.device(path.device):
        stream = torch.cuda.current_stream().cuda_stream
        _check(load_library().sig_backward_static(ws._h, ctypes.c_void_p(path.data_ptr()), ctypes.c_void_p(coeffs.data_ptr()),
                                                  ctypes.c_void_p(grad_coeffs.data_ptr()), B, P, ctypes.c_void_p(out.data_ptr()),
                                                  ctypes.c_void_p(stream)), "sig_backward_static")
    return out


def sig_probe_fma_tflops(blocks: int = 256 * 32, iters: int = 4096, repeats: int = 5) -> float:
    """Measured rate of plain (unpacked) FP32 multiply-adds: a register-only kernel timed with events on the current
    stream, best of `repeats`."""
    import torch
    lib = load_library()
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    best = float("inf")
    for _ in range(repeats + 1):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        _check(lib.sig_probe_fma(ctypes.c_void_p(out.data_ptr()), out.numel() * 4, blocks, iters, ctypes.c_void_p(stream)),
               "sig_probe_fma")
        e1.record()
        e1.synchronize()
        best = min(best, e0.elapsed_time(e1))
    return 2.0 * 16 * iters * 256 * blocks / (best * 1e-3) / 1e12


def sig_probe_issue_ns(mode: int, waves_per_simd: int = 1, iters: int = 8192, repeats: int = 3) -> float:
    """Nanoseconds a SIMD takes per probe iteration and wavefront (64 multiply-adds and / or 8 matrix instructions,
    see sig_probe_issue in include/sig.h) with `waves_per_simd` wavefronts resident on every SIMD; best of `repeats`."""
    import torch
    lib = load_library()
    blocks = 256 * waves_per_simd
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    best = float("inf")
    for _ in range(repeats + 1):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        _check(lib.sig_probe_issue(ctypes.c_void_p(out.data_ptr()), out.numel() * 4, blocks, iters, mode, ctypes.c_void_p(stream)),
               "sig_probe_issue")
        e1.record()
        e1.synchronize()
        best = min(best, e0.elapsed_time(e1))
    return best * 1e6 / iters / waves_per_simd


def sig_profile_enable(on, channels=None) -> None:
    """on: False / True (all four channels); channels: iterable of channel numbers 0..3 (forward main kernel,
    backward main kernel, whole forward call, whole backward call) to record only those."""
    arg = int(bool(on))
    if on and channels is not None:
        arg = 0
        for c in channels:
            arg |= 2 << int(c)
    _check(load_library().sig_profile_enable(arg), "sig_profile_enable")


def sig_profile_read(backward: bool, whole_call: bool = False) -> Tuple[int, float]:
    """(calls recorded, summed time in ms) since sig_profile_enable(True): of the main kernel, or with whole_call of
    everything the call enqueued."""
    n, ms = ctypes.c_int64(), ctypes.c_double()
    which = int(bool(backward)) + (2 if whole_call else 0)
    _check(load_library().sig_profile_read(which, ctypes.byref(n), ctypes.byref(ms)), "sig_profile_read")
    return int(n.value), float(ms.value)
