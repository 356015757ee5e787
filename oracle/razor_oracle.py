"""RazorAttention fp64 CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

ctypes front end of ``razor_oracle.c`` (same folder), which states the
paper's compressed-KV attention (Algorithm 1, Eq.(4), Eq.(5)) in plain fp64 C.
Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this module; the HIP library never does, and the two share no code.

Tensors are handed over as their stored bits: ``float32`` arrays, or
``uint16`` arrays holding bf16 bit patterns.  ``as_raw`` converts CPU torch
tensors (fp32 / bf16) without changing a bit.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "razor_oracle.c")
_LIB = os.path.join(_HERE, "librazor_oracle.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, vp, dbl, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_double, ctypes.c_int
        L.oracle_select.restype = i64
        L.oracle_select.argtypes = [i64, ci, i64, i64, vp, vp, vp]
        L.oracle_comp_token.restype = None
        L.oracle_comp_token.argtypes = [vp, vp, ci, i64, ci, i64, i64, vp, vp]
        L.oracle_decode_batch.restype = ci
        L.oracle_decode_batch.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, i64, i64, i64,
                                          vp, vp, vp, vp, i64, i64, vp, vp, vp, dbl, vp]
        L.oracle_compress_batch.restype = ci
        L.oracle_compress_batch.argtypes = [vp, vp, ci, ci, ci, ci, i64, i64, i64,
                                            vp, vp, i64, i64, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def as_raw(t):
    """CPU torch tensor (fp32 or bf16) or numpy array -> numpy array of stored bits."""
    if isinstance(t, np.ndarray):
        assert t.dtype in (np.float32, np.uint16), t.dtype
        return t
    import torch
    t = t.detach().cpu()
    if t.dtype == torch.float32:
        return t.numpy()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dtype_code(a: np.ndarray) -> int:
    return F32 if a.dtype == np.float32 else BF16


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def select(N: int, retrieval: bool, n_sink: int, window: int):
    """Algorithm 1 steps 2-3 for one head -> (kept positions, d_lo, d_hi)."""
    kept = np.empty(max(N, 1), dtype=np.int64)
    lo, hi = ctypes.c_int64(0), ctypes.c_int64(0)
    n = lib().oracle_select(N, int(bool(retrieval)), n_sink, window, _ptr(kept),
                            ctypes.byref(lo), ctypes.byref(hi))
    return kept[:n].copy(), lo.value, hi.value


class OracleCache:
    """Compressed cache as the paper defines it, kept as (positions, khat, vhat, N_d).

    K, V: [B, H_kv, N, d] stored bits (last dim contiguous, any outer strides).
    seq_lens[b] <= N is the valid length of sequence b; mask[h] != 0 marks a
    retrieval KV head.  Compression happens once, here (after prefill); decode
    steps append to every head and never evict.
    """

    def __init__(self, K, V, seq_lens, mask, n_sink: int, window: int, max_new: int = 0):
        self.K, self.V = as_raw(K), as_raw(V)
        assert self.K.shape == self.V.shape and self.K.ndim == 4
        assert self.K.dtype == self.V.dtype
        assert self.K.strides == self.V.strides
        B, H, N, d = self.K.shape
        es = self.K.itemsize
        assert self.K.strides[3] == es
        self.B, self.H, self.N, self.d = B, H, N, d
        self.dtype = _dtype_code(self.K)
        self.strides = tuple(s // es for s in self.K.strides[:3])
        self.seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int64)
        self.mask = np.ascontiguousarray(mask, dtype=np.uint8)
        assert self.seq_lens.shape == (B,) and self.mask.shape == (H,)
        assert (self.seq_lens >= 1).all() and (self.seq_lens <= N).all()
        self.n_sink, self.window = int(n_sink), int(window)

        self.kept = np.empty(int(self.seq_lens.sum()) * H, dtype=np.int64)
        self.kept_off = np.zeros(B * H + 1, dtype=np.int64)
        self.khat = np.zeros((B, H, d), dtype=np.float64)
        self.vhat = np.zeros((B, H, d), dtype=np.float64)
        self.N_d = np.zeros((B, H), dtype=np.int64)
        self.threads = lib().oracle_compress_batch(
            _ptr(self.K), _ptr(self.V), self.dtype, B, H, d, *self.strides,
            _ptr(self.seq_lens), _ptr(self.mask), self.n_sink, self.window,
            _ptr(self.kept), _ptr(self.kept_off), _ptr(self.khat), _ptr(self.vhat),
            _ptr(self.N_d))
        self.kept = self.kept[: self.kept_off[-1]].copy()

        self.cap_new = max(int(max_new), 1)
        self.K_new = np.zeros((B, H, self.cap_new, d), dtype=self.K.dtype)
        self.V_new = np.zeros((B, H, self.cap_new, d), dtype=self.K.dtype)
        self.n_new = 0

    def kept_of(self, b: int, h: int) -> np.ndarray:
        i = b * self.H + h
        return self.kept[self.kept_off[i]: self.kept_off[i + 1]]

    def rows(self) -> np.ndarray:
        """Cached rows per (b, h), compensation entry not counted."""
        return (np.diff(self.kept_off) + self.n_new).reshape(self.B, self.H)

    def append(self, k_new, v_new) -> None:
        k_new, v_new = as_raw(k_new), as_raw(v_new)
        assert k_new.shape == (self.B, self.H, self.d) and k_new.dtype == self.K.dtype
        assert self.n_new < self.cap_new, "append beyond max_new"
        self.K_new[:, :, self.n_new, :] = k_new
        self.V_new[:, :, self.n_new, :] = v_new
        self.n_new += 1

    def decode(self, Q, scale: float, use_comp: bool = True) -> np.ndarray:
        """Eq.(5) for every query head; Q [B, H_q, d] stored bits -> float64."""
        Q = np.ascontiguousarray(as_raw(Q))
        B, Hq, d = Q.shape
        assert B == self.B and d == self.d and Hq % self.H == 0 and Q.dtype == self.K.dtype
        out = np.empty((B, Hq, d), dtype=np.float64)
        N_d = self.N_d if use_comp else np.zeros_like(self.N_d)
        self.threads = lib().oracle_decode_batch(
            _ptr(Q), _ptr(self.K), _ptr(self.V), self.dtype, B, Hq, self.H, d, *self.strides,
            _ptr(self.kept), _ptr(self.kept_off), _ptr(self.K_new), _ptr(self.V_new),
            self.cap_new, self.n_new, _ptr(self.khat), _ptr(self.vhat),
            _ptr(np.ascontiguousarray(N_d)), float(scale), _ptr(out))
        return out
