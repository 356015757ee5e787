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
        L.oracle_comp_token2.restype = None
        L.oracle_comp_token2.argtypes = [vp, vp, ci, i64, ci, i64, i64, vp, vp, i64, i64, i64, vp, vp]
        L.oracle_decode_batch.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, i64, i64, i64,
                                          vp, vp, vp, vp, i64, i64, vp, vp, vp, vp, vp, vp, dbl, vp]
        L.oracle_compress_batch.restype = ci
        L.oracle_compress_batch.argtypes = [vp, vp, ci, ci, ci, ci, i64, i64, i64,
                                            vp, vp, i64, i64, vp, vp, vp, vp, vp, vp]
        L.oracle_head_scores.restype = ci
        L.oracle_head_scores.argtypes = [vp, vp, ci, ci, ci, i64, ci, dbl, i64, ci, vp, vp]
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


def widen(t) -> np.ndarray:
    """Stored fp32 / bf16 values as float64 (exact)."""
    a = as_raw(t)
    if a.dtype == np.uint16:
        a = (a.astype(np.uint32) << 16).view(np.float32)
    return a.astype(np.float64)


def column_sums(K, V, seq_lens) -> np.ndarray:
    """float64 [B, H, 2, d]: sums of the K rows and of the V rows over positions [0, seq_len).
    Together with the sums over the kept rows this gives the numerator of Eq.(4) by
    subtraction, since the dropped and the kept rows partition the sequence."""
    Kd, Vd = widen(K), widen(V)
    B, H, _, d = Kd.shape
    out = np.zeros((B, H, 2, d))
    for b in range(B):
        n = int(seq_lens[b])
        out[b, :, 0] = Kd[b, :, :n].sum(axis=1)
        out[b, :, 1] = Vd[b, :, :n].sum(axis=1)
    return out


def head_scores(Q, K, scale: float, period: int, all_copies: bool = False):
    """Sec. 3.3: (echo, induction) score of every query head, float64 [n_q_heads] each.
    Q [Hq, N, d], K [Hkv, N, d] (after the rotary transformation) for a prompt of `period`
    random tokens repeated to N tokens."""
    q, k = np.ascontiguousarray(as_raw(Q)), np.ascontiguousarray(as_raw(K))
    Hq, N, d = q.shape
    Hkv = k.shape[0]
    assert k.shape == (Hkv, N, d) and q.dtype == k.dtype
    echo, ind = np.zeros(Hq), np.zeros(Hq)
    rc = lib().oracle_head_scores(_ptr(q), _ptr(k), _dtype_code(q), Hq, Hkv, N, d, float(scale), int(period),
                                  int(bool(all_copies)), _ptr(echo), _ptr(ind))
    assert rc == 0, "oracle_head_scores: bad arguments"
    return echo, ind


def protected_count(n_heads: int, frac: float) -> int:
    """How many heads "top frac" of n_heads means: the nearest whole number, halves up."""
    return int(np.floor(frac * n_heads + 0.5))


def select_heads(echo, induction, group: int, frac_induction: float = 0.14, frac_echo: float = 0.01) -> np.ndarray:
    """Sec. 3.3 / Table 2: retrieval heads = the top frac_induction of all heads by induction score
    together with the top frac_echo by echo score (equal scores: the lower head index first).
    Sec. 4.1 (grouped-query models): a KV head is retrieval when any query head of its group is.
    Returns uint8 [n_heads / group]."""
    echo, induction = np.asarray(echo, np.float64), np.asarray(induction, np.float64)
    n = len(echo)
    assert len(induction) == n and n % group == 0
    chosen = np.zeros(n, bool)
    for score, frac in ((induction, frac_induction), (echo, frac_echo)):
        order = sorted(range(n), key=lambda i: (-score[i], i))
        chosen[order[:protected_count(n, frac)]] = True
    return chosen.reshape(n // group, group).any(axis=1).astype(np.uint8)


class OracleCache:
    """Compressed cache as the paper defines it, kept as (positions, khat, vhat, N_d).

    K, V: [B, H_kv, N, d] stored bits (last dim contiguous, any outer strides).
    seq_lens[b] <= N is the valid length of sequence b; mask[h] != 0 marks a
    retrieval KV head.  Compression happens once, here (after prefill); decode
    steps append to every head and never evict.

    sliding=True: Algorithm 1 is re-applied to the whole sequence (prefill + generated
    tokens) after every generated token, so the window slides and the compensation token
    of Eq.(4) absorbs every token that leaves it.  Stated literally: selection and the means
    are recomputed from scratch at each decode.
    """

    def __init__(self, K, V, seq_lens, mask, n_sink: int, window: int, max_new: int = 0,
                 sliding: bool = False, head_window=None, alibi_slopes=None):
        """head_window: buffer length per KV head (overrides `window`); alibi_slopes: l_h of
        Eq.(1) per query head -- the logits then carry -l_h (m - n) and decode must be called
        with use_comp=False (the compensation token has no position)."""
        self.sliding = bool(sliding)
        self.head_window = None if head_window is None else np.ascontiguousarray(head_window, dtype=np.int64)
        self.slopes = None if alibi_slopes is None else np.ascontiguousarray(alibi_slopes, dtype=np.float64)
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
        # sliding mode keeps the sinks inside the prefill (a shorter prefill would turn
        # generated tokens into sinks; not supported by either side)
        assert not self.sliding or (self.seq_lens >= self.n_sink).all()

        self.kept = np.empty(int(self.seq_lens.sum()) * H, dtype=np.int64)
        self.kept_off = np.zeros(B * H + 1, dtype=np.int64)
        self.khat = np.zeros((B, H, d), dtype=np.float64)
        self.vhat = np.zeros((B, H, d), dtype=np.float64)
        self.N_d = np.zeros((B, H), dtype=np.int64)
        self.threads = lib().oracle_compress_batch(
            _ptr(self.K), _ptr(self.V), self.dtype, B, H, d, *self.strides,
            _ptr(self.seq_lens), _ptr(self.mask), self.n_sink, self.window, _ptr(self.head_window),
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
        if self.sliding:
            return np.diff(self._reselect()[1]).reshape(self.B, self.H) + \
                (self.n_new - self._reselect()[2]).reshape(self.B, self.H)
        return (np.diff(self.kept_off) + self.n_new).reshape(self.B, self.H)

    def _reselect(self):
        """Sliding mode: Algorithm 1 steps 2-3 on the sequence as it stands now (seq_len + n_new
        tokens).  Returns kept prefill positions (concatenated), their offsets, the first kept
        appended row per head, and the dropped ranges in both stores."""
        B, H = self.B, self.H
        kept, off = [], np.zeros(B * H + 1, np.int64)
        new_lo = np.zeros(B * H, np.int64)
        d_pre = np.zeros((B * H, 2), np.int64)
        d_new = np.zeros((B * H, 2), np.int64)
        for b in range(B):
            N, T = int(self.seq_lens[b]), int(self.seq_lens[b]) + self.n_new
            for h in range(H):
                i = b * H + h
                win = self.window if self.head_window is None else int(self.head_window[h])
                idx, lo, hi = select(T, bool(self.mask[h]), self.n_sink, win)
                pre = idx[idx < N]
                app = idx[idx >= N] - N
                # kept appended rows are a suffix: everything older has moved into the dropped set
                assert len(app) == 0 or (app == np.arange(app[0], self.n_new)).all()
                new_lo[i] = app[0] if len(app) else self.n_new
                kept.append(pre)
                off[i + 1] = off[i] + len(pre)
                d_pre[i] = (min(lo, N), min(hi, N))
                d_new[i] = (max(lo, N) - N, max(hi, N) - N)
        kept = np.concatenate(kept) if kept else np.zeros(0, np.int64)
        return np.ascontiguousarray(kept, dtype=np.int64), off, new_lo, d_pre, d_new

    def _recompute_tokens(self):
        """Sliding mode: Eq.(4) from scratch over the dropped set as it stands now."""
        kept, off, new_lo, d_pre, d_new = self._reselect()
        B, H, d = self.B, self.H, self.d
        es = self.K.itemsize
        khat = np.zeros((B, H, d)); vhat = np.zeros((B, H, d)); N_d = np.zeros((B, H), np.int64)
        for b in range(B):
            for h in range(H):
                i = b * H + h
                n = int(d_pre[i, 1] - d_pre[i, 0] + d_new[i, 1] - d_new[i, 0])
                N_d[b, h] = n
                if n == 0:
                    continue
                kh, vh = np.zeros(d), np.zeros(d)
                lib().oracle_comp_token2(
                    self.K.ctypes.data + (b * self.strides[0] + h * self.strides[1]) * es,
                    self.V.ctypes.data + (b * self.strides[0] + h * self.strides[1]) * es,
                    self.dtype, self.strides[2], d, int(d_pre[i, 0]), int(d_pre[i, 1]),
                    self.K_new.ctypes.data + i * self.cap_new * d * es,
                    self.V_new.ctypes.data + i * self.cap_new * d * es, d,
                    int(d_new[i, 0]), int(d_new[i, 1]), _ptr(kh), _ptr(vh))
                khat[b, h], vhat[b, h] = kh, vh
        return kept, off, new_lo, khat, vhat, N_d

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
        if self.sliding:
            self.kept, self.kept_off, new_lo, self.khat, self.vhat, self.N_d = self._recompute_tokens()
        else:
            new_lo = None
        N_d = self.N_d if use_comp else np.zeros_like(self.N_d)
        assert self.slopes is None or (not use_comp and self.slopes.shape == (Hq,))
        self.threads = lib().oracle_decode_batch(
            _ptr(Q), _ptr(self.K), _ptr(self.V), self.dtype, B, Hq, self.H, d, *self.strides,
            _ptr(self.kept), _ptr(self.kept_off), _ptr(self.K_new), _ptr(self.V_new),
            self.cap_new, self.n_new, _ptr(new_lo), _ptr(np.ascontiguousarray(self.khat)),
            _ptr(np.ascontiguousarray(self.vhat)), _ptr(np.ascontiguousarray(N_d)),
            _ptr(self.slopes), _ptr(self.seq_lens), float(scale), _ptr(out))
        return out
