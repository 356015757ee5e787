"""Python binding of the razor C-ABI library (RazorAttention hot path on MI355X).

The functions `razor_plan`, `razor_compress`, `razor_column_sums`, `razor_decode_attn`,
`razor_decode_attn_static`, `razor_head_scores`, `razor_head_scores_workspace`, `razor_select_heads`
and `razor_strerror` carry the names and the argument order of `include/razor.h`
(`razor_profile_events`, `razor_probe_read_stream`, `razor_probe_copy`: `include/razor_bench.h`); they only marshal
arguments (torch tensors -> device pointers, numpy arrays -> host pointers).  Every
step of the path runs in the HIP kernels of `librazor.so`; there is no Python or CPU
fallback: a missing library raises on first use.

`RazorCache` is a convenience holder for the buffers one layer needs (torch is used
for device memory and streams only).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("RAZOR_LIBRARY", os.path.join(_HERE, "librazor.so"))   # override: debug builds

RAZOR_F32, RAZOR_BF16 = 0, 1
RAZOR_OK, RAZOR_EINVAL, RAZOR_ECAPACITY, RAZOR_EHIP = 0, -1, -2, -3
RAZOR_HEAD_RETRIEVAL, RAZOR_HEAD_COMP, RAZOR_HEAD_OVERFLOW = 1, 2, 4
RAZOR_BLOCK_ROWS = 16
RAZOR_MAX_GROUP = 16
RAZOR_MAX_WORKERS = 8192

RAZOR_MAX_HEADS = 65535
RAZOR_STATIC_SCRATCH_BYTES = 8 << 20
RAZOR_PROBE_CONTIGUOUS, RAZOR_PROBE_INTERLEAVED = 0, 1

# include/razor.h, then the measurement hooks of include/razor_bench.h
EXPORTS = ("razor_plan", "razor_compress", "razor_column_sums", "razor_decode_attn",
           "razor_decode_attn_static", "razor_head_scores_workspace", "razor_head_scores",
           "razor_select_heads", "razor_strerror",
           "razor_profile_events", "razor_probe_read_stream", "razor_probe_copy")


class RazorParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("n_sink", ctypes.c_int32), ("window", ctypes.c_int32),
                ("max_new", ctypes.c_int32), ("use_comp", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("scale", ctypes.c_float), ("n_workers", ctypes.c_int32),
                ("sliding", ctypes.c_int32), ("reserved0", ctypes.c_int32),
                ("head_window_host", ctypes.c_void_p), ("alibi_slopes", ctypes.c_void_p)]


class RazorHeadDesc(ctypes.Structure):
    _fields_ = [("row_off", ctypes.c_int64), ("kept_off", ctypes.c_int64),
                ("rows", ctypes.c_int32), ("cap", ctypes.c_int32),
                ("n_dropped", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("evicted", ctypes.c_int32), ("window", ctypes.c_int32),
                ("reserved", ctypes.c_int32 * 2)]


class RazorSizes(ctypes.Structure):
    _fields_ = [("arena_bytes", ctypes.c_uint64), ("comp_bytes", ctypes.c_uint64),
                ("desc_bytes", ctypes.c_uint64), ("kept_idx_bytes", ctypes.c_uint64),
                ("workspace_bytes", ctypes.c_uint64), ("total_rows", ctypes.c_int64),
                ("total_cap", ctypes.c_int64)]


DESC_DTYPE = np.dtype([("row_off", "<i8"), ("kept_off", "<i8"), ("rows", "<i4"), ("cap", "<i4"),
                       ("n_dropped", "<i4"), ("flags", "<u4"), ("evicted", "<i4"), ("window", "<i4"),
                       ("reserved", "<i4", (2,))])
assert DESC_DTYPE.itemsize == ctypes.sizeof(RazorHeadDesc) == 48


class RazorError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {razor_strerror(status)} (status {status})")


_lib = None


def load_library():
    """Load librazor.so (built by `__graft_entry__.build()`); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: run `python __graft_entry__.py` to build the HIP "
                           "library; there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    PP = ctypes.POINTER(RazorParams)
    L.razor_plan.restype = ctypes.c_int
    L.razor_plan.argtypes = [PP, vp, vp, vp, vp, ctypes.POINTER(RazorSizes)]
    L.razor_compress.restype = ctypes.c_int
    L.razor_compress.argtypes = [PP, vp, vp, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.razor_column_sums.restype = ctypes.c_int
    L.razor_column_sums.argtypes = [PP, vp, vp, i64, i64, i64, vp, vp, vp, sz, vp]
    L.razor_decode_attn.restype = ctypes.c_int
    L.razor_decode_attn.argtypes = [PP, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.razor_decode_attn_static.restype = ctypes.c_int
    L.razor_decode_attn_static.argtypes = [PP, vp, vp, vp, vp, vp, vp, vp, vp]
    ci = ctypes.c_int
    L.razor_head_scores_workspace.restype = sz
    L.razor_head_scores_workspace.argtypes = [ci, ci]
    L.razor_head_scores.restype = ci
    L.razor_head_scores.argtypes = [vp, vp, ci, ci, ci, ci, ci, i64, i64, i64, i64, ctypes.c_float, ci, ci,
                                    vp, vp, vp, sz, vp]
    L.razor_select_heads.restype = ci
    L.razor_select_heads.argtypes = [vp, vp, ci, ci, ctypes.c_double, ctypes.c_double, vp]
    L.razor_profile_events.restype = ctypes.c_int
    L.razor_profile_events.argtypes = [vp, vp]
    L.razor_probe_read_stream.restype = ctypes.c_int
    L.razor_probe_read_stream.argtypes = [vp, sz, ci, ci, ci, ci, vp, vp]
    L.razor_probe_copy.restype = ctypes.c_int
    L.razor_probe_copy.argtypes = [vp, vp, sz, ci, ci, ci, vp]
    L.razor_strerror.restype = ctypes.c_char_p
    L.razor_strerror.argtypes = [ctypes.c_int]
    _lib = L
    return L


def _dev(t) -> Optional[int]:
    """Device pointer of a torch tensor (None -> NULL)."""
    return None if t is None else t.data_ptr()


def _host(a) -> Optional[int]:
    return None if a is None else a.ctypes.data


def razor_strerror(status: int) -> str:
    return load_library().razor_strerror(int(status)).decode()


def razor_plan(params: RazorParams, seq_lens_host: np.ndarray, retrieval_mask_host: np.ndarray,
               desc_host: Optional[np.ndarray] = None, kept_idx_host: Optional[np.ndarray] = None,
               sizes: Optional[RazorSizes] = None) -> int:
    """Host-only planner.  seq_lens_host int32[B], retrieval_mask_host uint8[H_kv],
    desc_host DESC_DTYPE[B*H_kv] (optional), kept_idx_host int32[total_rows] (optional)."""
    assert seq_lens_host.dtype == np.int32 and retrieval_mask_host.dtype == np.uint8
    assert desc_host is None or (desc_host.dtype == DESC_DTYPE and desc_host.flags.c_contiguous)
    assert kept_idx_host is None or kept_idx_host.dtype == np.int32
    return load_library().razor_plan(ctypes.byref(params), _host(seq_lens_host),
                                     _host(retrieval_mask_host), _host(desc_host),
                                     _host(kept_idx_host),
                                     ctypes.byref(sizes) if sizes is not None else None)


def razor_compress(params: RazorParams, K, V, stride_b: int, stride_h: int, stride_n: int,
                   seq_lens_host: np.ndarray, retrieval_mask_host: np.ndarray, arena, comp,
                   desc_dev, kept_idx_dev, col_sums, workspace, workspace_bytes: int,
                   stream: int = 0) -> int:
    assert seq_lens_host.dtype == np.int32 and retrieval_mask_host.dtype == np.uint8
    return load_library().razor_compress(
        ctypes.byref(params), _dev(K), _dev(V), stride_b, stride_h, stride_n,
        _host(seq_lens_host), _host(retrieval_mask_host), _dev(arena), _dev(comp), _dev(desc_dev),
        _dev(kept_idx_dev), _dev(col_sums), _dev(workspace), workspace_bytes, stream or None)


def razor_column_sums(params: RazorParams, K, V, stride_b: int, stride_h: int, stride_n: int,
                      seq_lens_host: np.ndarray, col_sums, workspace, workspace_bytes: int,
                      stream: int = 0) -> int:
    assert seq_lens_host.dtype == np.int32
    return load_library().razor_column_sums(
        ctypes.byref(params), _dev(K), _dev(V), stride_b, stride_h, stride_n, _host(seq_lens_host),
        _dev(col_sums), _dev(workspace), workspace_bytes, stream or None)


def razor_decode_attn(params: RazorParams, Q, k_new, v_new, arena, comp, desc_dev, O, workspace,
                      workspace_bytes: int, stream: int = 0) -> int:
    return load_library().razor_decode_attn(
        ctypes.byref(params), _dev(Q), _dev(k_new), _dev(v_new), _dev(arena), _dev(comp),
        _dev(desc_dev), _dev(O), _dev(workspace), workspace_bytes, stream or None)


def razor_decode_attn_static(params: RazorParams, Q, k_new, v_new, arena, comp, desc_dev, O,
                             stream: int = 0) -> int:
    return load_library().razor_decode_attn_static(
        ctypes.byref(params), _dev(Q), _dev(k_new), _dev(v_new), _dev(arena), _dev(comp),
        _dev(desc_dev), _dev(O), stream or None)


def razor_head_scores_workspace(n_q_heads: int, n_tokens: int) -> int:
    return load_library().razor_head_scores_workspace(n_q_heads, n_tokens)


def razor_head_scores(Q, K, dtype: int, n_q_heads: int, n_kv_heads: int, head_dim: int, n_tokens: int,
                      q_stride_h: int, q_stride_n: int, k_stride_h: int, k_stride_n: int, scale: float,
                      period: int, all_copies: int, echo, induction, workspace, workspace_bytes: int,
                      stream: int = 0) -> int:
    return load_library().razor_head_scores(
        _dev(Q), _dev(K), dtype, n_q_heads, n_kv_heads, head_dim, n_tokens, q_stride_h, q_stride_n,
        k_stride_h, k_stride_n, scale, period, all_copies, _dev(echo), _dev(induction), _dev(workspace),
        workspace_bytes, stream or None)


def razor_select_heads(echo_host: np.ndarray, induction_host: np.ndarray, n_heads: int, group: int,
                       frac_induction: float, frac_echo: float, mask_host: np.ndarray) -> int:
    assert echo_host.dtype == np.float32 and induction_host.dtype == np.float32 and mask_host.dtype == np.uint8
    return load_library().razor_select_heads(_host(echo_host), _host(induction_host), n_heads, group,
                                             frac_induction, frac_echo, _host(mask_host))


def razor_profile_events(ev_start, ev_stop) -> int:
    """ev_start / ev_stop: raw hipEvent_t handles (ctypes.c_void_p) or None."""
    return load_library().razor_profile_events(ev_start, ev_stop)


def razor_probe_read_stream(buf, nbytes: int, n_workers: int, pattern: int, depth: int, nontemporal: int,
                            sink, stream: int = 0) -> int:
    """buf: device tensor, or a raw device address (int) inside one."""
    addr = buf if isinstance(buf, int) else _dev(buf)
    return load_library().razor_probe_read_stream(addr, nbytes, n_workers, pattern, depth, nontemporal,
                                                  _dev(sink), stream or None)


def razor_probe_copy(dst, src, nbytes: int, n_workers: int, pattern: int, nontemporal: int,
                     stream: int = 0) -> int:
    """dst, src: device tensors, or raw device addresses (int)."""
    d = dst if isinstance(dst, int) else _dev(dst)
    s = src if isinstance(src, int) else _dev(src)
    return load_library().razor_probe_copy(d, s, nbytes, n_workers, pattern, nontemporal, stream or None)


def _check(status: int, where: str) -> None:
    if status != RAZOR_OK:
        raise RazorError(status, where)


def head_scores(Q, K, scale: float, period: int, all_copies: bool = False):
    """(echo, induction) float32 device tensors [H_q] for Q [H_q, N, d], K [H_kv, N, d] (bf16 device
    tensors, last dimension contiguous) of a prompt that repeats every `period` tokens."""
    import torch
    assert Q.dtype == torch.bfloat16 and K.dtype == torch.bfloat16 and Q.stride(2) == 1 and K.stride(2) == 1
    Hq, N, d = Q.shape
    assert K.shape[1:] == (N, d)
    ws_bytes = razor_head_scores_workspace(Hq, N)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=Q.device)
    echo = torch.empty(Hq, dtype=torch.float32, device=Q.device)
    induction = torch.empty(Hq, dtype=torch.float32, device=Q.device)
    _check(razor_head_scores(Q, K, RAZOR_BF16, Hq, K.shape[0], d, N, Q.stride(0), Q.stride(1), K.stride(0),
                             K.stride(1), scale, period, int(bool(all_copies)), echo, induction, ws, ws.numel(),
                             torch.cuda.current_stream(Q.device).cuda_stream), "razor_head_scores")
    return echo, induction


def select_heads(echo, induction, group: int, frac_induction: float = 0.14, frac_echo: float = 0.01) -> np.ndarray:
    """uint8 retrieval mask [n_heads / group] from per-query-head scores (host arrays, all layers)."""
    e = np.ascontiguousarray(echo, dtype=np.float32)
    i = np.ascontiguousarray(induction, dtype=np.float32)
    assert e.ndim == 1 and e.shape == i.shape
    mask = np.zeros(max(len(e) // max(group, 1), 1), np.uint8)
    _check(razor_select_heads(e, i, len(e), group, frac_induction, frac_echo, mask), "razor_select_heads")
    return mask


class RazorCache:
    """Buffers of one layer's compressed cache plus the calls that fill and read them."""

    def __init__(self, *, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                 seq_lens, retrieval_mask, n_sink: int, window: int, max_new: int,
                 dtype, scale: Optional[float] = None, out_dtype=None, use_comp: bool = True,
                 n_workers: int = 0, device="cuda", want_kept_idx: bool = False,
                 sliding: bool = False, head_window=None, alibi_slopes=None):
        """head_window: buffer length per KV head (int array, overrides `window`);
        alibi_slopes: float32 device tensor [n_q_heads] (selects Eq.(1) logits; use_comp must be False)."""
        import torch
        self.torch = torch
        code = {torch.float32: RAZOR_F32, torch.bfloat16: RAZOR_BF16}
        self.dtype = dtype
        self.out_dtype = out_dtype or torch.float32
        self.params = RazorParams(batch, n_q_heads, n_kv_heads, head_dim, n_sink, window, max_new,
                                  int(use_comp), code[dtype], code[self.out_dtype],
                                  float(scale if scale is not None else head_dim ** -0.5), n_workers,
                                  int(sliding), 0, None, None)
        # the params struct points at these: keep them alive with the cache
        self.head_window = None if head_window is None else np.ascontiguousarray(head_window, dtype=np.int32)
        self.alibi_slopes = alibi_slopes
        if self.head_window is not None:
            assert self.head_window.shape == (n_kv_heads,)
            self.params.head_window_host = self.head_window.ctypes.data
        if alibi_slopes is not None:
            assert alibi_slopes.dtype == torch.float32 and alibi_slopes.is_contiguous()
            assert tuple(alibi_slopes.shape) == (n_q_heads,) and alibi_slopes.device.type == "cuda"
            self.params.alibi_slopes = alibi_slopes.data_ptr()
        self.seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
        self.mask = np.ascontiguousarray(retrieval_mask, dtype=np.uint8)
        assert self.seq_lens.shape == (batch,) and self.mask.shape == (n_kv_heads,)
        self.sizes = RazorSizes()
        self.desc_host = np.zeros(batch * n_kv_heads, dtype=DESC_DTYPE)
        _check(razor_plan(self.params, self.seq_lens, self.mask, self.desc_host, None, self.sizes),
               "razor_plan")
        self.device = torch.device(device)
        u8 = dict(dtype=torch.uint8, device=self.device)
        self.arena = torch.empty(max(int(self.sizes.arena_bytes), 16), **u8)
        self.comp = torch.empty(int(self.sizes.comp_bytes) // 4, dtype=torch.float32, device=self.device)
        self.desc_dev = torch.empty(int(self.sizes.desc_bytes), **u8)
        self.workspace = torch.empty(int(self.sizes.workspace_bytes), **u8)
        self.kept_idx_dev = (torch.empty(max(int(self.sizes.total_rows), 1), dtype=torch.int32,
                                         device=self.device) if want_kept_idx else None)
        self.n_appended = 0

    @classmethod
    def from_workload(cls, w, **kw):
        return cls(batch=w.B, n_q_heads=w.Hq, n_kv_heads=w.Hkv, head_dim=w.d, seq_lens=w.seq_lens,
                   retrieval_mask=w.mask, n_sink=w.n_sink, window=w.window, max_new=w.max_new,
                   dtype=w.dtype, scale=w.scale, device=w.device, **kw)

    def _stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def _check_source(self, K, V) -> None:
        assert K.dtype == self.dtype and V.dtype == self.dtype and K.stride() == V.stride()
        assert K.stride(3) == 1 and K.shape[:2] == (self.params.batch, self.params.n_kv_heads)
        assert K.shape[2] >= int(self.seq_lens.max()) and K.shape[3] == self.params.head_dim

    def column_sums(self, K, V):
        """float32 [B, H_kv, 2, d]: sums of K and V over the valid rows (what a prefill epilogue gives)."""
        self._check_source(K, V)
        p = self.params
        out = self.torch.empty(p.batch, p.n_kv_heads, 2, p.head_dim, dtype=self.torch.float32, device=self.device)
        _check(razor_column_sums(p, K, V, K.stride(0), K.stride(1), K.stride(2), self.seq_lens, out,
                                 self.workspace, self.workspace.numel(), self._stream()), "razor_column_sums")
        return out

    def compress(self, K, V, col_sums=None) -> None:
        """K, V: [B, H_kv, N, d] device tensors, last dimension contiguous.  col_sums: optional
        float32 [B, H_kv, 2, d] sums over the valid rows; with it the dropped rows are not read."""
        self._check_source(K, V)
        if col_sums is not None:
            p = self.params
            assert col_sums.dtype == self.torch.float32 and col_sums.is_contiguous()
            assert tuple(col_sums.shape) == (p.batch, p.n_kv_heads, 2, p.head_dim)
        _check(razor_compress(self.params, K, V, K.stride(0), K.stride(1), K.stride(2), self.seq_lens,
                              self.mask, self.arena, self.comp, self.desc_dev, self.kept_idx_dev, col_sums,
                              self.workspace, self.workspace.numel(), self._stream()), "razor_compress")
        self.n_appended = 0

    def decode(self, Q, k_new=None, v_new=None, out=None):
        """One decode step; returns O [B, H_q, d]."""
        p = self.params
        assert Q.dtype == self.dtype and Q.is_contiguous() and tuple(Q.shape) == (p.batch, p.n_q_heads, p.head_dim)
        if k_new is not None:
            assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.dtype == self.dtype
            assert tuple(k_new.shape) == (p.batch, p.n_kv_heads, p.head_dim) == tuple(v_new.shape)
            if self.n_appended >= p.max_new:
                raise RazorError(RAZOR_ECAPACITY, "RazorCache.decode: max_new appends already stored")
            self.n_appended += 1
        if out is None:
            out = self.torch.empty(p.batch, p.n_q_heads, p.head_dim, dtype=self.out_dtype, device=self.device)
        _check(razor_decode_attn(p, Q, k_new, v_new, self.arena, self.comp, self.desc_dev, out,
                                 self.workspace, self.workspace.numel(), self._stream()), "razor_decode_attn")
        return out

    def comp_tokens(self):
        """khat, vhat of Eq.(4) as a [B, H_kv, 2, d] view of `comp` (in sliding mode the buffer also
        holds the low-order parts of the running means behind them)."""
        p = self.params
        n = p.batch * p.n_kv_heads * 2 * p.head_dim
        return self.comp[:n].view(p.batch, p.n_kv_heads, 2, p.head_dim)

    def desc(self) -> np.ndarray:
        """Device descriptor table copied to the host (synchronises)."""
        return self.desc_dev.cpu().numpy().view(DESC_DTYPE).copy()
