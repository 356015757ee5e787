"""CPU-only checks of the HIP library's host side: it loads, exports what the header
declares, plans exactly the table the oracle derives from Algorithm 1, and turns bad
arguments into error codes before touching a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2407_15891_amd as razor
from oracle import razor_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def params(**kw):
    base = dict(batch=2, n_q_heads=8, n_kv_heads=4, head_dim=128, n_sink=4, window=32, max_new=8,
                use_comp=1, dtype=razor.RAZOR_BF16, out_dtype=razor.RAZOR_F32, scale=0.088, n_workers=0,
                sliding=0, reserved0=0, head_window_host=None, alibi_slopes=None)
    base.update(kw)
    return razor.RazorParams(**base)


def plan(p, seq_lens, mask, want_idx=True):
    seq_lens = np.asarray(seq_lens, np.int32)
    mask = np.asarray(mask, np.uint8)
    sizes = razor.RazorSizes()
    rc = razor.razor_plan(p, seq_lens, mask, None, None, sizes)
    if rc != razor.RAZOR_OK:
        return rc, None, None, None
    desc = np.zeros(p.batch * p.n_kv_heads, razor.DESC_DTYPE)
    idx = np.zeros(max(sizes.total_rows, 1), np.int32) if want_idx else None
    rc = razor.razor_plan(p, seq_lens, mask, desc, idx, sizes)
    return rc, desc, idx, sizes


def test_library_exports_every_declared_symbol():
    lib = razor.load_library()
    declared = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):       # razor.h and razor_bench.h
        header = open(os.path.join(ROOT, "include", name)).read()
        declared |= set(re.findall(r"^RAZOR_API [^;]*?\b(razor_[a-z_]+)\s*\(", header, re.M | re.S))
    assert len(declared) == 12 and declared == set(razor.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert razor.razor_strerror(razor.RAZOR_OK) == "ok"
    assert "invalid" in razor.razor_strerror(razor.RAZOR_EINVAL)
    assert "workspace" in razor.razor_strerror(razor.RAZOR_ECAPACITY)
    assert ctypes.sizeof(razor.RazorHeadDesc) == 48 and ctypes.sizeof(razor.RazorParams) == 72


@pytest.mark.parametrize("seq_lens,mask,n_sink,window", [
    ([2048], [1, 0, 0, 0, 0, 1, 0, 0], 4, 256),           # config 1
    ([100, 37, 5, 36], [0, 1, 0, 0], 4, 32),               # ragged; 36 = exactly covered; 37 drops one
    ([64, 64], [0, 0, 0, 0], 0, 16),                       # no sinks
    ([64, 64], [0, 0, 1, 0], 4, 0),                        # no window
    ([50, 1], [0, 0, 0, 0], 0, 0),                         # nothing kept but the compensation token
    ([131072, 131072], [0, 1, 0, 0], 4, 19660),            # config 3 lengths
])
def test_plan_matches_oracle_table(seq_lens, mask, n_sink, window):
    B, H = len(seq_lens), len(mask)
    p = params(batch=B, n_kv_heads=H, n_q_heads=H, n_sink=n_sink, window=window)
    rc, desc, idx, sizes = plan(p, seq_lens, mask)
    assert rc == razor.RAZOR_OK
    total = 0
    for b in range(B):
        for h in range(H):
            e = desc[b * H + h]
            kept, lo, hi = orc.select(seq_lens[b], bool(mask[h]), n_sink, window)
            assert e["rows"] == len(kept) and e["n_dropped"] == hi - lo          # bit-exact lengths
            assert e["kept_off"] == total
            np.testing.assert_array_equal(idx[total: total + len(kept)], kept)   # bit-exact positions
            assert bool(e["flags"] & razor.RAZOR_HEAD_RETRIEVAL) == bool(mask[h])
            assert bool(e["flags"] & razor.RAZOR_HEAD_COMP) == (hi > lo)
            total += len(kept)
    assert sizes.total_rows == total
    # layout: regions are disjoint, in order, block-aligned, with room for the appends
    off = 0
    for e in desc:
        assert e["row_off"] == off and e["cap"] % razor.RAZOR_BLOCK_ROWS == 0
        assert e["rows"] + p.max_new <= e["cap"] < e["rows"] + p.max_new + razor.RAZOR_BLOCK_ROWS
        off += e["cap"]
    assert sizes.total_cap == off
    assert sizes.arena_bytes == off * 2 * p.head_dim * 2
    assert sizes.comp_bytes == B * H * 2 * p.head_dim * 4 and sizes.desc_bytes == B * H * 48
    assert sizes.kept_idx_bytes == 4 * total and sizes.workspace_bytes > 0


def test_plan_reproduces_table2_ratio():
    # 15 % retrieval heads, buffer max(4000, N/5), 4 sinks -> 3.125x (Table 2 caption)
    N, H = 1_000_000, 20
    mask = np.zeros(H, np.uint8); mask[:3] = 1
    p = params(batch=1, n_kv_heads=H, n_q_heads=H, n_sink=4, window=max(4000, N // 5), max_new=0)
    rc, desc, _, sizes = plan(p, [N], mask, want_idx=False)
    assert rc == razor.RAZOR_OK
    assert H * N / sizes.total_rows == pytest.approx(3.125, rel=1e-4)


@pytest.mark.parametrize("kw", [
    dict(head_dim=96), dict(head_dim=256), dict(n_q_heads=6), dict(n_q_heads=4 * 32), dict(batch=0),
    dict(n_sink=-1), dict(window=-1), dict(max_new=-1), dict(dtype=2), dict(out_dtype=7),
    dict(use_comp=2), dict(scale=0.0), dict(scale=float("nan")), dict(n_workers=-1),
    dict(n_workers=razor.RAZOR_MAX_WORKERS + 1), dict(sliding=2), dict(sliding=1, window=0),
    dict(reserved0=1), dict(alibi_slopes=4096),          # slopes with use_comp = 1
])
def test_bad_params_are_rejected(kw):
    p = params(**kw)
    sizes = razor.RazorSizes()
    seq = np.full(max(p.batch, 1), 100, np.int32)
    mask = np.zeros(p.n_kv_heads, np.uint8)
    assert razor.razor_plan(p, seq, mask, None, None, sizes) == razor.RAZOR_EINVAL


def test_bad_arguments_are_rejected_before_any_gpu_work():
    p = params()
    seq = np.array([100, 0], np.int32)            # empty sequence
    mask = np.zeros(4, np.uint8)
    sizes = razor.RazorSizes()
    assert razor.razor_plan(p, seq, mask, None, None, sizes) == razor.RAZOR_EINVAL
    assert razor.razor_plan(p, seq, mask, None, None, None) == razor.RAZOR_EINVAL
    L = razor.load_library()
    pp = ctypes.byref(p)
    seq = np.array([100, 100], np.int32)
    fake = 4096   # never dereferenced: validation fails first
    # null tensors
    assert L.razor_compress(pp, None, fake, 1, 1, 128, seq.ctypes.data, mask.ctypes.data, fake, fake,
                            fake, None, None, fake, 1 << 30, None) == razor.RAZOR_EINVAL
    # row stride shorter than a row / misaligned stride / misaligned pointer
    for strides, k in (((100 * 64, 64, 64), fake), ((100 * 132, 132 * 100, 132), fake),
                       ((100 * 128 * 4, 100 * 128, 128), fake + 2)):
        assert L.razor_compress(pp, k, fake, *strides, seq.ctypes.data, mask.ctypes.data, fake, fake,
                                fake, None, None, fake, 1 << 30, None) == razor.RAZOR_EINVAL
        assert L.razor_column_sums(pp, k, fake, *strides, seq.ctypes.data, fake, fake, 1 << 30, None) == razor.RAZOR_EINVAL
    # workspace too small
    assert L.razor_compress(pp, fake, fake, 4 * 100 * 128, 100 * 128, 128, seq.ctypes.data,
                            mask.ctypes.data, fake, fake, fake, None, None, fake, 16, None) == razor.RAZOR_ECAPACITY
    assert L.razor_column_sums(pp, fake, fake, 4 * 100 * 128, 100 * 128, 128, seq.ctypes.data, fake, fake, 16,
                               None) == razor.RAZOR_ECAPACITY
    assert L.razor_decode_attn(pp, fake, None, None, fake, fake, fake, fake, fake, 16, None) == razor.RAZOR_ECAPACITY
    assert L.razor_decode_attn(pp, None, None, None, fake, fake, fake, fake, fake, 1 << 30, None) == razor.RAZOR_EINVAL
    # k_new without v_new
    assert L.razor_decode_attn(pp, fake, fake, None, fake, fake, fake, fake, fake, 1 << 30, None) == razor.RAZOR_EINVAL
    # a descriptor table that is not 16-byte aligned (its entries are fetched with 128-bit loads)
    assert L.razor_decode_attn(pp, fake, None, None, fake, fake, fake + 8, fake, fake, 1 << 30, None) == razor.RAZOR_EINVAL
    assert L.razor_compress(pp, fake, fake, 4 * 100 * 128, 100 * 128, 128, seq.ctypes.data, mask.ctypes.data, fake,
                            fake, fake + 8, None, None, fake, 1 << 30, None) == razor.RAZOR_EINVAL
    # the variant that owns its scratch: same checks, and a step that does not fit is refused
    assert L.razor_decode_attn_static(pp, None, None, None, fake, fake, fake, fake, None) == razor.RAZOR_EINVAL
    assert L.razor_decode_attn_static(pp, fake, fake, None, fake, fake, fake, fake, None) == razor.RAZOR_EINVAL
    big = params(batch=64, n_kv_heads=8, n_q_heads=128, n_workers=razor.RAZOR_MAX_WORKERS)   # 8704 slots x 16 x 130 floats
    assert L.razor_decode_attn_static(ctypes.byref(big), fake, None, None, fake, fake, fake, fake, None) == razor.RAZOR_ECAPACITY
    assert "razor_decode_attn_static" in razor.razor_strerror(razor.RAZOR_ECAPACITY)


def test_more_heads_than_a_launch_can_index_are_rejected_up_front():
    """(sequence, KV head) pairs index one grid dimension of the compaction launches (limit 65535):
    a call beyond that must fail in validation, not at a launch after other work was enqueued."""
    ok = params(batch=65535 // 8, n_kv_heads=8, n_q_heads=8)
    bad = params(batch=70000 // 8, n_kv_heads=8, n_q_heads=8)             # 70 000 pairs
    sizes = razor.RazorSizes()
    mask = np.zeros(8, np.uint8)
    assert razor.razor_plan(ok, np.full(ok.batch, 40, np.int32), mask, None, None, sizes) == razor.RAZOR_OK
    seq = np.full(bad.batch, 40, np.int32)
    assert razor.razor_plan(bad, seq, mask, None, None, sizes) == razor.RAZOR_EINVAL
    L = razor.load_library()
    fake, pp = 4096, ctypes.byref(bad)
    assert L.razor_compress(pp, fake, fake, 8 * 40 * 128, 40 * 128, 128, seq.ctypes.data, mask.ctypes.data, fake,
                            fake, fake, None, None, fake, 1 << 40, None) == razor.RAZOR_EINVAL
    assert L.razor_column_sums(pp, fake, fake, 8 * 40 * 128, 40 * 128, 128, seq.ctypes.data, fake, fake, 1 << 40,
                               None) == razor.RAZOR_EINVAL
    assert L.razor_decode_attn(pp, fake, None, None, fake, fake, fake, fake, fake, 1 << 40, None) == razor.RAZOR_EINVAL
    assert L.razor_decode_attn_static(pp, fake, None, None, fake, fake, fake, fake, None) == razor.RAZOR_EINVAL


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(razor, "_lib", None)
    monkeypatch.setattr(razor, "LIB_PATH", "/nonexistent/librazor.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        razor.load_library()


def test_plan_sliding_mode_caps_the_window_heads():
    # sliding: a non-retrieval head never holds more than n_sink + window rows
    p = params(batch=3, n_kv_heads=2, n_q_heads=2, n_sink=4, window=32, max_new=1000, sliding=1)
    rc, desc, _, sizes = plan(p, [500, 20, 36], [0, 1], want_idx=False)
    assert rc == razor.RAZOR_OK
    rows = desc["rows"].reshape(3, 2).tolist()
    cap = desc["cap"].reshape(3, 2).tolist()
    assert rows == [[36, 500], [20, 20], [36, 36]]
    assert cap == [[48, 1504], [48, 1024], [48, 1040]]          # 36 -> 48; retrieval: rows + 1000 rounded up
    assert (desc["evicted"] == 0).all()
    # the sinks must lie inside the prefill
    assert plan(p, [500, 3, 36], [0, 1], want_idx=False)[0] == razor.RAZOR_EINVAL


def test_plan_per_head_windows_match_oracle():
    # ALiBi models: one buffer length (vision scope) per KV head, no sinks
    hw = np.array([5, 1000, 64, 0], np.int32)
    p = params(batch=2, n_kv_heads=4, n_q_heads=8, n_sink=0, window=7, use_comp=0, head_window_host=hw.ctypes.data)
    rc, desc, idx, sizes = plan(p, [300, 40], [0, 0, 0, 0])
    assert rc == razor.RAZOR_OK
    total = 0
    for b, N in enumerate([300, 40]):
        for h in range(4):
            e = desc[b * 4 + h]
            kept, lo, hi = orc.select(N, False, 0, int(hw[h]))
            assert e["rows"] == len(kept) and e["n_dropped"] == hi - lo and e["window"] == hw[h]
            np.testing.assert_array_equal(idx[total: total + len(kept)], kept)
            total += len(kept)
    assert desc["rows"].reshape(2, 4).tolist() == [[5, 300, 64, 0], [5, 40, 40, 0]]
    hw_bad = np.array([5, -1, 64, 0], np.int32)
    assert razor.razor_plan(params(n_kv_heads=4, head_window_host=hw_bad.ctypes.data), np.array([300, 40], np.int32),
                            np.zeros(4, np.uint8), None, None, razor.RazorSizes()) == razor.RAZOR_EINVAL


def test_plan_random_tables_match_oracle():
    """Seeded sweep over lengths, masks, sinks, windows (global and per head), static and sliding."""
    rng = np.random.default_rng(2024)
    for trial in range(300):
        B, H = int(rng.integers(1, 6)), int(rng.integers(1, 9))
        n_sink = int(rng.choice([0, 1, 4, 9]))
        sliding = int(rng.integers(0, 2))
        window = int(rng.choice([1, 2, 15, 16, 17, 100, 5000]))
        lens = rng.integers(max(1, n_sink if sliding else 1), 400, size=B).astype(np.int32)
        mask = (rng.random(H) < 0.3).astype(np.uint8)
        hw = rng.choice([1, 3, 16, 64, 10 ** 6], size=H).astype(np.int32) if rng.random() < 0.4 else None
        max_new = int(rng.choice([0, 1, 33]))
        p = params(batch=B, n_kv_heads=H, n_q_heads=H * int(rng.choice([1, 2, 4])), n_sink=n_sink, window=window,
                   max_new=max_new, sliding=sliding, head_window_host=None if hw is None else hw.ctypes.data)
        rc, desc, idx, sizes = plan(p, lens, mask)
        assert rc == razor.RAZOR_OK, trial
        total, off = 0, 0
        for b in range(B):
            for h in range(H):
                e = desc[b * H + h]
                win = window if hw is None else int(hw[h])
                kept, lo, hi = orc.select(int(lens[b]), bool(mask[h]), n_sink, win)
                assert e["rows"] == len(kept) and e["n_dropped"] == hi - lo and e["window"] == win, trial
                np.testing.assert_array_equal(idx[total: total + len(kept)], kept)
                assert e["row_off"] == off and e["cap"] % 16 == 0 and e["cap"] >= e["rows"]
                grow = e["rows"] + max_new
                if sliding and not mask[h]:
                    grow = min(grow, n_sink + win)
                assert grow <= e["cap"] < grow + 16, trial
                total += len(kept); off += e["cap"]
        assert sizes.total_rows == total and sizes.total_cap == off


# ----------------------------------------------------------------- head selection (Sec. 3.3)
def test_select_heads_matches_oracle_on_random_scores():
    rng = np.random.default_rng(8)
    for trial in range(200):
        group = int(rng.choice([1, 2, 4, 8]))
        n = group * int(rng.integers(1, 65))
        # few distinct values: plenty of ties, so the tie rule is exercised
        echo = rng.integers(0, 6, n).astype(np.float32) / 5
        ind = rng.integers(0, 6, n).astype(np.float32) / 5
        fi, fe = float(rng.uniform(0, 0.5)), float(rng.uniform(0, 0.2))
        got = razor.select_heads(echo, ind, group, fi, fe)
        np.testing.assert_array_equal(got, orc.select_heads(echo, ind, group, fi, fe), err_msg=f"trial {trial}")
    got = razor.select_heads(np.linspace(0, 1, 1024), np.linspace(1, 0, 1024), 1)
    assert got.sum() == 143 + 10 and got[:143].all() and got[-10:].all()          # Table 2's fractions


def test_select_heads_rejects_bad_arguments():
    e = np.zeros(8, np.float32)
    m = np.zeros(8, np.uint8)
    assert razor.razor_select_heads(e, e, 8, 3, 0.1, 0.1, m) == razor.RAZOR_EINVAL     # 8 % 3
    assert razor.razor_select_heads(e, e, 8, 2, 1.5, 0.1, m) == razor.RAZOR_EINVAL
    assert razor.razor_select_heads(e, e, 8, 2, 0.1, -0.1, m) == razor.RAZOR_EINVAL
    assert razor.razor_select_heads(e, e, 0, 1, 0.1, 0.1, m) == razor.RAZOR_EINVAL
    bad = e.copy(); bad[3] = np.nan
    assert razor.razor_select_heads(bad, e, 8, 2, 0.1, 0.1, m) == razor.RAZOR_EINVAL
    assert razor.razor_select_heads(e, e, 8, 2, 0.1, 0.1, m) == razor.RAZOR_OK


def test_head_scores_arguments_are_checked_before_any_gpu_work():
    L = razor.load_library()
    fake = ctypes.c_void_p(0x1000)
    ok = dict(dtype=razor.RAZOR_BF16, hq=8, hkv=2, d=128, n=1000, qsh=128000, qsn=128, ksh=128000, ksn=128,
              scale=0.088, period=250)

    def call(ws_bytes=1 << 30, Q=fake, **kw):
        a = dict(ok, **kw)
        return L.razor_head_scores(Q, fake, a["dtype"], a["hq"], a["hkv"], a["d"], a["n"], a["qsh"], a["qsn"],
                                   a["ksh"], a["ksn"], a["scale"], a["period"], 0, fake, fake, fake, ws_bytes, None)
    for kw in (dict(dtype=razor.RAZOR_F32), dict(d=96), dict(hq=7), dict(hkv=0), dict(period=0), dict(period=1000),
               dict(n=1), dict(scale=0.0), dict(scale=float("nan")), dict(qsn=64), dict(ksn=132), dict(qsh=-8),
               dict(Q=None), dict(Q=ctypes.c_void_p(0x1008)), dict(hq=70000, hkv=70000)):
        assert call(**kw) == razor.RAZOR_EINVAL, kw
    need = razor.razor_head_scores_workspace(8, 1000)
    assert need == 8 * 8 * 4 * 2 * 4                                  # 8 tiles of 128 queries, 4 waves, 2 sums
    assert call(ws_bytes=need - 1) == razor.RAZOR_ECAPACITY
    assert razor.razor_head_scores_workspace(0, 10) == 0


def test_read_stream_probe_arguments_are_checked():
    L = razor.load_library()
    fake = ctypes.c_void_p(0x1000)
    assert L.razor_probe_read_stream(None, 1 << 20, 0, 0, 2, 1, fake, None) == razor.RAZOR_EINVAL
    assert L.razor_probe_read_stream(fake, 1 << 20, 0, 0, 2, 1, None, None) == razor.RAZOR_EINVAL
    assert L.razor_probe_read_stream(ctypes.c_void_p(0x1004), 1 << 20, 0, 0, 2, 1, fake, None) == razor.RAZOR_EINVAL
    assert L.razor_probe_read_stream(fake, 100, 0, 0, 2, 1, fake, None) == razor.RAZOR_EINVAL     # less than one piece
    assert L.razor_probe_read_stream(fake, 1 << 20, -3, 0, 2, 1, fake, None) == razor.RAZOR_EINVAL
    assert L.razor_probe_read_stream(fake, 1 << 20, 0, -9000, 2, 1, fake, None) == razor.RAZOR_EINVAL  # unknown pattern
    assert L.razor_probe_read_stream(fake, 1 << 20, 0, 0, 3, 1, fake, None) == razor.RAZOR_EINVAL  # unsupported depth
    far = ctypes.c_void_p(0x10000000)
    assert L.razor_probe_copy(None, fake, 1 << 20, 0, 0, 3, None) == razor.RAZOR_EINVAL
    assert L.razor_probe_copy(far, ctypes.c_void_p(0x1008), 1 << 20, 0, 0, 3, None) == razor.RAZOR_EINVAL
    assert L.razor_probe_copy(fake, ctypes.c_void_p(0x2000), 1 << 20, 0, 0, 3, None) == razor.RAZOR_EINVAL   # overlap
    assert L.razor_probe_copy(far, fake, 1 << 20, 0, 0, 4, None) == razor.RAZOR_EINVAL             # unknown hint bits
    assert L.razor_probe_copy(far, fake, 100, 0, 0, 3, None) == razor.RAZOR_EINVAL
