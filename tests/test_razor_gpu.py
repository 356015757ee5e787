"""GPU parity: the HIP library, called through its C ABI, against the fp64 CPU oracle on
the same seeded inputs.

Bars: integer work (row counts, kept positions, copied K/V bits) bit-exact; Eq.(4)
means within fp32 accumulation error; attention outputs max-abs <= 2e-3 and per-row
relative L2 error <= 1e-2 (bf16 inputs, fp32 accumulation)."""
import numpy as np
import pytest
import torch

import paper_2407_15891_amd as razor
from oracle import razor_oracle as orc
from paper_2407_15891_amd.workloads import make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ABS_TOL, REL_TOL = 2e-3, 1e-2


# ----------------------------------------------------------------- helpers
def say(msg):
    print(msg, flush=True)


def check_output(out, ref, what, bf16_out=False):
    out = out.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(out).all(), what
    err = np.abs(out - ref)
    # a bf16 result carries its own half-ulp rounding (2^-9 relative) on top of the arithmetic
    tol = ABS_TOL + (np.abs(ref) * 2.0 ** -8 if bf16_out else 0.0)
    assert (err <= tol).all(), f"{what}: max-abs {err.max():.3e}"
    rel = np.linalg.norm(out - ref, axis=-1) / np.maximum(np.linalg.norm(ref, axis=-1), 1e-30)
    assert rel.max() <= REL_TOL, f"{what}: row-relative {rel.max():.3e}"
    return err.max(), rel.max()


def arena_rows(cache, desc, i):
    """(K rows, V rows) of head i as raw bytes [rows, row_bytes], K de-tiled."""
    p = cache.params
    rb = p.head_dim * (4 if p.dtype == razor.RAZOR_F32 else 2)
    e = desc[i]
    base = int(e["row_off"]) * 2 * rb
    cap, rows = int(e["cap"]), int(e["rows"])
    arena = cache.arena.cpu().numpy()
    kplane = arena[base: base + cap * rb].reshape(cap // 16, rb // 16, 16, 16)   # [block, piece, row, 16 B]
    k = kplane.transpose(0, 2, 1, 3).reshape(cap, rb)
    v = arena[base + cap * rb: base + 2 * cap * rb].reshape(cap, rb)
    return k[:rows], v[:rows]


def raw_bytes(t):
    """[..., d] tensor -> numpy uint8 [..., d * itemsize]."""
    a = orc.as_raw(t.cpu())
    return np.ascontiguousarray(a).view(np.uint8).reshape(*a.shape[:-1], -1)


def make_pair(w, **kw):
    cache = razor.RazorCache.from_workload(w, want_kept_idx=True, **kw)
    cache.compress(w.K, w.V)
    oc = orc.OracleCache(w.K.cpu(), w.V.cpu(), w.seq_lens, w.mask, w.n_sink, w.window, max_new=max(w.max_new, 1))
    return cache, oc


def check_compress(w, cache, oc, what, comp_atol=4e-6):
    desc = cache.desc()
    kept_dev = cache.kept_idx_dev.cpu().numpy()
    comp = cache.comp_tokens().cpu().numpy().astype(np.float64)
    Kb, Vb = raw_bytes(w.K), raw_bytes(w.V)
    np.testing.assert_array_equal(desc, cache.desc_host)                      # device table == planned table
    scale_in = float(w.K.abs().max())
    for b in range(w.B):
        for h in range(w.Hkv):
            i = b * w.Hkv + h
            e = desc[i]
            kept = oc.kept_of(b, h)
            assert e["rows"] == len(kept) and e["n_dropped"] == oc.N_d[b, h], what
            np.testing.assert_array_equal(kept_dev[e["kept_off"]: e["kept_off"] + e["rows"]], kept)
            k, v = arena_rows(cache, desc, i)
            np.testing.assert_array_equal(k, Kb[b, h][kept], err_msg=f"{what} K rows head {i}")
            np.testing.assert_array_equal(v, Vb[b, h][kept], err_msg=f"{what} V rows head {i}")
            np.testing.assert_allclose(comp[b, h, 0], oc.khat[b, h], rtol=0, atol=comp_atol * scale_in, err_msg=what)
            np.testing.assert_allclose(comp[b, h, 1], oc.vhat[b, h], rtol=0, atol=comp_atol * scale_in, err_msg=what)


def run_steps(w, cache, oc, steps, what, append=True, use_comp=True, bf16_out=False):
    worst = (0.0, 0.0)
    for t in range(steps):
        Q, k, v = w.step_inputs(t, append=append)
        out = cache.decode(Q, k, v)
        if append:
            oc.append(k.cpu(), v.cpu())
        ref = oc.decode(Q.cpu(), w.scale, use_comp=use_comp)
        e = check_output(out, ref, f"{what} step {t}", bf16_out)
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
    say(f"    {what}: {steps} step(s), max-abs {worst[0]:.2e}, row-rel {worst[1]:.2e}")


def check_bf16_output(cache, Q, ref, what):
    """The same step (no append) written out as bf16: the write-out rounds the fp32 result to
    nearest even, so it must equal the fp32 output rounded by torch bit for bit, and it lies
    within the arithmetic bar plus half a bf16 ulp (<= 2^-9 |ref| * 2) of the oracle."""
    p = cache.params
    out32 = torch.empty(p.batch, p.n_q_heads, p.head_dim, dtype=torch.float32, device=DEV)
    out16 = torch.empty(p.batch, p.n_q_heads, p.head_dim, dtype=torch.bfloat16, device=DEV)
    keep = p.out_dtype
    try:
        p.out_dtype = razor.RAZOR_F32
        cache.decode(Q, out=out32)
        p.out_dtype = razor.RAZOR_BF16
        cache.decode(Q, out=out16)
    finally:
        p.out_dtype = keep
    assert torch.equal(out16, out32.to(torch.bfloat16)), f"{what}: bf16 write-out is not the rounded fp32 result"
    return check_output(out16, ref, f"{what} (bf16 output)", bf16_out=True)


# ----------------------------------------------------------------- compress
@pytest.mark.parametrize("cfg,context,window,batch", [
    (1, 2048, 256, 1),        # config 1 at full size
    (1, 1000, 100, 3),        # ragged tail: 104 kept rows = 6.5 blocks
    (2, 3000, None, 1),
    (3, 5000, 700, 2),
    (4, 6000, 333, 5),        # ragged sequence lengths
])
def test_compress_parity(cfg, context, window, batch):
    say(f"compress parity cfg={cfg} context={context} window={window} batch={batch}")
    w = make_workload(cfg, DEV, context=context, window=window, batch=batch, max_new=3)
    cache, oc = make_pair(w)
    check_compress(w, cache, oc, f"cfg{cfg}")


@pytest.mark.parametrize("cfg,context,window,batch", [
    (1, 2048, 256, 1),
    (1, 1000, 100, 3),
    (3, 5000, 700, 2),
    (4, 6000, 333, 5),        # ragged sequence lengths
])
def test_compress_from_column_sums(cfg, context, window, batch):
    """Eq.(4) by subtraction: sums over all rows (the stand-in for a prefill epilogue) minus the
    kept rows.  The sums carry fp32 rounding of a value up to seq_len * max|x|, divided by N_d:
    a few 1e-7 * seq_len / N_d relative to max|x|, bounded here by 2e-5."""
    say(f"compress from column sums cfg={cfg} context={context} window={window} batch={batch}")
    w = make_workload(cfg, DEV, context=context, window=window, batch=batch, max_new=3)
    cache = razor.RazorCache.from_workload(w, want_kept_idx=True)
    sums = cache.column_sums(w.K, w.V)
    ref = orc.column_sums(w.K.cpu(), w.V.cpu(), w.seq_lens)
    scale_in = float(w.K.abs().max())
    tol = 2e-7 * scale_in * np.asarray(w.seq_lens, np.float64)[:, None, None, None]
    assert (np.abs(sums.cpu().numpy().astype(np.float64) - ref) <= tol).all()
    cache.compress(w.K, w.V, col_sums=sums)
    oc = orc.OracleCache(w.K.cpu(), w.V.cpu(), w.seq_lens, w.mask, w.n_sink, w.window, max_new=3)
    check_compress(w, cache, oc, f"cfg{cfg} column sums", comp_atol=2e-5)
    run_steps(w, cache, oc, 2, f"cfg{cfg} column sums")
    # same bits on a second run (fixed summation order)
    again = cache.column_sums(w.K, w.V)
    assert torch.equal(again, sums)


def test_compress_from_column_sums_when_no_row_is_kept():
    """No sinks, no window, no retrieval head: every head is its compensation token alone.  Given
    column sums nothing is copied at all and Eq.(4) is col_sums / N_d."""
    say("compress from column sums, heads that keep no row")
    w = make_workload(3, DEV, context=700, window=0, batch=2, max_new=2, mask=np.zeros(8, np.uint8))
    w.n_sink = 0
    cache = razor.RazorCache.from_workload(w, want_kept_idx=True)
    assert (cache.desc_host["rows"] == 0).all()
    sums = cache.column_sums(w.K, w.V)
    cache.compress(w.K, w.V, col_sums=sums)
    oc = orc.OracleCache(w.K.cpu(), w.V.cpu(), w.seq_lens, w.mask, 0, 0, max_new=2)
    check_compress(w, cache, oc, "no kept rows, column sums", comp_atol=2e-5)
    run_steps(w, cache, oc, 1, "no kept rows", append=False)
    run_steps(w, cache, oc, 2, "no kept rows + appended")


def test_compress_strided_input_and_fp32_dim128():
    say("compress parity: strided K/V views, fp32 head_dim 128, bf16 head_dim 64")
    for dtype, d in ((torch.float32, 128), (torch.bfloat16, 64), (torch.float32, 64), (torch.bfloat16, 128)):
        g = torch.Generator(device=DEV); g.manual_seed(77)
        big_k = torch.randn(2, 3, 777, d + 16, generator=g, device=DEV).to(dtype)
        big_v = torch.randn(2, 3, 777, d + 16, generator=g, device=DEV).to(dtype)
        K, V = big_k[:, :, 5:705, 8:8 + d], big_v[:, :, 5:705, 8:8 + d]      # 16-byte aligned views
        seq, mask = np.array([700, 431], np.int32), np.array([0, 1, 0], np.uint8)
        cache = razor.RazorCache(batch=2, n_q_heads=6, n_kv_heads=3, head_dim=d, seq_lens=seq,
                                 retrieval_mask=mask, n_sink=4, window=50, max_new=2, dtype=dtype,
                                 device=DEV, want_kept_idx=True)
        cache.compress(K, V)
        oc = orc.OracleCache(K.cpu().contiguous(), V.cpu().contiguous(), seq, mask, 4, 50, max_new=2)

        class W:  # the few fields check_compress reads
            pass
        w = W(); w.B, w.Hkv, w.d, w.K, w.V = 2, 3, d, K.contiguous(), V.contiguous()
        check_compress(w, cache, oc, f"strided {dtype} d={d}")
        cache.compress(K, V, col_sums=cache.column_sums(K, V))
        check_compress(w, cache, oc, f"strided {dtype} d={d} column sums", comp_atol=2e-5)
        # and the cache answers queries correctly
        Q = torch.randn(2, 6, d, generator=g, device=DEV).to(dtype)
        check_output(cache.decode(Q), oc.decode(Q.cpu(), d ** -0.5), f"strided {dtype} d={d}")


# ----------------------------------------------------------------- decode
@pytest.mark.parametrize("cfg,context,window,batch,workers", [
    (1, 2048, 256, 1, 0),      # config 1, fp32 MHA
    (1, 777, 90, 2, 16),       # few workers: every wave crosses head boundaries
    (2, 4096, None, 1, 0),     # bf16 MHA with outlier channels
    (2, 1500, 200, 2, 64),
    (3, 9000, 1000, 2, 0),     # GQA g = 4
    (3, 3001, 500, 3, 24),
    (4, 8000, 300, 4, 0),      # GQA g = 8, ragged lengths
    (4, 2500, 77, 6, 40),
    (3, 3001, 500, 3, 7),      # worker counts that are no multiple of a workgroup's four waves
    (2, 1500, 200, 2, 1023),
    (1, 777, 90, 2, 1),        # a single wave does everything
    (4, 2500, 77, 6, 8192),    # far more waves than blocks
])
def test_decode_parity(cfg, context, window, batch, workers):
    say(f"decode parity cfg={cfg} context={context} window={window} batch={batch} workers={workers}")
    w = make_workload(cfg, DEV, context=context, window=window, batch=batch, max_new=20)
    cache, oc = make_pair(w, n_workers=workers)
    run_steps(w, cache, oc, 1, "no append", append=False)
    run_steps(w, cache, oc, 20, "with append")           # crosses a 16-row block boundary
    d = cache.desc()
    np.testing.assert_array_equal(d["rows"], oc.rows().reshape(-1))
    assert not (d["flags"] & razor.RAZOR_HEAD_OVERFLOW).any()


@pytest.mark.parametrize("cfg", [1, 3])
def test_decode_special_cases(cfg):
    say(f"decode special cases cfg={cfg}")
    base = dict(context=1200, batch=2, max_new=2)
    # every head retrieval; nothing dropped (window covers); single dropped token; comp token only
    Hkv = 8
    for name, kw in (("all retrieval", dict(window=100, mask=np.ones(Hkv, np.uint8))),
                     ("window covers context", dict(window=1196)),
                     ("one dropped token", dict(window=1195)),
                     ("no window", dict(window=0)),
                     ("short window", dict(window=5))):
        w = make_workload(cfg, DEV, **base, **kw)
        cache, oc = make_pair(w)
        run_steps(w, cache, oc, 2, name)
    # ablation: compensation term off
    w = make_workload(cfg, DEV, window=64, **base)
    cache, oc = make_pair(w, use_comp=False)
    run_steps(w, cache, oc, 2, "use_comp=0", use_comp=False)
    # bf16 output
    if w.dtype == torch.bfloat16:
        cache, oc = make_pair(w, out_dtype=torch.bfloat16)
        run_steps(w, cache, oc, 2, "bf16 output", bf16_out=True)


def test_decode_only_compensation_token():
    say("decode: heads that keep no row at all (n_sink = 0, window = 0)")
    w = make_workload(3, DEV, context=500, window=0, batch=2, max_new=2)
    w.n_sink = 0
    cache, oc = make_pair(w)
    run_steps(w, cache, oc, 1, "comp token only", append=False)
    run_steps(w, cache, oc, 2, "comp token + appended rows")


def test_decode_peaked_queries_exercise_absolute_bound():
    say("decode: queries aligned with one cached key (outputs of order 1)")
    for cfg in (1, 2, 3):
        w = make_workload(cfg, DEV, context=3000, window=400, batch=2, max_new=1)
        cache, oc = make_pair(w)
        g = w.Hq // w.Hkv
        rng = np.random.default_rng(5)
        Q = torch.empty(w.B, w.Hq, w.d, device=DEV, dtype=w.dtype)
        for b in range(w.B):
            for j in range(w.Hq):
                kept = oc.kept_of(b, j // g)
                Q[b, j] = w.K[b, j // g, int(rng.choice(kept))] * 4
        out = cache.decode(Q)
        ref = oc.decode(Q.cpu(), w.scale)
        assert np.abs(ref).max() > 0.5
        e = check_output(out, ref, f"peaked cfg{cfg}")
        say(f"    peaked cfg{cfg}: max-abs {e[0]:.2e}, row-rel {e[1]:.2e}, max|ref| {np.abs(ref).max():.2f}")


def test_decode_is_bit_reproducible():
    say("decode: same inputs twice -> identical bits")
    w = make_workload(3, DEV, context=20000, window=3000, batch=2, max_new=1)
    cache, _ = make_pair(w)
    Q, _, _ = w.step_inputs(0, append=False)
    a = cache.decode(Q).clone()
    comp_a = cache.comp.clone()
    cache.compress(w.K, w.V)
    b = cache.decode(Q)
    assert torch.equal(a, b) and torch.equal(comp_a, cache.comp)


def test_append_overflow_sets_flag_and_keeps_answering():
    say("decode: append beyond cap sets the overflow flag, no fault")
    w = make_workload(1, DEV, context=300, window=12, batch=1, max_new=0)   # rows 16 -> cap 16, full
    cache, oc = make_pair(w)
    assert (cache.desc_host["cap"][cache.desc_host["n_dropped"] > 0] == 16).all()
    Q, k, v = w.step_inputs(0)
    out = torch.empty(w.B, w.Hq, w.d, dtype=torch.float32, device=DEV)
    rc = razor.razor_decode_attn(cache.params, Q, k, v, cache.arena, cache.comp, cache.desc_dev, out,
                                 cache.workspace, cache.workspace.numel(), 0)
    assert rc == razor.RAZOR_OK
    torch.cuda.synchronize()
    d = cache.desc()
    full = d["rows"] == d["cap"]
    assert full.any() and ((d["flags"] & razor.RAZOR_HEAD_OVERFLOW) != 0)[full].all()
    # full heads answered without the new token; the others (retrieval heads: 300 rows, cap 304) took it
    ref_without = oc.decode(Q.cpu(), w.scale)
    oc.append(k.cpu(), v.cpu())
    ref_with = oc.decode(Q.cpu(), w.scale)
    ref = np.where(np.repeat(full.reshape(w.B, w.Hkv), w.Hq // w.Hkv, 1)[..., None], ref_without, ref_with)
    check_output(out, ref, "overflow")


# ----------------------------------------------------------------- full-size configurations
def test_full_size_config2():
    say("full size: config 2 (32 heads x 32768 x 128 bf16), compress + 64 decode steps")
    w = make_workload(2, DEV)
    cache, oc = make_pair(w)
    check_compress(w, cache, oc, "config 2")
    run_steps(w, cache, oc, w.decode_steps, "config 2")
    Q, _, _ = w.step_inputs(1000, append=False)
    e = check_bf16_output(cache, Q, oc.decode(Q.cpu(), w.scale), "config 2")
    say(f"    config 2 bf16 output: max-abs {e[0]:.2e}, row-rel {e[1]:.2e}")


def test_full_size_config3():
    say("full size: config 3 (4 x 8 KV heads x 131072 x 128 bf16, g = 4)")
    w = make_workload(3, DEV)
    cache, oc = make_pair(w)
    say("    compressed; checking tables and means")
    desc = cache.desc()
    np.testing.assert_array_equal(desc["rows"], oc.rows().reshape(-1))
    np.testing.assert_array_equal(desc["n_dropped"], oc.N_d.reshape(-1))
    comp = cache.comp_tokens().cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(comp[:, :, 0], oc.khat, rtol=0, atol=3e-5)
    np.testing.assert_allclose(comp[:, :, 1], oc.vhat, rtol=0, atol=3e-5)
    # sampled heads: copied bits
    Kb, Vb = raw_bytes(w.K[:1]), raw_bytes(w.V[:1])
    for h in range(w.Hkv):
        k, v = arena_rows(cache, desc, h)
        np.testing.assert_array_equal(k, Kb[0, h][oc.kept_of(0, h)])
        np.testing.assert_array_equal(v, Vb[0, h][oc.kept_of(0, h)])
    run_steps(w, cache, oc, 1, "config 3", append=False)
    run_steps(w, cache, oc, 1, "config 3 append")
    Q, _, _ = w.step_inputs(1000, append=False)
    e = check_bf16_output(cache, Q, oc.decode(Q.cpu(), w.scale), "config 3")
    say(f"    config 3 bf16 output: max-abs {e[0]:.2e}, row-rel {e[1]:.2e}")


def test_full_size_config4():
    say("full size: config 4 (16 ragged sequences, 8 KV heads, g = 8)")
    w = make_workload(4, DEV)
    cache, oc = make_pair(w)
    desc = cache.desc()
    np.testing.assert_array_equal(desc["rows"], oc.rows().reshape(-1))
    np.testing.assert_array_equal(desc["n_dropped"], oc.N_d.reshape(-1))
    # copied bits of the shortest, the longest and two more sequences (every KV head of each)
    order = np.argsort(w.seq_lens)
    for b in (int(order[0]), int(order[-1]), int(order[5]), int(order[10])):
        Kb, Vb = raw_bytes(w.K[b:b + 1]), raw_bytes(w.V[b:b + 1])
        for h in range(w.Hkv):
            k, v = arena_rows(cache, desc, b * w.Hkv + h)
            np.testing.assert_array_equal(k, Kb[0, h][oc.kept_of(b, h)])
            np.testing.assert_array_equal(v, Vb[0, h][oc.kept_of(b, h)])
    run_steps(w, cache, oc, 1, "config 4")
    Q, _, _ = w.step_inputs(1000, append=False)
    check_bf16_output(cache, Q, oc.decode(Q.cpu(), w.scale), "config 4")


def test_full_size_config5_sampled_layers():
    """Config 5: layers of the 32-layer stack are independent here (attention only), so a
    sample of layers covering every retrieval pattern (0, 1, 2, 3 retrieval KV heads) is run
    through all 256 decode steps; the oracle checks steps 0, 127 and 255 of every
    (sequence, head) of those layers: 3 steps x 8 sequences x 32 query heads per layer."""
    from paper_2407_15891_amd.workloads import retrieval_pairs_stack
    table = retrieval_pairs_stack(32, 8, 0.15, 5000)
    assert table.sum() == 38
    counts = table.sum(1)
    layers = [int(np.flatnonzero(counts == c)[0]) for c in sorted(set(counts.tolist()))]
    say(f"full size: config 5, sampled layers {layers} (retrieval KV heads per layer: {[int(counts[l]) for l in layers]})")
    check_at = (0, 127, 255)
    for layer in layers:
        w = make_workload(5, DEV, layer=layer)
        assert w.max_new == 256 and (w.mask == table[layer]).all()
        cache = razor.RazorCache.from_workload(w)
        cache.compress(w.K, w.V)
        oc = orc.OracleCache(w.K.cpu(), w.V.cpu(), w.seq_lens, w.mask, w.n_sink, w.window, max_new=256)
        w_K0, w_V0 = w.K[:1].cpu(), w.V[:1].cpu()
        w.K = w.V = None
        say(f"    layer {layer}: compressed, oracle cache built")
        np.testing.assert_array_equal(cache.desc()["n_dropped"], oc.N_d.reshape(-1))
        comp = cache.comp_tokens().cpu().numpy().astype(np.float64)
        np.testing.assert_allclose(comp[:, :, 0], oc.khat, rtol=0, atol=3e-5)
        np.testing.assert_allclose(comp[:, :, 1], oc.vhat, rtol=0, atol=3e-5)
        desc = cache.desc()
        Kb, Vb = raw_bytes(w_K0), raw_bytes(w_V0)            # copied bits of sequence 0, every KV head
        for h in range(w.Hkv):
            k, v = arena_rows(cache, desc, h)
            np.testing.assert_array_equal(k, Kb[0, h][oc.kept_of(0, h)])
            np.testing.assert_array_equal(v, Vb[0, h][oc.kept_of(0, h)])
        del Kb, Vb, w_K0, w_V0
        worst = (0.0, 0.0)
        for t in range(256):
            Q, k, v = w.step_inputs(t)
            out = cache.decode(Q, k, v)
            oc.append(k.cpu(), v.cpu())
            if t in check_at:
                e = check_output(out, oc.decode(Q.cpu(), w.scale), f"config 5 layer {layer} step {t}")
                worst = (max(worst[0], e[0]), max(worst[1], e[1]))
        np.testing.assert_array_equal(cache.desc()["rows"], oc.rows().reshape(-1))
        say(f"    layer {layer}: 256 steps, checked {check_at}: max-abs {worst[0]:.2e}, row-rel {worst[1]:.2e}")
        del cache, oc
        torch.cuda.empty_cache()


# ----------------------------------------------------------------- sliding mode
@pytest.mark.parametrize("cfg,context,window,batch,workers,steps", [
    (1, 300, 40, 2, 0, 100),      # fp32; the 40-row ring wraps 2.5 times
    (2, 700, 50, 1, 0, 120),      # bf16 MHA, outlier channels
    (3, 900, 33, 2, 16, 80),      # GQA, few workers, window not a multiple of 16
    (4, 400, 100, 5, 0, 60),      # ragged: some sequences start below n_sink + window and fill up first
])
def test_sliding_mode_parity(cfg, context, window, batch, workers, steps):
    say(f"sliding parity cfg={cfg} context={context} window={window} batch={batch} workers={workers} steps={steps}")
    w = make_workload(cfg, DEV, context=context, window=window, batch=batch, max_new=steps)
    cache = razor.RazorCache.from_workload(w, n_workers=workers, sliding=True)
    cache.compress(w.K, w.V)
    oc = orc.OracleCache(w.K.cpu(), w.V.cpu(), w.seq_lens, w.mask, w.n_sink, w.window, max_new=steps, sliding=True)
    worst = (0.0, 0.0)
    for t in range(steps):
        Q, k, v = w.step_inputs(t)
        out = cache.decode(Q, k, v)
        oc.append(k.cpu(), v.cpu())
        e = check_output(out, oc.decode(Q.cpu(), w.scale), f"sliding step {t}")
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
        if t in (0, steps // 2, steps - 1):
            d = cache.desc()
            np.testing.assert_array_equal(d["rows"], oc.rows().reshape(-1))
            np.testing.assert_array_equal(d["n_dropped"], oc.N_d.reshape(-1))
            comp = cache.comp_tokens().cpu().numpy().astype(np.float64)
            tol = 1e-5 * float(w.K.abs().max())
            np.testing.assert_allclose(comp[:, :, 0], oc.khat, rtol=0, atol=tol)
            np.testing.assert_allclose(comp[:, :, 1], oc.vhat, rtol=0, atol=tol)
    d = cache.desc()
    nonret = np.tile(w.mask == 0, w.B)
    assert (d["rows"][nonret] <= w.n_sink + w.window).all() and not (d["flags"] & razor.RAZOR_HEAD_OVERFLOW).any()
    say(f"    {steps} steps: max-abs {worst[0]:.2e}, row-rel {worst[1]:.2e}, evicted up to {int(d['evicted'].max())}")


@pytest.mark.parametrize("cfg,context,window,batch,steps", [
    (3, 600, 48, 2, 20000),      # bf16 GQA: the 48-row ring wraps 400 times, N_d grows from 548 to 20548
    (1, 500, 40, 1, 20000),      # fp32 MHA
])
def test_sliding_mode_long_generation(cfg, context, window, batch, steps):
    """Sliding mode exists for generations of any length: 20 000 steps on a small shape, the oracle
    (Eq.(4) from scratch in fp64 over everything dropped so far) checked at ten steps including the
    last.  K and V carry a constant offset so that the means are of order one and their fp32
    rounding would show: the running means must stay within 4 ulp of the fp64 means (a plain fp32
    update is off by tens of ulp by then), outputs within the usual bars."""
    say(f"sliding long generation cfg={cfg} context={context} window={window} batch={batch} steps={steps}")
    w = make_workload(cfg, DEV, context=context, window=window, batch=batch, max_new=steps)
    w.K += 1.5
    w.V -= 2.0
    cache = razor.RazorCache.from_workload(w, sliding=True)
    cache.compress(w.K, w.V)
    oc = orc.OracleCache(w.K.cpu(), w.V.cpu(), w.seq_lens, w.mask, w.n_sink, w.window, max_new=steps, sliding=True)
    gen = torch.Generator(device=DEV); gen.manual_seed(31337 + cfg)
    check_at = sorted(set(int(x) for x in np.linspace(0, steps - 1, 10)))
    chunk, worst, worst_ulp = 2000, (0.0, 0.0), 0.0
    out = torch.empty(w.B, w.Hq, w.d, dtype=torch.float32, device=DEV)
    for t0 in range(0, steps, chunk):
        n = min(chunk, steps - t0)
        Qs = torch.randn(n, w.B, w.Hq, w.d, generator=gen, device=DEV).to(w.dtype)
        ks = (torch.randn(n, w.B, w.Hkv, w.d, generator=gen, device=DEV) + 1.5).to(w.dtype)
        vs = (torch.randn(n, w.B, w.Hkv, w.d, generator=gen, device=DEV) - 2.0).to(w.dtype)
        ks_c, vs_c = ks.cpu(), vs.cpu()
        for j in range(n):
            t = t0 + j
            cache.decode(Qs[j], ks[j], vs[j], out=out)
            oc.append(ks_c[j], vs_c[j])
            if t in check_at:
                e = check_output(out, oc.decode(Qs[j].cpu(), w.scale), f"long sliding step {t}")
                worst = (max(worst[0], e[0]), max(worst[1], e[1]))
                d = cache.desc()
                np.testing.assert_array_equal(d["rows"], oc.rows().reshape(-1))
                np.testing.assert_array_equal(d["n_dropped"], oc.N_d.reshape(-1))
                comp = cache.comp_tokens().cpu().numpy().astype(np.float64)
                for got, ref in ((comp[:, :, 0], oc.khat), (comp[:, :, 1], oc.vhat)):
                    ulp = np.spacing(np.abs(ref).astype(np.float32)).astype(np.float64)
                    worst_ulp = max(worst_ulp, float((np.abs(got - ref) / ulp).max()))
                    # the prefill part of each mean comes from the compression pass (fp32 partial sums: a few
                    # 1e-7 relative to max|x|); the decode-time updates add at most an ulp on top
                    assert (np.abs(got - ref) <= 4 * ulp + 4e-7 * 6.0).all(), f"step {t}: mean off by {worst_ulp:.1f} ulp"
        say(f"    through step {t0 + n - 1}: max-abs {worst[0]:.2e}, row-rel {worst[1]:.2e}, means within {worst_ulp:.1f} ulp")
    d = cache.desc()
    nonret = np.tile(w.mask == 0, w.B)
    assert (d["rows"][nonret] == w.n_sink + w.window).all() and (d["evicted"][nonret] == steps).all()


def test_sliding_mode_without_compensation_is_sinks_plus_window():
    say("sliding, use_comp = 0: attention over the sinks and the last `window` tokens")
    w = make_workload(3, DEV, context=500, window=64, batch=2, max_new=70)
    cache = razor.RazorCache.from_workload(w, sliding=True, use_comp=False)
    cache.compress(w.K, w.V)
    oc = orc.OracleCache(w.K.cpu(), w.V.cpu(), w.seq_lens, w.mask, w.n_sink, w.window, max_new=70, sliding=True)
    for t in range(70):
        Q, k, v = w.step_inputs(t)
        out = cache.decode(Q, k, v)
        oc.append(k.cpu(), v.cpu())
        check_output(out, oc.decode(Q.cpu(), w.scale, use_comp=False), f"sliding no-comp step {t}")


# ----------------------------------------------------------------- ALiBi form (Eq.(1)), per-head buffer lengths
def alibi_slopes(n_heads):
    """The usual geometric ALiBi slopes 2^(-8 i / n), i = 1..n."""
    return (2.0 ** (-8.0 * np.arange(1, n_heads + 1) / n_heads)).astype(np.float32)


@pytest.mark.parametrize("cfg,context,batch,sliding,workers,steps", [
    (1, 1500, 2, False, 0, 20),     # fp32 MHA
    (2, 2000, 1, False, 0, 20),     # bf16 MHA 32 heads (the Baichuan-style case)
    (3, 1800, 2, False, 24, 20),    # bf16 GQA: slopes differ inside a group
    (2, 600, 2, True, 0, 90),       # sliding: short scopes wrap several times
    (3, 500, 3, True, 16, 70),
    (1, 400, 1, True, 0, 60),
])
def test_alibi_parity(cfg, context, batch, sliding, workers, steps):
    say(f"alibi parity cfg={cfg} context={context} batch={batch} sliding={sliding} workers={workers} steps={steps}")
    w = make_workload(cfg, DEV, context=context, batch=batch, max_new=steps)
    rng = np.random.default_rng(99 + cfg)
    # per-KV-head vision scopes: a few local heads, a few that keep everything (the "retrieval" heads)
    hw = rng.choice([17, 48, 100, 10 ** 6], size=w.Hkv).astype(np.int32)
    hw[0], hw[-1] = 17, 10 ** 6
    slopes = alibi_slopes(w.Hq)
    mask = np.zeros(w.Hkv, np.uint8)
    cache = razor.RazorCache(batch=w.B, n_q_heads=w.Hq, n_kv_heads=w.Hkv, head_dim=w.d, seq_lens=w.seq_lens,
                             retrieval_mask=mask, n_sink=0, window=0 if not sliding else 1, max_new=steps,
                             dtype=w.dtype, scale=w.scale, use_comp=False, n_workers=workers, device=DEV,
                             sliding=sliding, head_window=hw, alibi_slopes=torch.from_numpy(slopes).to(DEV))
    cache.compress(w.K, w.V)
    oc = orc.OracleCache(w.K.cpu(), w.V.cpu(), w.seq_lens, mask, 0, 0, max_new=steps, sliding=sliding,
                         head_window=hw, alibi_slopes=slopes)
    np.testing.assert_array_equal(cache.desc()["rows"], oc.rows().reshape(-1))
    worst = (0.0, 0.0)
    for t in range(steps):
        Q, k, v = w.step_inputs(t)
        out = cache.decode(Q, k, v)
        oc.append(k.cpu(), v.cpu())
        e = check_output(out, oc.decode(Q.cpu(), w.scale, use_comp=False), f"alibi step {t}")
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
    np.testing.assert_array_equal(cache.desc()["rows"], oc.rows().reshape(-1))
    say(f"    {steps} steps: max-abs {worst[0]:.2e}, row-rel {worst[1]:.2e}")


def test_alibi_with_sinks_static():
    say("alibi + sink rows (true prefill distances for the sinks)")
    w = make_workload(3, DEV, context=900, window=60, batch=2, max_new=10)
    slopes = alibi_slopes(w.Hq)
    cache = razor.RazorCache.from_workload(w, use_comp=False, alibi_slopes=torch.from_numpy(slopes).to(DEV))
    cache.compress(w.K, w.V)
    oc = orc.OracleCache(w.K.cpu(), w.V.cpu(), w.seq_lens, w.mask, w.n_sink, w.window, max_new=10, alibi_slopes=slopes)
    for t in range(10):
        Q, k, v = w.step_inputs(t)
        out = cache.decode(Q, k, v)
        oc.append(k.cpu(), v.cpu())
        check_output(out, oc.decode(Q.cpu(), w.scale, use_comp=False), f"alibi sinks step {t}")


# ----------------------------------------------------------------- HIP graph capture
def test_decode_under_hip_graph_capture_matches_eager():
    """A decode step enqueues kernels only (no allocation, no synchronisation, no memset), so it
    can be captured once and replayed: every replay, with eager work in between, must give the
    bits the eager path gives."""
    say("decode captured in a HIP graph and replayed")
    w = make_workload(3, DEV, context=6000, window=700, batch=2, max_new=12)
    eager = razor.RazorCache.from_workload(w); eager.compress(w.K, w.V)
    graphed = razor.RazorCache.from_workload(w); graphed.compress(w.K, w.V)
    Qs, ks, vs = (torch.empty_like(x) for x in w.step_inputs(0))
    out_g = torch.empty(w.B, w.Hq, w.d, dtype=torch.float32, device=DEV)
    # warm up on a side stream as torch asks, on a third cache so that `graphed` stays untouched
    side = razor.RazorCache.from_workload(w); side.compress(w.K, w.V)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        side.decode(Qs, ks, vs, out=out_g)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.decode(Qs, ks, vs, out=out_g)
    for t in range(8):
        Q, k, v = w.step_inputs(t)
        ref = eager.decode(Q, k, v).clone()
        Qs.copy_(Q); ks.copy_(k); vs.copy_(v)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g, ref), f"replay {t}"
        _ = (w.K[0, 0, :64].float().sum()).item()          # unrelated eager work between replays
    np.testing.assert_array_equal(graphed.desc()["rows"], eager.desc()["rows"])


# ----------------------------------------------------------------- group sizes and head dims
@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 64), (torch.float32, 128)])
@pytest.mark.parametrize("g", [2, 3, 5, 16])
def test_every_group_size_and_head_dim(dtype, d, g):
    say(f"group size {g}, head_dim {d}, {dtype}")
    Hkv, B, N = 3, 2, 1100
    gen = torch.Generator(device=DEV); gen.manual_seed(1234 + g + d)
    K = torch.randn(B, Hkv, N, d, generator=gen, device=DEV).to(dtype)
    V = torch.randn(B, Hkv, N, d, generator=gen, device=DEV).to(dtype)
    seq, mask = np.array([1100, 777], np.int32), np.array([0, 1, 0], np.uint8)
    cache = razor.RazorCache(batch=B, n_q_heads=Hkv * g, n_kv_heads=Hkv, head_dim=d, seq_lens=seq,
                             retrieval_mask=mask, n_sink=4, window=150, max_new=4, dtype=dtype, device=DEV)
    cache.compress(K, V)
    oc = orc.OracleCache(K.cpu(), V.cpu(), seq, mask, 4, 150, max_new=4)
    for t in range(4):
        Q = torch.randn(B, Hkv * g, d, generator=gen, device=DEV).to(dtype)
        k = torch.randn(B, Hkv, d, generator=gen, device=DEV).to(dtype)
        v = torch.randn(B, Hkv, d, generator=gen, device=DEV).to(dtype)
        out = cache.decode(Q, k, v)
        oc.append(k.cpu(), v.cpu())
        check_output(out, oc.decode(Q.cpu(), d ** -0.5), f"g={g} d={d} step {t}")


def test_many_heads():
    say("1000 (sequence, head) pairs: the block-prefix scans run over 16 chunks of 64 heads")
    B, Hkv, g, d, N = 125, 8, 2, 64, 96
    gen = torch.Generator(device=DEV); gen.manual_seed(4321)
    K = torch.randn(B, Hkv, N, d, generator=gen, device=DEV).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, d, generator=gen, device=DEV).to(torch.bfloat16)
    seq = np.random.default_rng(3).integers(1, N + 1, size=B).astype(np.int32)
    mask = np.array([0, 1, 0, 0, 0, 0, 1, 0], np.uint8)
    cache = razor.RazorCache(batch=B, n_q_heads=Hkv * g, n_kv_heads=Hkv, head_dim=d, seq_lens=seq,
                             retrieval_mask=mask, n_sink=2, window=20, max_new=3, dtype=torch.bfloat16, device=DEV)
    cache.compress(K, V)
    oc = orc.OracleCache(K.cpu(), V.cpu(), seq, mask, 2, 20, max_new=3)
    comp = cache.comp_tokens().cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(comp[:, :, 0], oc.khat, rtol=0, atol=2e-5)
    for t in range(3):
        Q = torch.randn(B, Hkv * g, d, generator=gen, device=DEV).to(torch.bfloat16)
        k = torch.randn(B, Hkv, d, generator=gen, device=DEV).to(torch.bfloat16)
        v = torch.randn(B, Hkv, d, generator=gen, device=DEV).to(torch.bfloat16)
        out = cache.decode(Q, k, v)
        oc.append(k.cpu(), v.cpu())
        check_output(out, oc.decode(Q.cpu(), d ** -0.5), f"many heads step {t}")
    np.testing.assert_array_equal(cache.desc()["rows"], oc.rows().reshape(-1))


@pytest.mark.parametrize("batch,n_kv", [(8, 8), (13, 5), (32, 8), (257, 1)])
def test_head_count_boundaries(batch, n_kv):
    """64, 65, 256 and 257 (sequence, head) pairs: the table as a kernel argument / uploaded, the
    streamed sums with the second level riding in the copy / the sums inside the copy launch."""
    n_heads = batch * n_kv
    say(f"{n_heads} (sequence, head) pairs")
    g, d, N, n_sink, window = 2, 64, 700, 3, 50
    gen = torch.Generator(device=DEV); gen.manual_seed(1000 + n_heads)
    K = torch.randn(batch, n_kv, N, d, generator=gen, device=DEV).to(torch.bfloat16)
    V = torch.randn(batch, n_kv, N, d, generator=gen, device=DEV).to(torch.bfloat16)
    seq = np.random.default_rng(n_heads).integers(40, N + 1, size=batch).astype(np.int32)
    seq[0] = N
    mask = (np.arange(n_kv) % 4 == 1).astype(np.uint8)
    cache = razor.RazorCache(batch=batch, n_q_heads=n_kv * g, n_kv_heads=n_kv, head_dim=d, seq_lens=seq,
                             retrieval_mask=mask, n_sink=n_sink, window=window, max_new=2, dtype=torch.bfloat16,
                             device=DEV, want_kept_idx=True)
    cache.compress(K, V)
    oc = orc.OracleCache(K.cpu(), V.cpu(), seq, mask, n_sink, window, max_new=2)
    desc = cache.desc()
    np.testing.assert_array_equal(desc, cache.desc_host)
    comp = cache.comp_tokens().cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(comp[:, :, 0], oc.khat, rtol=0, atol=2e-5)
    np.testing.assert_allclose(comp[:, :, 1], oc.vhat, rtol=0, atol=2e-5)
    Kb, Vb = raw_bytes(K), raw_bytes(V)
    for i in (0, 1, n_heads // 2, n_heads - 2, n_heads - 1):
        b, h = divmod(i, n_kv)
        kept = oc.kept_of(b, h)
        k, v = arena_rows(cache, desc, i)
        np.testing.assert_array_equal(k, Kb[b, h][kept])
        np.testing.assert_array_equal(v, Vb[b, h][kept])
    for t in range(2):
        Q = torch.randn(batch, n_kv * g, d, generator=gen, device=DEV).to(torch.bfloat16)
        k = torch.randn(batch, n_kv, d, generator=gen, device=DEV).to(torch.bfloat16)
        v = torch.randn(batch, n_kv, d, generator=gen, device=DEV).to(torch.bfloat16)
        out = cache.decode(Q, k, v)
        oc.append(k.cpu(), v.cpu())
        check_output(out, oc.decode(Q.cpu(), d ** -0.5), f"{n_heads} pairs step {t}")


# ----------------------------------------------------------------- seeded random sweep
def test_read_stream_probe_runs_on_odd_sizes():
    """The measurement hook reads whole 4 KB pieces inside the buffer whatever the size and worker count."""
    buf = torch.ones(5 * 4096 * 1031 + 777, dtype=torch.uint8, device=DEV)
    sink = torch.zeros(4 * razor.RAZOR_MAX_WORKERS, dtype=torch.uint8, device=DEV)
    for nbytes, workers in ((4096, 0), (4096 * 3 + 5, 4), (buf.numel(), 0), (buf.numel(), 1000), (buf.numel(), 8192)):
        for pattern in (razor.RAZOR_PROBE_CONTIGUOUS, razor.RAZOR_PROBE_INTERLEAVED, 7, 64, -5, -32):
            for depth, nt in ((1, 1), (2, 0), (4, 1), (8, 0)):
                assert razor.razor_probe_read_stream(buf, nbytes, workers, pattern, depth, nt, sink) == razor.RAZOR_OK
    torch.cuda.synchronize()
    assert int(sink.sum()) == 0          # the sink is only written if a checksum hits one value in 2^32


def test_copy_probe_copies_whole_pieces_and_nothing_else():
    src = torch.randint(0, 255, (4096 * 517 + 100,), dtype=torch.uint8, device=DEV)
    for workers in (0, 4, 1000, 8192):
        for pattern in (razor.RAZOR_PROBE_CONTIGUOUS, razor.RAZOR_PROBE_INTERLEAVED, 5, 100, -3, -64):
            for hints in range(4):
                dst = torch.zeros_like(src)
                assert razor.razor_probe_copy(dst, src, src.numel(), workers, pattern, hints) == razor.RAZOR_OK
                n = src.numel() // 4096 * 4096
                assert torch.equal(dst[:n], src[:n]) and int(dst[n:].sum()) == 0


@pytest.mark.parametrize("seed", list(range(24)))
def test_random_shapes_parity(seed):
    """Random but seeded shapes: batch, heads, group, head_dim, dtype, ragged lengths, sinks,
    window (global or per head), workers, static / sliding, with and without compensation."""
    rng = np.random.default_rng(5000 + seed)
    dtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
    d = int(rng.choice([64, 128]))
    B, Hkv, g = int(rng.integers(1, 5)), int(rng.integers(1, 6)), int(rng.choice([1, 2, 4, 7, 8]))
    N = int(rng.choice([40, 200, 1000, 3000]))
    n_sink = int(rng.choice([0, 2, 4]))
    sliding = bool(rng.integers(0, 2))
    window = int(rng.choice([1, 5, 16, 37, 250]))
    use_comp = bool(rng.random() < 0.8)
    steps = int(rng.choice([3, 25]))
    workers = int(rng.choice([0, 4, 12, 200]))
    lens = rng.integers(max(1, n_sink), N + 1, size=B).astype(np.int32)
    mask = (rng.random(Hkv) < 0.3).astype(np.uint8)
    hw = rng.choice([1, 7, 64, 10 ** 6], size=Hkv).astype(np.int32) if rng.random() < 0.3 else None
    say(f"random seed={seed}: {dtype} d={d} B={B} Hkv={Hkv} g={g} N={N} lens={lens.tolist()} sinks={n_sink} "
        f"window={window} head_window={None if hw is None else hw.tolist()} sliding={sliding} comp={use_comp} "
        f"workers={workers} steps={steps}")
    gen = torch.Generator(device=DEV); gen.manual_seed(9000 + seed)
    K = torch.randn(B, Hkv, N, d, generator=gen, device=DEV).to(dtype)
    V = torch.randn(B, Hkv, N, d, generator=gen, device=DEV).to(dtype)
    cache = razor.RazorCache(batch=B, n_q_heads=Hkv * g, n_kv_heads=Hkv, head_dim=d, seq_lens=lens,
                             retrieval_mask=mask, n_sink=n_sink, window=window, max_new=steps, dtype=dtype,
                             use_comp=use_comp, n_workers=workers, device=DEV, sliding=sliding, head_window=hw)
    cache.compress(K, V)
    oc = orc.OracleCache(K.cpu(), V.cpu(), lens, mask, n_sink, window, max_new=steps, sliding=sliding, head_window=hw)
    for t in range(steps):
        Q = torch.randn(B, Hkv * g, d, generator=gen, device=DEV).to(dtype)
        k = torch.randn(B, Hkv, d, generator=gen, device=DEV).to(dtype)
        v = torch.randn(B, Hkv, d, generator=gen, device=DEV).to(dtype)
        out = cache.decode(Q, k, v)
        oc.append(k.cpu(), v.cpu())
        check_output(out, oc.decode(Q.cpu(), d ** -0.5, use_comp=use_comp), f"seed {seed} step {t}")
    check_bf16_output(cache, Q, oc.decode(Q.cpu(), d ** -0.5, use_comp=use_comp), f"seed {seed}")
    dsc = cache.desc()
    np.testing.assert_array_equal(dsc["rows"], oc.rows().reshape(-1))
    np.testing.assert_array_equal(dsc["n_dropped"], oc.N_d.reshape(-1))
    assert not (dsc["flags"] & razor.RAZOR_HEAD_OVERFLOW).any()
