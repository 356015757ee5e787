"""Pins for the fp64 oracle: everything here is fixed by the paper or by mathematics,
none of it by the oracle itself (and none of it by the HIP library).

  P-hand   Eq.(5) worked by hand on a 4-token, d=1 example (exact rationals)
  I1       all heads retrieval            == library softmax attention (torch SDPA, fp64)
  I2       sinks + window cover the cache == full attention
  I3       one dropped token              == keeping that token (full attention)
  I4       identical dropped keys         == full attention (closed form)
  I5       q = 0                          == mean of all N value rows (closed form)
  I6       brute force: compensation token replicated N_d times, textbook softmax
  I7       Jensen: compensation weight <= true weight of the dropped set
  I8       adding one vector to every key leaves the output unchanged
  I9       output is a convex combination of {vhat} and the kept values
  I10      GQA head j == MHA run on KV head j // g; dropped-row order is irrelevant
  I11      kept-row ratio -> 3.125 (Table 2 caption)
  select   closed-form index tables, boundary cases
  append   decode-time appends are ordinary kept rows
  bits     bf16 / fp32 widening is exact
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import razor_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- helpers (independent of the oracle)
def softmax_attention(q, K, V, scale, weights=None):
    """Textbook softmax attention of one query over rows of K/V (numpy, fp64)."""
    s = scale * (K @ q)
    if weights is not None:
        s = s + np.log(weights)
    s = s - s.max()
    p = np.exp(s)
    return (p[:, None] * V).sum(0) / p.sum()


def rand_case(rng, B, Hkv, g, N, d, dtype=np.float32):
    K = rng.standard_normal((B, Hkv, N, d)).astype(np.float32)
    V = rng.standard_normal((B, Hkv, N, d)).astype(np.float32)
    Q = rng.standard_normal((B, Hkv * g, d)).astype(np.float32)
    if dtype == "bf16":
        K, V, Q = (torch.from_numpy(x).to(torch.bfloat16) for x in (K, V, Q))
    return K, V, Q


def f64(x):
    if isinstance(x, torch.Tensor):
        return x.to(torch.float64).numpy()
    return x.astype(np.float64)


def full_attention(K, V, Q, seq_lens, scale, g):
    Kd, Vd, Qd = f64(K), f64(V), f64(Q)
    B, Hq, d = Qd.shape
    out = np.empty((B, Hq, d))
    for b in range(B):
        for j in range(Hq):
            n = seq_lens[b]
            out[b, j] = softmax_attention(Qd[b, j], Kd[b, j // g, :n], Vd[b, j // g, :n], scale)
    return out


# ----------------------------------------------------------------- P-hand
def test_hand_worked_eq5():
    # 4 tokens, d = 1, one sink, window 1, D = {1, 2}; q = 1, scale = 1.
    # k = [0, ln2, ln8, 0], v = [1, 2, 4, 8]  ->  khat = ln4, vhat = 3, N_d = 2
    # Eq.(5): (2*4*3 + 1*1 + 1*8) / (2*4 + 1 + 1) = 33/10
    # full attention on the same data: (1 + 2*2 + 8*4 + 8) / (1 + 2 + 8 + 1) = 45/12
    K = np.array([0.0, math.log(2), math.log(8), 0.0], np.float32).reshape(1, 1, 4, 1)
    V = np.array([1, 2, 4, 8], np.float32).reshape(1, 1, 4, 1)
    Q = np.ones((1, 1, 1), np.float32)
    c = orc.OracleCache(K, V, [4], [0], n_sink=1, window=1)
    assert c.N_d[0, 0] == 2 and list(c.kept_of(0, 0)) == [0, 3]
    assert c.vhat[0, 0, 0] == pytest.approx(3.0, abs=1e-15)
    assert c.khat[0, 0, 0] == pytest.approx(math.log(4), rel=1e-7)   # fp32 storage of ln2, ln8
    assert c.decode(Q, 1.0)[0, 0, 0] == pytest.approx(3.3, rel=1e-6)
    # retrieval head on the same data gives the full-attention value
    c = orc.OracleCache(K, V, [4], [1], n_sink=1, window=1)
    assert c.decode(Q, 1.0)[0, 0, 0] == pytest.approx(3.75, rel=1e-6)
    # ablation (no compensation term): (1 + 8) / 2
    c = orc.OracleCache(K, V, [4], [0], n_sink=1, window=1)
    assert c.decode(Q, 1.0, use_comp=False)[0, 0, 0] == pytest.approx(4.5, rel=1e-12)
    # scale multiplies every logit, the compensation one included: scale = 2 -> e^{2 ln4} = 16
    assert c.decode(Q, 2.0)[0, 0, 0] == pytest.approx((2 * 16 * 3 + 1 + 8) / (2 * 16 + 2), rel=1e-6)


# ----------------------------------------------------------------- I1 / I2
@pytest.mark.parametrize("dtype", [np.float32, "bf16"])
@pytest.mark.parametrize("g", [1, 4])
def test_I1_all_retrieval_equals_sdpa(dtype, g):
    rng = np.random.default_rng(1)
    B, Hkv, N, d = 2, 3, 97, 16
    K, V, Q = rand_case(rng, B, Hkv, g, N, d, dtype)
    scale = 1 / math.sqrt(d)
    c = orc.OracleCache(K, V, [N] * B, [1] * Hkv, n_sink=4, window=8)
    out = c.decode(Q, scale)
    Kt, Vt, Qt = (torch.as_tensor(f64(x)) for x in (K, V, Q))
    ref = torch.nn.functional.scaled_dot_product_attention(
        Qt[:, :, None, :], Kt.repeat_interleave(g, 1), Vt.repeat_interleave(g, 1),
        scale=scale)[:, :, 0, :].numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-14)
    assert (c.N_d == 0).all()


def test_I2_window_covers_context():
    rng = np.random.default_rng(2)
    B, Hkv, g, N, d = 1, 4, 2, 40, 8
    K, V, Q = rand_case(rng, B, Hkv, g, N, d)
    for n_sink, window in [(4, 36), (4, 40), (0, 40), (10, 35), (40, 0)]:
        c = orc.OracleCache(K, V, [N], [0] * Hkv, n_sink=n_sink, window=window)
        assert (c.N_d == 0).all()
        np.testing.assert_allclose(c.decode(Q, 0.3), full_attention(K, V, Q, [N], 0.3, g),
                                   rtol=1e-12, atol=1e-14)


# ----------------------------------------------------------------- I3 / I4 / I5
def test_I3_single_dropped_token():
    rng = np.random.default_rng(3)
    B, Hkv, g, N, d = 2, 2, 2, 30, 8
    K, V, Q = rand_case(rng, B, Hkv, g, N, d)
    c = orc.OracleCache(K, V, [N] * B, [0] * Hkv, n_sink=4, window=N - 5)
    assert (c.N_d == 1).all()
    np.testing.assert_allclose(c.decode(Q, 0.5), full_attention(K, V, Q, [N] * B, 0.5, g),
                               rtol=1e-12, atol=1e-14)


def test_I4_identical_dropped_keys():
    rng = np.random.default_rng(4)
    B, Hkv, g, N, d = 1, 3, 2, 64, 8
    K, V, Q = rand_case(rng, B, Hkv, g, N, d)
    n_sink, window = 3, 10
    K[:, :, n_sink:N - window, :] = K[:, :, n_sink:n_sink + 1, :]      # dropped keys all equal
    c = orc.OracleCache(K, V, [N], [0] * Hkv, n_sink=n_sink, window=window)
    assert (c.N_d == N - n_sink - window).all()
    np.testing.assert_allclose(c.decode(Q, 0.7), full_attention(K, V, Q, [N], 0.7, g),
                               rtol=1e-11, atol=1e-13)
    # and it must differ once the dropped keys differ (the method is an approximation)
    K2 = K.copy(); K2[:, :, n_sink + 1, :] += 1.0
    c2 = orc.OracleCache(K2, V, [N], [0] * Hkv, n_sink=n_sink, window=window)
    assert np.abs(c2.decode(Q, 0.7) - full_attention(K2, V, Q, [N], 0.7, g)).max() > 1e-4


def test_I5_zero_query_gives_mean_of_all_values():
    rng = np.random.default_rng(5)
    B, Hkv, g, N, d = 2, 2, 1, 50, 8
    K, V, Q = rand_case(rng, B, Hkv, g, N, d)
    Q[:] = 0
    lens = [50, 37]
    c = orc.OracleCache(K, V, lens, [0, 0], n_sink=4, window=6)
    out = c.decode(Q, 1.0)
    for b in range(B):
        for h in range(Hkv):
            np.testing.assert_allclose(out[b, h], f64(V)[b, h, :lens[b]].mean(0), rtol=1e-12, atol=1e-14)


# ----------------------------------------------------------------- I6 brute force
@pytest.mark.parametrize("dtype", [np.float32, "bf16"])
@pytest.mark.parametrize("scale", [1.0, 0.25])
def test_I6_bruteforce_replicated_token(dtype, scale):
    rng = np.random.default_rng(6)
    B, Hkv, g, N, d = 2, 3, 2, 23, 4
    K, V, Q = rand_case(rng, B, Hkv, g, N, d, dtype)
    lens, mask, n_sink, window = [23, 17], [0, 1, 0], 2, 5
    c = orc.OracleCache(K, V, lens, mask, n_sink=n_sink, window=window)
    out = c.decode(Q, scale)
    Kd, Vd, Qd = f64(K), f64(V), f64(Q)
    for b in range(B):
        n = lens[b]
        for j in range(Hkv * g):
            h = j // g
            if mask[h]:
                Kx, Vx = Kd[b, h, :n], Vd[b, h, :n]
            else:
                keep = list(range(n_sink)) + list(range(n - window, n))
                drop = list(range(n_sink, n - window))
                kh, vh = Kd[b, h, drop].mean(0), Vd[b, h, drop].mean(0)
                Kx = np.concatenate([Kd[b, h, keep]] + [kh[None]] * len(drop))
                Vx = np.concatenate([Vd[b, h, keep]] + [vh[None]] * len(drop))
            np.testing.assert_allclose(out[b, j], softmax_attention(Qd[b, j], Kx, Vx, scale),
                                       rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------------- I7 Jensen
def test_I7_compensation_weight_below_true_dropped_weight():
    rng = np.random.default_rng(7)
    B, Hkv, g, N, d = 1, 4, 1, 80, 8
    K, _, Q = rand_case(rng, B, Hkv, g, N, d)
    n_sink, window = 4, 16
    V = np.zeros((B, Hkv, N, d), np.float32)
    V[:, :, n_sink:N - window, 0] = 1.0                 # indicator of the dropped set in column 0
    c = orc.OracleCache(K, V, [N], [0] * Hkv, n_sink=n_sink, window=window)
    w_comp = c.decode(Q, 1.0)[..., 0]                   # weight Eq.(5) gives the compensation token
    w_true = full_attention(K, V, Q, [N], 1.0, g)[..., 0]
    assert (w_comp > 0).all() and (w_comp <= w_true + 1e-15).all()
    assert (w_comp < w_true - 1e-6).any()


# ----------------------------------------------------------------- I8 / I9 / I10
def test_I8_key_shift_invariance():
    rng = np.random.default_rng(8)
    B, Hkv, g, N, d = 1, 2, 2, 60, 8
    K, V, Q = rand_case(rng, B, Hkv, g, N, d)
    K, V, Q = (np.round(x * 8) / 8 for x in (K, V, Q))              # exact in fp32 after the shift
    u = (np.round(rng.standard_normal(d) * 8) / 8).astype(np.float32)
    a = orc.OracleCache(K, V, [N], [0, 0], 4, 12).decode(Q, 0.5)
    b = orc.OracleCache((K + u).astype(np.float32), V, [N], [0, 0], 4, 12).decode(Q, 0.5)
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)


def test_I9_convex_combination():
    rng = np.random.default_rng(9)
    B, Hkv, g, N, d = 1, 3, 1, 70, 8
    K, V, Q = rand_case(rng, B, Hkv, g, N, d)
    c = orc.OracleCache(K, V, [N], [0] * Hkv, 4, 10)
    out = c.decode(Q, 1.0)
    Vd = f64(V)
    for h in range(Hkv):
        pool = np.concatenate([Vd[0, h, c.kept_of(0, h)], c.vhat[0, h][None]])
        assert (out[0, h] >= pool.min(0) - 1e-12).all() and (out[0, h] <= pool.max(0) + 1e-12).all()
    # all-ones values -> weights sum to one
    ones = np.ones_like(V)
    np.testing.assert_allclose(orc.OracleCache(K, ones, [N], [0] * Hkv, 4, 10).decode(Q, 1.0), 1.0, rtol=1e-13)


def test_I10_gqa_and_permutation():
    rng = np.random.default_rng(10)
    B, Hkv, g, N, d = 2, 2, 4, 48, 8
    K, V, Q = rand_case(rng, B, Hkv, g, N, d)
    mask = [0, 1]
    out = orc.OracleCache(K, V, [N] * B, mask, 4, 8).decode(Q, 0.4)
    # MHA with the KV heads (and the mask) repeated g times
    Km, Vm = np.repeat(K, g, 1), np.repeat(V, g, 1)
    out_mha = orc.OracleCache(Km, Vm, [N] * B, np.repeat(mask, g), 4, 8).decode(Q, 0.4)
    np.testing.assert_allclose(out, out_mha, rtol=1e-13, atol=1e-15)
    # permuting the dropped rows (K and V together) changes nothing
    perm = 4 + rng.permutation(N - 12)
    Kp, Vp = K.copy(), V.copy()
    Kp[:, :, 4:N - 8], Vp[:, :, 4:N - 8] = K[:, :, perm], V[:, :, perm]
    out_p = orc.OracleCache(Kp, Vp, [N] * B, mask, 4, 8).decode(Q, 0.4)
    np.testing.assert_allclose(out[:, :g], out_p[:, :g], rtol=1e-11, atol=1e-13)
    # strided (non-contiguous) storage gives the same answer
    big = np.zeros((B, Hkv, N + 7, d + 0), np.float32); big[:, :, :N] = K
    bigv = np.zeros_like(big); bigv[:, :, :N] = V
    out_s = orc.OracleCache(big[:, :, :N], bigv[:, :, :N], [N] * B, mask, 4, 8).decode(Q, 0.4)
    np.testing.assert_array_equal(out, out_s)


# ----------------------------------------------------------------- I11 and the index table
def read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    return vals


def test_I11_table2_ratio():
    gold = read_golden("table2_compression_ratio.txt")
    n_heads, N = 100, 2_000_000
    n_prot = int(round(gold["protected_head_fraction"] * n_heads))
    window = max(int(gold["buffer_floor"]), N // int(gold["buffer_divisor"]))
    kept = 0
    for h in range(n_heads):
        idx, lo, hi = orc.select(N, h < n_prot, int(gold["sink_tokens"]), window)
        kept += len(idx)
    ratio = n_heads * N / kept
    assert ratio == pytest.approx(gold["compression_ratio"], rel=1e-4)
    assert 1 - 1 / ratio == pytest.approx(gold["reduction"], abs=1e-4)
    # short contexts fall on the floor of the buffer length: at N = 8000, 4004 rows stay
    idx, lo, hi = orc.select(8000, False, 4, max(4000, 8000 // 5))
    assert len(idx) == 4004 and (lo, hi) == (4, 4000)


@pytest.mark.parametrize("N,retr,n_sink,window,exp_kept,exp_D", [
    (10, False, 2, 3, [0, 1, 7, 8, 9], (2, 7)),
    (10, True, 2, 3, list(range(10)), (0, 0)),
    (10, False, 0, 3, [7, 8, 9], (0, 7)),            # no sinks
    (10, False, 2, 0, [0, 1], (2, 10)),              # no window
    (5, False, 2, 3, [0, 1, 2, 3, 4], (0, 0)),       # exactly covered: nothing dropped
    (6, False, 2, 3, [0, 1, 3, 4, 5], (2, 3)),       # one dropped token
    (4, False, 4, 256, [0, 1, 2, 3], (0, 0)),        # shorter than the sinks
    (1, False, 4, 4, [0], (0, 0)),
])
def test_select_closed_form(N, retr, n_sink, window, exp_kept, exp_D):
    idx, lo, hi = orc.select(N, retr, n_sink, window)
    assert list(idx) == exp_kept and (lo, hi) == exp_D
    assert len(idx) + (hi - lo) == N                 # kept and dropped partition the cache


def test_ragged_batch_table():
    rng = np.random.default_rng(11)
    B, Hkv, N, d = 3, 3, 40, 4
    K, V, _ = rand_case(rng, B, Hkv, 1, N, d)
    lens = [40, 9, 25]
    c = orc.OracleCache(K, V, lens, [0, 1, 0], n_sink=4, window=6)
    exp_rows = [[10, 40, 10], [9, 9, 9], [10, 25, 10]]
    exp_nd = [[30, 0, 30], [0, 0, 0], [15, 0, 15]]
    assert c.rows().tolist() == exp_rows and c.N_d.tolist() == exp_nd
    assert list(c.kept_of(2, 0)) == [0, 1, 2, 3, 19, 20, 21, 22, 23, 24]
    np.testing.assert_allclose(c.khat[2, 0], f64(K)[2, 0, 4:19].mean(0), rtol=1e-13)
    np.testing.assert_allclose(c.vhat[0, 2], f64(V)[0, 2, 4:34].mean(0), rtol=1e-13)
    assert (c.khat[:, 1] == 0).all()


# ----------------------------------------------------------------- appends
def test_append_rows_are_kept_rows():
    rng = np.random.default_rng(12)
    B, Hkv, g, N, d = 2, 2, 2, 33, 8
    K, V, Q = rand_case(rng, B, Hkv, g, N, d)
    T = 3
    lens = [33, 21]
    c = orc.OracleCache(K, V, lens, [1, 0], n_sink=2, window=7, max_new=T)
    news = [(rng.standard_normal((B, Hkv, d)).astype(np.float32),
             rng.standard_normal((B, Hkv, d)).astype(np.float32)) for _ in range(T)]
    for kn, vn in news:
        c.append(kn, vn)
    out = c.decode(Q, 0.6)
    assert c.rows().tolist() == [[36, 12], [24, 12]]
    Kd, Vd, Qd = f64(K), f64(V), f64(Q)
    for b in range(B):
        n = lens[b]
        kn = np.stack([f64(x[0])[b] for x in news], 1)      # [Hkv, T, d]
        vn = np.stack([f64(x[1])[b] for x in news], 1)
        for j in range(Hkv * g):
            h = j // g
            if h == 0:        # retrieval: plain attention over prefill rows + appended rows
                Kx = np.concatenate([Kd[b, h, :n], kn[h]]); Vx = np.concatenate([Vd[b, h, :n], vn[h]])
                w = None
            else:             # compressed: the compensation token still stands for the prefill-time D
                keep = [0, 1] + list(range(n - 7, n))
                drop = list(range(2, n - 7))
                Kx = np.concatenate([Kd[b, h, keep], kn[h], Kd[b, h, drop].mean(0)[None]])
                Vx = np.concatenate([Vd[b, h, keep], vn[h], Vd[b, h, drop].mean(0)[None]])
                w = np.ones(len(Kx)); w[-1] = len(drop)
            np.testing.assert_allclose(out[b, j], softmax_attention(Qd[b, j], Kx, Vx, 0.6, w),
                                       rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------------- stored bits
def test_widening_is_exact():
    rng = np.random.default_rng(13)
    x = torch.from_numpy(rng.standard_normal((1, 1, 64, 8)).astype(np.float32) * 100)
    xb = x.to(torch.bfloat16)
    q = torch.zeros(1, 1, 8)
    # with q = 0 and one retrieval head the output is the plain mean of the stored values
    for t, qq in ((x, q), (xb, q.to(torch.bfloat16))):
        out = orc.OracleCache(t, t, [64], [1], 0, 0).decode(qq, 1.0)[0, 0]
        ref = t.to(torch.float64).numpy()[0, 0].mean(0)
        np.testing.assert_allclose(out, ref, rtol=1e-14)
    raw = orc.as_raw(xb)
    assert raw.dtype == np.uint16
    back = torch.from_numpy(raw.view(np.int16)).view(torch.bfloat16)
    assert torch.equal(back, xb)


# ----------------------------------------------------------------- planted mistakes are caught
def test_column_sums_closed_form_and_partition_identity():
    """Rows n of a head hold the value n (+ column c for V): Gauss's sum pins the routine; then
    Eq.(4)'s mean equals (all rows - kept rows) / N_d because D and the kept set partition [0, N)."""
    B, H, N, d = 2, 3, 301, 64
    n = np.arange(N, dtype=np.float32)
    K = np.broadcast_to(n[None, None, :, None], (B, H, N, d)).copy()
    V = K + np.arange(d, dtype=np.float32)
    seq = np.array([301, 120], np.int32)
    cs = orc.column_sums(K, V, seq)
    for b, L in enumerate(seq):
        L = int(L)
        assert (cs[b, :, 0] == L * (L - 1) / 2).all()
        np.testing.assert_array_equal(cs[b, :, 1], L * (L - 1) / 2 + L * np.arange(d)[None, :].repeat(H, 0))
    rng = np.random.default_rng(5)
    K = rng.standard_normal((B, H, N, d)).astype(np.float32)
    V = rng.standard_normal((B, H, N, d)).astype(np.float32)
    mask = np.array([0, 1, 0], np.uint8)
    oc = orc.OracleCache(K, V, seq, mask, 4, 50)
    cs = orc.column_sums(K, V, seq)
    for b in range(B):
        for h in range(H):
            if oc.N_d[b, h] == 0:
                continue
            kept = oc.kept_of(b, h)
            np.testing.assert_allclose((cs[b, h, 0] - K[b, h][kept].astype(np.float64).sum(0)) / oc.N_d[b, h],
                                       oc.khat[b, h], rtol=0, atol=1e-12)
            np.testing.assert_allclose((cs[b, h, 1] - V[b, h][kept].astype(np.float64).sum(0)) / oc.N_d[b, h],
                                       oc.vhat[b, h], rtol=0, atol=1e-12)


def test_pins_catch_planted_mistakes():
    """A dropped N_d factor, a missing ln N_d in the shift, or means taken over the wrong
    range all change the brute-force value by far more than the pin tolerances."""
    rng = np.random.default_rng(14)
    N, d, n_sink, window = 40, 4, 2, 6
    K = rng.standard_normal((N, d)); V = rng.standard_normal((N, d)); q = rng.standard_normal(d)
    keep = list(range(n_sink)) + list(range(N - window, N)); drop = list(range(n_sink, N - window))
    Kf = np.asarray(K, np.float32).reshape(1, 1, N, d); Vf = np.asarray(V, np.float32).reshape(1, 1, N, d)
    qf = np.asarray(q, np.float32).reshape(1, 1, d)
    out = orc.OracleCache(Kf, Vf, [N], [0], n_sink, window).decode(qf, 1.0)[0, 0]
    Kd, Vd, qd = Kf[0, 0].astype(np.float64), Vf[0, 0].astype(np.float64), qf[0, 0].astype(np.float64)

    def variant(nd_weight, rng_lo, rng_hi):
        kh, vh = Kd[rng_lo:rng_hi].mean(0), Vd[rng_lo:rng_hi].mean(0)
        w = np.ones(len(keep) + 1); w[-1] = nd_weight
        return softmax_attention(qd, np.concatenate([Kd[keep], kh[None]]),
                                 np.concatenate([Vd[keep], vh[None]]), 1.0, w)
    good = variant(len(drop), n_sink, N - window)
    np.testing.assert_allclose(out, good, rtol=1e-11, atol=1e-13)
    for bad in (variant(1, n_sink, N - window),              # N_d factor dropped
                variant(len(drop), n_sink + 1, N - window),  # off-by-one at the sink edge
                variant(len(drop), n_sink, N - window + 1),  # off-by-one at the window edge
                variant(len(drop) + 1, n_sink, N - window)): # wrong count
        assert np.abs(bad - out).max() > 1e-4
