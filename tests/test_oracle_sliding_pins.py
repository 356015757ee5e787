"""Pins for the oracle's sliding mode (Algorithm 1 re-applied to the whole sequence after
every generated token: the window slides, Eq.(4) absorbs each token that leaves it).

  S1  brute force at every step: concatenate prefill and generated tokens, select by
      definition, replicate the compensation token N_d times, textbook softmax
  S2  while the sequence fits in sinks + window nothing is dropped: full attention
  S3  without the compensation term it is attention over the sinks and the last L tokens
  S4  equals the one-shot compression of the concatenated sequence (the pinned static path)
  S5  bookkeeping: rows stay at n_sink + window once full, N_d grows by one per token
"""
import numpy as np
import pytest

from oracle import razor_oracle as orc


def softmax_attention(q, K, V, scale, weights=None):
    s = scale * (K @ q)
    if weights is not None:
        s = s + np.log(weights)
    s = s - s.max()
    p = np.exp(s)
    return (p[:, None] * V).sum(0) / p.sum()


def make(rng, B, H, g, N, d, T):
    K = rng.standard_normal((B, H, N, d)).astype(np.float32)
    V = rng.standard_normal((B, H, N, d)).astype(np.float32)
    news = [(rng.standard_normal((B, H, d)).astype(np.float32),
             rng.standard_normal((B, H, d)).astype(np.float32)) for _ in range(T)]
    Qs = [rng.standard_normal((B, H * g, d)).astype(np.float32) for _ in range(T)]
    return K, V, news, Qs


def brute(K, V, news, t, q, b, h, N, retrieval, n_sink, window, scale, use_comp=True):
    """Head (b, h) after t+1 generated tokens, by the definition."""
    Kc = np.concatenate([K[b, h, :N], np.stack([n[0][b, h] for n in news[:t + 1]])]).astype(np.float64)
    Vc = np.concatenate([V[b, h, :N], np.stack([n[1][b, h] for n in news[:t + 1]])]).astype(np.float64)
    T = len(Kc)
    if retrieval or T <= n_sink + window:
        return softmax_attention(q, Kc, Vc, scale)
    keep = list(range(n_sink)) + list(range(T - window, T))
    drop = list(range(n_sink, T - window))
    if not use_comp:
        return softmax_attention(q, Kc[keep], Vc[keep], scale)
    Kx = np.concatenate([Kc[keep], np.repeat(Kc[drop].mean(0)[None], len(drop), 0)])
    Vx = np.concatenate([Vc[keep], np.repeat(Vc[drop].mean(0)[None], len(drop), 0)])
    return softmax_attention(q, Kx, Vx, scale)


@pytest.mark.parametrize("n_sink,window,lens", [(2, 5, [12, 9]), (0, 4, [6, 3]), (3, 3, [3, 7]), (4, 30, [10, 20])])
def test_S1_S3_bruteforce_every_step(n_sink, window, lens):
    rng = np.random.default_rng(21)
    B, H, g, N, d, T = 2, 3, 2, max(lens), 4, 14
    K, V, news, Qs = make(rng, B, H, g, N, d, T)
    mask = [0, 1, 0]
    for use_comp in (True, False):
        c = orc.OracleCache(K, V, lens, mask, n_sink, window, max_new=T, sliding=True)
        for t in range(T):
            c.append(*news[t])
            out = c.decode(Qs[t], 0.5, use_comp=use_comp)
            for b in range(B):
                for j in range(H * g):
                    h = j // g
                    ref = brute(K, V, news, t, Qs[t][b, j].astype(np.float64), b, h, lens[b],
                                mask[h], n_sink, window, 0.5, use_comp)
                    np.testing.assert_allclose(out[b, j], ref, rtol=1e-10, atol=1e-12)


def test_S2_no_drop_while_it_fits():
    rng = np.random.default_rng(22)
    K, V, news, Qs = make(rng, 1, 2, 1, 8, 4, 5)
    c = orc.OracleCache(K, V, [8], [0, 0], 4, 9, max_new=5, sliding=True)
    for t in range(5):
        c.append(*news[t])
        out = c.decode(Qs[t], 1.0)
        assert (c.N_d == 0).all()                       # 8 + 5 = 13 = 4 + 9: still fits
        Kc = np.concatenate([K[0, 0], np.stack([n[0][0, 0] for n in news[:t + 1]])]).astype(np.float64)
        Vc = np.concatenate([V[0, 0], np.stack([n[1][0, 0] for n in news[:t + 1]])]).astype(np.float64)
        np.testing.assert_allclose(out[0, 0], softmax_attention(Qs[t][0, 0].astype(np.float64), Kc, Vc, 1.0),
                                   rtol=1e-12)


def test_S4_equals_one_shot_compression_of_the_concatenated_sequence():
    rng = np.random.default_rng(23)
    B, H, g, N, d, T = 2, 2, 2, 40, 8, 25
    K, V, news, Qs = make(rng, B, H, g, N, d, T)
    lens, mask, n_sink, window = [40, 31], [0, 1], 4, 10
    c = orc.OracleCache(K, V, lens, mask, n_sink, window, max_new=T, sliding=True)
    for t in range(T):
        c.append(*news[t])
        if t not in (0, 9, 24):
            continue
        out = c.decode(Qs[t], 0.3)
        for b in range(B):          # one-shot compression needs per-sequence arrays (ragged)
            n = lens[b]
            Kc = np.concatenate([K[b:b + 1, :, :n], np.stack([x[0][b] for x in news[:t + 1]], 1)[None]], 2)
            Vc = np.concatenate([V[b:b + 1, :, :n], np.stack([x[1][b] for x in news[:t + 1]], 1)[None]], 2)
            one = orc.OracleCache(np.ascontiguousarray(Kc), np.ascontiguousarray(Vc), [n + t + 1], mask,
                                  n_sink, window).decode(Qs[t][b:b + 1], 0.3)
            np.testing.assert_allclose(out[b], one[0], rtol=1e-12, atol=1e-14)


def test_S5_bookkeeping():
    rng = np.random.default_rng(24)
    K, V, news, Qs = make(rng, 1, 2, 1, 20, 4, 12)
    c = orc.OracleCache(K, V, [20], [0, 1], 4, 10, max_new=12, sliding=True)
    assert c.N_d.tolist() == [[6, 0]]
    for t in range(12):
        c.append(*news[t])
        c.decode(Qs[t], 1.0)
        assert c.N_d.tolist() == [[6 + t + 1, 0]]
        assert c.rows().tolist() == [[14, 20 + t + 1]]
    # static mode on the same data keeps growing instead
    s = orc.OracleCache(K, V, [20], [0, 1], 4, 10, max_new=12)
    for t in range(12):
        s.append(*news[t])
    assert s.rows().tolist() == [[26, 32]] and s.N_d.tolist() == [[6, 0]]
