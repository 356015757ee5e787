"""Pins for the oracle's ALiBi form (Eq.(1): S = q_m k_n^T - l_h (m - n); each head keeps
only its most recent L_h tokens, Sec. 3.1).

  B0  a 3-token example worked by hand
  B1  full cache + slopes            == torch SDPA with the additive bias -l_h (m - n), fp64
  B2  per-head windows (no sinks)    == SDPA over the last L_h tokens with their true distances
  B3  Theorem 1: with L_h = (2C - ln eps) / l_h, C >= |logit|, every dropped token weighs
      <= eps, and truncating moves the output by <= 2 * (dropped weight) * max|v|
  B4  sliding: at every step == SDPA over the last L_h tokens of prefill + generated text
"""
import math

import numpy as np
import pytest
import torch

from oracle import razor_oracle as orc


def sdpa_bias(q, K, V, scale, slope, q_pos, pos):
    """One query, fp64, library routine with an additive mask."""
    qt = torch.as_tensor(q)[None, None, None, :]
    Kt, Vt = torch.as_tensor(K)[None, None], torch.as_tensor(V)[None, None]
    bias = torch.as_tensor(-slope * (q_pos - np.asarray(pos, np.float64)))[None, None, None, :]
    return torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, attn_mask=bias, scale=scale)[0, 0, 0].numpy()


def test_B0_hand_worked_eq1():
    # d = 1, q = 1, keys all 0, slope = ln 2, positions 0, 1, 2, query at 2:
    # logits -2 ln2, -ln2, 0 -> weights 1/4, 1/2, 1 (sum 7/4); v = 7, 14, 28 -> (7/4 + 7 + 28) / (7/4) = 21
    K = np.zeros((1, 1, 3, 1), np.float32)
    V = np.array([7, 14, 28], np.float32).reshape(1, 1, 3, 1)
    Q = np.ones((1, 1, 1), np.float32)
    c = orc.OracleCache(K, V, [3], [1], 0, 0, alibi_slopes=[math.log(2)])
    assert c.decode(Q, 1.0, use_comp=False)[0, 0, 0] == pytest.approx(21.0, rel=1e-12)
    # keeping only the last 2 tokens: (7 + 28) / (3/2)
    c = orc.OracleCache(K, V, [3], [0], 0, 2, alibi_slopes=[math.log(2)])
    assert c.decode(Q, 1.0, use_comp=False)[0, 0, 0] == pytest.approx(70.0 / 3.0, rel=1e-12)


@pytest.mark.parametrize("g", [1, 4])
def test_B1_B2_full_and_truncated_match_sdpa(g):
    rng = np.random.default_rng(31)
    B, H, N, d, T = 2, 3, 50, 8, 4
    K = rng.standard_normal((B, H, N, d)).astype(np.float32)
    V = rng.standard_normal((B, H, N, d)).astype(np.float32)
    slopes = 2.0 ** -rng.uniform(1, 6, H * g)
    lens = [50, 33]
    news = [(rng.standard_normal((B, H, d)).astype(np.float32), rng.standard_normal((B, H, d)).astype(np.float32))
            for _ in range(T)]
    Q = rng.standard_normal((B, H * g, d)).astype(np.float32)
    for head_window in ([10 ** 6] * H, [7, 20, 1]):
        c = orc.OracleCache(K, V, lens, [0] * H, 0, 0, max_new=T, head_window=head_window, alibi_slopes=slopes)
        for kn, vn in news:
            c.append(kn, vn)
        out = c.decode(Q, 0.4, use_comp=False)
        for b in range(B):
            n = lens[b]
            for j in range(H * g):
                h = j // g
                Kc = np.concatenate([K[b, h, :n], np.stack([x[0][b, h] for x in news])]).astype(np.float64)
                Vc = np.concatenate([V[b, h, :n], np.stack([x[1][b, h] for x in news])]).astype(np.float64)
                pos = np.arange(n + T)
                keep = pos if head_window[h] >= n else np.concatenate([np.arange(n - head_window[h], n), n + np.arange(T)])
                ref = sdpa_bias(Q[b, j].astype(np.float64), Kc[keep], Vc[keep], 0.4, slopes[j], n + T - 1, pos[keep])
                np.testing.assert_allclose(out[b, j], ref, rtol=1e-11, atol=1e-13)


def test_B3_theorem1_vision_scope():
    rng = np.random.default_rng(32)
    H, N, d, eps = 4, 400, 8, 1e-3
    K = rng.standard_normal((1, H, N, d)).astype(np.float32)
    Q = rng.standard_normal((1, H, d)).astype(np.float32)
    slopes = np.array([0.5, 0.25, 0.125, 0.01])
    scale = 0.3
    C = np.abs(scale * np.einsum("hnd,hd->hn", K[0].astype(np.float64), Q[0].astype(np.float64))).max(1)
    L = np.ceil((2 * C - math.log(eps)) / slopes).astype(np.int64)       # Eq.(2) with C in place of the norm bound
    assert L[0] < N and L[3] > N                                          # a local head and a "retrieval" head
    # indicator of the tokens farther than L_h: their total weight under full ALiBi attention
    V = np.zeros((1, H, N, d), np.float32)
    for h in range(H):
        V[0, h, : max(N - L[h], 0), 0] = 1.0
    full = orc.OracleCache(K, V, [N], [1] * H, 0, 0, alibi_slopes=slopes).decode(Q, scale, use_comp=False)
    for h in range(H):
        n_far = max(N - L[h], 0)
        assert full[0, h, 0] <= n_far * eps + 1e-15                      # each far token weighs <= eps
    # truncation to L_h moves the output by at most 2 * (dropped weight) * max|v|
    Vr = rng.standard_normal((1, H, N, d)).astype(np.float32)
    a = orc.OracleCache(K, Vr, [N], [1] * H, 0, 0, alibi_slopes=slopes).decode(Q, scale, use_comp=False)
    b = orc.OracleCache(K, Vr, [N], [0] * H, 0, 0, head_window=L, alibi_slopes=slopes).decode(Q, scale, use_comp=False)
    for h in range(H):
        assert np.abs(a[0, h] - b[0, h]).max() <= 2 * full[0, h, 0] * np.abs(Vr[0, h]).max() + 1e-12
    assert np.abs(a[0, 3] - b[0, 3]).max() == 0.0                        # the long-scope head kept everything


def test_B4_sliding_alibi_every_step():
    rng = np.random.default_rng(33)
    B, H, g, N, d, T = 1, 2, 2, 12, 4, 15
    K = rng.standard_normal((B, H, N, d)).astype(np.float32)
    V = rng.standard_normal((B, H, N, d)).astype(np.float32)
    slopes = np.array([0.3, 0.2, 0.1, 0.05])
    head_window = [5, 100]
    c = orc.OracleCache(K, V, [N], [0, 0], 0, 0, max_new=T, sliding=True, head_window=head_window, alibi_slopes=slopes)
    Kc, Vc = [K[0, h].astype(np.float64) for h in range(H)], [V[0, h].astype(np.float64) for h in range(H)]
    for t in range(T):
        kn = rng.standard_normal((B, H, d)).astype(np.float32); vn = rng.standard_normal((B, H, d)).astype(np.float32)
        Q = rng.standard_normal((B, H * g, d)).astype(np.float32)
        c.append(kn, vn)
        out = c.decode(Q, 0.5, use_comp=False)
        for h in range(H):
            Kc[h] = np.concatenate([Kc[h], kn[0, h][None].astype(np.float64)])
            Vc[h] = np.concatenate([Vc[h], vn[0, h][None].astype(np.float64)])
        Tn = N + t + 1
        for j in range(H * g):
            h = j // g
            keep = np.arange(max(Tn - head_window[h], 0), Tn)
            ref = sdpa_bias(Q[0, j].astype(np.float64), Kc[h][keep], Vc[h][keep], 0.5, slopes[j], Tn - 1, keep)
            np.testing.assert_allclose(out[0, j], ref, rtol=1e-11, atol=1e-13)
