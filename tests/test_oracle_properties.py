"""Property tests of the fp64 oracle on small random shapes (hypothesis draws the shapes and the
seeds; CPU only).  Each property follows from Eq.(4) / Eq.(5) alone and is checked against code
that shares nothing with the oracle:

* Eq.(5) says the compensation token counts N_d times: attention over the kept rows plus khat, vhat
  replicated N_d times, by a textbook softmax written here, gives the oracle's output;
* softmax attention does not depend on the order of the cache rows, and Eq.(4) does not depend on
  the order of the dropped rows;
* adding one vector to every key (dropped ones included) shifts every logit, the compensation
  one too, by the same amount: the output does not move;
* the output is a convex combination of the kept values and vhat.
"""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import razor_oracle as orc


def softmax_attention(q, K, V, scale):
    s = scale * (K @ q)
    p = np.exp(s - s.max())
    return (p[:, None] * V).sum(0) / p.sum()


shapes = st.tuples(st.integers(1, 3),            # batch
                   st.integers(1, 3),            # KV heads
                   st.sampled_from([1, 2, 4]),   # group
                   st.integers(6, 60),           # context
                   st.sampled_from([4, 8, 16]),  # head_dim
                   st.integers(0, 4),            # sinks
                   st.integers(0, 12),           # window
                   st.integers(0, 2 ** 31 - 1))  # seed


def draw(shape):
    B, H, g, N, d, n_sink, window, seed = shape
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((B, H, N, d)).astype(np.float32)
    V = rng.standard_normal((B, H, N, d)).astype(np.float32)
    Q = rng.standard_normal((B, H * g, d)).astype(np.float32)
    lens = rng.integers(max(1, N // 2), N + 1, size=B)
    mask = (rng.random(H) < 0.3).astype(np.uint8)
    return rng, K, V, Q, lens, mask


@settings(max_examples=60, deadline=None)
@given(shapes)
def test_compensation_token_counts_n_d_times(shape):
    B, H, g, N, d, n_sink, window, _ = shape
    rng, K, V, Q, lens, mask = draw(shape)
    scale = 1.0 / np.sqrt(d)
    c = orc.OracleCache(K, V, lens, mask, n_sink, window)
    out = c.decode(Q, scale)
    for b in range(B):
        for j in range(H * g):
            h = j // g
            kept = c.kept_of(b, h)
            Kx, Vx = K[b, h, kept].astype(np.float64), V[b, h, kept].astype(np.float64)
            n_d = int(c.N_d[b, h])
            assert n_d == lens[b] - len(kept)
            if n_d:
                dropped = np.setdiff1d(np.arange(lens[b]), kept)
                khat, vhat = K[b, h, dropped].astype(np.float64).mean(0), V[b, h, dropped].astype(np.float64).mean(0)
                Kx = np.concatenate([Kx, np.repeat(khat[None], n_d, 0)])
                Vx = np.concatenate([Vx, np.repeat(vhat[None], n_d, 0)])
            ref = softmax_attention(Q[b, j].astype(np.float64), Kx, Vx, scale)
            np.testing.assert_allclose(out[b, j], ref, rtol=1e-10, atol=1e-12)


@settings(max_examples=40, deadline=None)
@given(shapes)
def test_key_shift_and_dropped_row_order_do_not_matter(shape):
    B, H, g, N, d, n_sink, window, _ = shape
    rng, K, V, Q, lens, mask = draw(shape)
    scale = 1.0 / np.sqrt(d)
    base = orc.OracleCache(K, V, lens, mask, n_sink, window).decode(Q, scale)
    # one vector added to every key of a sequence
    u = rng.standard_normal((B, 1, 1, d))
    K64 = K.astype(np.float64) + u                      # keep the shift exact: hand the oracle fp32 values that
    Ks = K64.astype(np.float32)                         # carry rounding, and compare at the size of that rounding
    shifted = orc.OracleCache(Ks, V, lens, mask, n_sink, window).decode(Q, scale)
    tol = 4e-6 * float(np.abs(K64).max()) * float(np.abs(Q).max()) * d * float(np.abs(V).max())
    np.testing.assert_allclose(shifted, base, rtol=0, atol=max(tol, 1e-9))
    # the dropped rows of every head in another order
    Kp, Vp = K.copy(), V.copy()
    for b in range(B):
        lo, hi = n_sink, int(lens[b]) - window
        if hi - lo >= 2:
            perm = lo + rng.permutation(hi - lo)
            Kp[b, :, lo:hi] = K[b][:, perm]
            Vp[b, :, lo:hi] = V[b][:, perm]
    permuted = orc.OracleCache(Kp, Vp, lens, mask, n_sink, window).decode(Q, scale)
    retr = np.repeat(mask.astype(bool), g)
    np.testing.assert_allclose(permuted[:, ~retr], base[:, ~retr], rtol=1e-9, atol=1e-12)


@settings(max_examples=40, deadline=None)
@given(shapes)
def test_output_is_a_convex_combination(shape):
    B, H, g, N, d, n_sink, window, _ = shape
    rng, K, V, Q, lens, mask = draw(shape)
    c = orc.OracleCache(K, V, lens, mask, n_sink, window)
    out = c.decode(Q * 3.0, 1.0)
    for b in range(B):
        for j in range(H * g):
            h = j // g
            vals = V[b, h, c.kept_of(b, h)].astype(np.float64)
            if c.N_d[b, h]:
                vals = np.concatenate([vals, c.vhat[b, h][None]])
            assert (out[b, j] <= vals.max(0) + 1e-12).all() and (out[b, j] >= vals.min(0) - 1e-12).all()
