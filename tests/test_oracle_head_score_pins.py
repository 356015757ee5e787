"""Pins for the head-scoring oracle (Sec. 3.3) and the head selection (Sec. 3.3, Table 2,
Sec. 4.1): closed forms on constructed prompts, a library softmax on random data, hand-worked
selections.  The paper prints no score values, so there is no golden fixture for this pass."""
import numpy as np
import pytest
import torch

from oracle import razor_oracle as orc
from paper_2407_15891_amd.workloads import make_scoring_workload


def harmonic_mean_weight(N, K):
    return sum(1.0 / (m + 1) for m in range(K, N)) / (N - K)


def test_uniform_attention_closed_form():
    """Zero queries: every causal row is uniform, A[m, n] = 1 / (m + 1)."""
    N, K, d = 97, 20, 8
    Q = np.zeros((3, N, d), np.float32)
    Kk = np.random.default_rng(0).standard_normal((1, N, d)).astype(np.float32)
    e, i = orc.head_scores(Q, Kk, 0.7, K)
    np.testing.assert_allclose(e, harmonic_mean_weight(N, K), rtol=1e-13)
    np.testing.assert_allclose(i, harmonic_mean_weight(N, K), rtol=1e-13)
    e, i = orc.head_scores(Q, Kk, 0.7, K, all_copies=True)
    copies = sum((m // K) / (m + 1) for m in range(K, N)) / (N - K)
    np.testing.assert_allclose(e, copies, rtol=1e-13)
    np.testing.assert_allclose(i, copies, rtol=1e-13)


def one_hot_prompt(N, K, beta):
    """Token t of the period is unit vector e_t; the query carries beta * e_token."""
    tok = np.arange(N) % K
    E = np.eye(K, dtype=np.float32)
    q = beta * E[tok]
    k_own = E[tok]                                                  # echo-type keys
    k_before = np.concatenate([np.zeros((1, K), np.float32), E[tok[:-1]]])   # induction-type keys
    return q, k_own, k_before


@pytest.mark.parametrize("all_copies", [False, True])
def test_one_hot_prompt_closed_forms(all_copies):
    """Logit beta where the key's vector equals the query's token, 0 elsewhere, so every weight is
    e^beta / (c e^beta + m + 1 - c) or 1 / (...), c = matching keys among positions 0..m."""
    N, K, beta = 53, 12, 2.0
    q, k_own, k_before = one_hot_prompt(N, K, beta)
    Q = np.stack([q, q]); Kk = np.stack([k_own, k_before])           # head 0: echo type, head 1: induction type
    e, i = orc.head_scores(Q, Kk, 1.0, K, all_copies=all_copies)
    B = np.exp(beta)
    exp_e = np.zeros(2); exp_i = np.zeros(2)
    for m in range(K, N):
        prev = m // K                                               # earlier copies of the current token
        use = prev if all_copies else 1
        # echo-type keys: positions m, m-K, ... match (prev + 1 of them); the token after a copy never does
        den = (prev + 1) * B + (m + 1 - (prev + 1))
        exp_e[0] += use * B / den
        exp_i[0] += use * 1.0 / den
        # induction-type keys: positions m+1-K, m+1-2K, ... match (prev of them); the copies themselves do not
        den = prev * B + (m + 1 - prev)
        exp_e[1] += use * 1.0 / den
        exp_i[1] += use * B / den
    np.testing.assert_allclose(e, exp_e / (N - K), rtol=1e-12)
    np.testing.assert_allclose(i, exp_i / (N - K), rtol=1e-12)
    assert e[0] > 5 * i[0] and i[1] > 5 * e[1]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_against_library_softmax_with_grouped_heads(dtype):
    g = torch.Generator().manual_seed(3)
    Hq, Hkv, N, d, K, scale = 6, 2, 75, 16, 19, 0.31
    Q = torch.randn(Hq, N, d, generator=g).to(dtype)
    Kk = torch.randn(Hkv, N, d, generator=g).to(dtype)
    logits = scale * torch.einsum("hmd,hnd->hmn", Q.double(), Kk.double().repeat_interleave(Hq // Hkv, 0))
    causal = torch.ones(N, N, dtype=torch.bool).tril()
    A = torch.softmax(logits.masked_fill(~causal, float("-inf")), dim=-1).numpy()
    m = np.arange(K, N)
    e, i = orc.head_scores(Q, Kk, scale, K)
    np.testing.assert_allclose(e, A[:, m, m - K].mean(axis=1), rtol=1e-12)
    np.testing.assert_allclose(i, A[:, m, m - K + 1].mean(axis=1), rtol=1e-12)
    e, i = orc.head_scores(Q, Kk, scale, K, all_copies=True)
    exp_e = sum(A[:, mm, mm - j * K] for mm in m for j in range(1, mm // K + 1)) / (N - K)
    exp_i = sum(A[:, mm, mm - j * K + 1] for mm in m for j in range(1, mm // K + 1)) / (N - K)
    np.testing.assert_allclose(e, exp_e, rtol=1e-12)
    np.testing.assert_allclose(i, exp_i, rtol=1e-12)
    # plausible mistakes are far outside that tolerance: neighbouring position, no causal mask,
    # the other operand order, the mean taken over all N rows
    full = torch.softmax(logits, dim=-1).numpy()
    swapped = torch.softmax((scale * torch.einsum("hnd,hmd->hmn", Q.double(), Kk.double().repeat_interleave(Hq // Hkv, 0)))
                            .masked_fill(~causal, float("-inf")), dim=-1).numpy()
    e, i = orc.head_scores(Q, Kk, scale, K)
    for bad in (A[:, m, m - K - 1].mean(axis=1), full[:, m, m - K].mean(axis=1),
                swapped[:, m, m - K].mean(axis=1), A[:, m, m - K].sum(axis=1) / N):
        assert np.abs(bad - e).max() > 1e-4
    assert np.abs(A[:, m, m - K + 2].mean(axis=1) - i).max() > 1e-4


def test_scores_are_attention_mass():
    w = make_scoring_workload(n_q_heads=8, n_kv_heads=4, head_dim=32, period=40, seed=2)
    e1, i1 = orc.head_scores(w.Q, w.K, w.scale, w.period)
    e2, i2 = orc.head_scores(w.Q, w.K, w.scale, w.period, all_copies=True)
    assert (e1 > 0).all() and (i1 > 0).all()
    assert (e2 >= e1).all() and (i2 >= i1).all() and (e2 + i2 <= 1 + 1e-12).all()
    # the heads built as echo / induction heads come out on top of their own score
    grp = w.Hq // w.Hkv
    assert set(np.argsort(-e1)[:grp] // grp) == set(w.echo_kv)
    assert set(np.argsort(-i1)[:grp] // grp) == set(w.induction_kv)
    with pytest.raises(AssertionError):
        orc.head_scores(w.Q, w.K, w.scale, w.N)                      # no position has a previous copy


# ----------------------------------------------------------------- selection
def test_protected_counts_of_table2():
    """Table 2: top 14 % by induction score and top 1 % by echo score.  On 1024 heads (32 layers
    of 32) that is 143 and 10 heads, on 32 heads 4 and 0."""
    assert orc.protected_count(1024, 0.14) == 143 and orc.protected_count(1024, 0.01) == 10
    assert orc.protected_count(32, 0.14) == 4 and orc.protected_count(32, 0.01) == 0
    assert orc.protected_count(50, 0.01) == 1                        # 0.5 rounds up


def test_selection_by_hand():
    ind = [0.1, 0.9, 0.2, 0.8, 0.0, 0.3, 0.05, 0.01, 0.0, 0.0]
    ech = [0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.00, 0.70, 0.6, 0.0]
    # 10 heads: top 20 % induction = heads 1, 3; top 10 % echo = head 7
    np.testing.assert_array_equal(orc.select_heads(ech, ind, 1, 0.2, 0.1), [0, 1, 0, 1, 0, 0, 0, 1, 0, 0])
    # grouped by 2: a KV head is retrieval when either of its query heads is (Sec. 4.1)
    np.testing.assert_array_equal(orc.select_heads(ech, ind, 2, 0.2, 0.1), [1, 1, 0, 1, 0])
    np.testing.assert_array_equal(orc.select_heads(ech, ind, 5, 0.2, 0.1), [1, 1])
    np.testing.assert_array_equal(orc.select_heads(ech, ind, 1, 0.0, 0.0), np.zeros(10))
    # equal scores: the lower index wins
    np.testing.assert_array_equal(orc.select_heads([0] * 4, [1, 1, 1, 1], 1, 0.5, 0.0), [1, 1, 0, 0])
    # a head chosen twice counts once
    np.testing.assert_array_equal(orc.select_heads([0, 9, 0, 0], [0, 9, 0, 0], 1, 0.25, 0.25), [0, 1, 0, 0])
