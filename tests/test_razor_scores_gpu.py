"""GPU parity of the head-scoring pass (Sec. 3.3) against the fp64 oracle, through the C ABI.

Bar: scores are means of softmax weights computed from bf16 inputs with fp32 accumulation and
the hardware exp2; relative error <= 1e-4 (plus 1e-7 absolute for near-zero scores).  The
selection derived from them must be the oracle's."""
import numpy as np
import pytest
import torch

import paper_2407_15891_amd as razor
from oracle import razor_oracle as orc
from paper_2407_15891_amd.workloads import make_scoring_workload

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
REL, ABS = 1e-4, 1e-7


def say(msg):
    print(msg, flush=True)


def check(Q, K, scale, period, all_copies, what):
    e, i = razor.head_scores(Q, K, scale, period, all_copies)
    re, ri = orc.head_scores(Q.cpu().contiguous(), K.cpu().contiguous(), scale, period, all_copies)
    e, i = e.cpu().numpy().astype(np.float64), i.cpu().numpy().astype(np.float64)
    assert np.isfinite(e).all() and np.isfinite(i).all(), what
    err = max(np.abs(e - re).max(), np.abs(i - ri).max())
    rel = max((np.abs(e - re) / np.maximum(np.abs(re), 1e-30)).max(), (np.abs(i - ri) / np.maximum(np.abs(ri), 1e-30)).max())
    assert (np.abs(e - re) <= REL * np.abs(re) + ABS).all(), f"{what}: echo, worst relative {rel:.2e}"
    assert (np.abs(i - ri) <= REL * np.abs(ri) + ABS).all(), f"{what}: induction, worst relative {rel:.2e}"
    say(f"    {what}: max-abs {err:.2e}, worst relative {rel:.2e}")
    return e, i, re, ri


@pytest.mark.parametrize("hq,hkv,d,period,n_tokens", [
    (8, 4, 64, 150, None),        # 600 tokens: three query tiles, ragged last one
    (4, 1, 128, 150, None),       # one KV head shared by four query heads
    (4, 2, 128, 100, 257),        # one row into the second tile; 257 is no multiple of the period
    (2, 2, 64, 37, 200),          # a single tile, five and a half repeats
    (6, 3, 128, 256, 1024),       # everything aligned to the tile sizes
    (3, 3, 64, 1, 130),           # period 1: the induction token is the current one
    (1, 1, 64, 1, 2),             # the smallest prompt there is: one scored row
    (2, 1, 128, 7, 33),           # one wave and one row of the next
    (2, 2, 64, 64, 65),           # one scored row, the first of the second stage
    (2, 2, 128, 5, 129),          # one row into the second workgroup
])
@pytest.mark.parametrize("all_copies", [False, True])
def test_scores_parity(hq, hkv, d, period, n_tokens, all_copies):
    say(f"head scores parity Hq={hq} Hkv={hkv} d={d} period={period} N={n_tokens} all_copies={all_copies}")
    w = make_scoring_workload(DEV, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, period=period, n_tokens=n_tokens,
                              n_echo_kv=1, n_induction_kv=1 if hkv > 1 else 0, seed=hq + d)
    check(w.Q, w.K, w.scale, w.period, all_copies, "planted prompt")


def test_scores_parity_on_unstructured_and_peaked_inputs():
    say("head scores parity: Gaussian Q/K, small and large logits, strided views")
    g = torch.Generator(device=DEV); g.manual_seed(5)
    for d, gain in ((128, 1.0), (64, 1.0), (128, 6.0)):       # gain 6: logits of +-100, weights from 1 down to 0
        big_q = torch.randn(5, 700, d + 16, generator=g, device=DEV).mul(gain).to(torch.bfloat16)
        big_k = torch.randn(5, 700, d + 8, generator=g, device=DEV).to(torch.bfloat16)
        Q, K = big_q[:4, 3:650, 8:8 + d], big_k[1:3, 3:650, :d]
        check(Q, K, d ** -0.5, 161, False, f"d={d} gain={gain}")
        check(Q, K, d ** -0.5, 161, True, f"d={d} gain={gain} all copies")


@pytest.mark.parametrize("log2_per_key", [0.25, 1.0, 5.0, -1.0])
def test_scores_with_steadily_climbing_logits(log2_per_key):
    """Logits that rise by a fixed amount per key: the running sum of an interior step passes any
    fixed range again and again (at 5 units per key every 32-key step overflows fp32 against the
    previous reference), so the denominators only come out right if every rebasing does.  With
    period 1 the two targets are the newest key and the one before it, whose weights are not small."""
    say(f"head scores: logits climbing {log2_per_key} log2 units per key")
    N, d = 700, 128
    u = torch.zeros(d); u[3] = 1.0
    ramp = torch.arange(N, dtype=torch.float32) * (log2_per_key * np.log(2.0))
    g = torch.Generator().manual_seed(11)
    K = (0.05 * torch.randn(1, N, d, generator=g) + ramp[None, :, None] * u).to(torch.bfloat16).to(DEV)
    Q = (0.05 * torch.randn(2, N, d, generator=g) + u).to(torch.bfloat16).to(DEV)
    e, i, re, ri = check(Q, K, 1.0, 1, False, f"ramp {log2_per_key}")
    if log2_per_key > 0:
        assert (ri > 0.1).all() and (re > 0.01).all()        # the comparison above was not about zeros


def test_scores_one_hot_prompt_closed_form():
    """The constructed prompt of the oracle's pins, on the GPU: logit beta on matching keys."""
    say("head scores: one-hot prompt")
    N, P, beta, d = 300, 50, 3.0, 64
    tok = np.arange(N) % P
    E = np.eye(d, dtype=np.float32)[:P]
    q = torch.tensor(beta * E[tok]); k_own = torch.tensor(E[tok])
    k_before = torch.cat([torch.zeros(1, d), k_own[:-1]])
    Q = torch.stack([q, q]).to(torch.bfloat16).to(DEV); K = torch.stack([k_own, k_before]).to(torch.bfloat16).to(DEV)
    e, i, _, _ = check(Q, K, 1.0, P, False, "one-hot")
    B = np.exp(beta)
    exp_e0 = np.mean([B / ((m // P + 1) * B + m + 1 - (m // P + 1)) for m in range(P, N)])
    exp_i1 = np.mean([B / ((m // P) * B + m + 1 - (m // P)) for m in range(P, N)])
    assert abs(e[0] - exp_e0) <= REL * exp_e0 and abs(i[1] - exp_i1) <= REL * exp_i1


def test_scores_are_bit_reproducible():
    w = make_scoring_workload(DEV, n_q_heads=8, n_kv_heads=2, head_dim=128, period=300, seed=4)
    a = razor.head_scores(w.Q, w.K, w.scale, w.period)
    b = razor.head_scores(w.Q, w.K, w.scale, w.period)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_selection_from_gpu_scores_is_the_oracles():
    """Four "layers" of 8/4 heads scored one by one, selected together: the mask from the
    library's scores equals the mask from the oracle's, and it contains the planted heads."""
    say("head scores -> selection, four layers")
    e_all, i_all, re_all, ri_all, planted = [], [], [], [], []
    for layer in range(4):
        w = make_scoring_workload(DEV, n_q_heads=8, n_kv_heads=4, head_dim=64, period=120, seed=40 + layer)
        e, i, re, ri = check(w.Q, w.K, w.scale, w.period, False, f"layer {layer}")
        e_all.append(e); i_all.append(i); re_all.append(re); ri_all.append(ri)
        planted += [layer * 4 + j for j in list(w.echo_kv) + list(w.induction_kv)]
    e, i = np.concatenate(e_all), np.concatenate(i_all)
    mask = razor.select_heads(e, i, 2, frac_induction=0.25, frac_echo=0.25)
    np.testing.assert_array_equal(mask, orc.select_heads(np.concatenate(re_all), np.concatenate(ri_all), 2, 0.25, 0.25))
    assert mask[planted].all() and mask.sum() == len(planted)


def test_scores_full_size_sampled_heads():
    """The paper's prompt size (2500 random tokens, four times) on a 32/8 x 128 layer; the oracle
    recomputes two of the 32 heads (an echo-type and an induction-type one)."""
    say("head scores: 10000-token prompt, 32/8 heads x 128, two heads against the oracle")
    w = make_scoring_workload(DEV, n_q_heads=32, n_kv_heads=8, head_dim=128, period=2500, seed=9)
    e, i = razor.head_scores(w.Q, w.K, w.scale, w.period)
    e, i = e.cpu().numpy().astype(np.float64), i.cpu().numpy().astype(np.float64)
    assert np.isfinite(e).all() and np.isfinite(i).all() and (e >= 0).all() and (e + i <= 1 + 1e-6).all()
    for h in (int(w.echo_kv[0]) * 4 + 1, int(w.induction_kv[0]) * 4 + 2):
        say(f"    oracle on head {h}")
        re, ri = orc.head_scores(w.Q[h:h + 1].cpu(), w.K[h // 4:h // 4 + 1].cpu(), w.scale, w.period)
        assert abs(e[h] - re[0]) <= REL * re[0] + ABS and abs(i[h] - ri[0]) <= REL * ri[0] + ABS, (h, e[h], re[0], i[h], ri[0])
    grp = np.argsort(-e)[:4] // 4
    assert set(grp) == set(w.echo_kv)
