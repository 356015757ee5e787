"""Seeded synthetic inputs shaped like the paper's long-context workloads.

This module only draws tensors and picks configuration constants.  It holds
none of the method's arithmetic (no selection, no means, no attention) and is
the one piece shared by the tests of the CPU oracle and of the HIP library.

The paper evaluates on trained long-context models (Llama-2 MHA 32x128,
Llama-3 GQA 32/8x128, a 70B-class GQA 64/8x128) with about 15 % retrieval
heads, 4 sink tokens and an N/5-style recent window (Table 2).  No weights or
benchmark prompts are used here: post-RoPE K/V/Q are replaced by seeded
Gaussian tensors of those shapes with the structure each configuration names
(large-norm sink keys, outlier channels, ragged lengths).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch


@dataclass
class Workload:
    name: str
    cfg: int
    B: int
    Hq: int
    Hkv: int
    d: int
    N: int                      # padded context (dim 2 of K/V)
    dtype: torch.dtype
    seq_lens: np.ndarray        # int32 [B]
    mask: np.ndarray            # uint8 [Hkv], 1 = retrieval KV head
    n_sink: int
    window: int
    max_new: int
    scale: float
    seed: int
    device: torch.device
    K: Optional[torch.Tensor] = None   # [B, Hkv, N, d]
    V: Optional[torch.Tensor] = None
    decode_steps: int = 1
    _gen: Optional[torch.Generator] = field(default=None, repr=False)

    def step_inputs(self, t: int, append: bool = True):
        """(Q [B,Hq,d], k_new [B,Hkv,d] | None, v_new | None) of decode step t."""
        g = torch.Generator(device=self.device)
        g.manual_seed(self.seed * 7919 + 104729 * (t + 1))
        Q = torch.randn(self.B, self.Hq, self.d, generator=g, device=self.device,
                        dtype=torch.float32).to(self.dtype)
        if not append:
            return Q, None, None
        k = torch.randn(self.B, self.Hkv, self.d, generator=g, device=self.device,
                        dtype=torch.float32).to(self.dtype)
        v = torch.randn(self.B, self.Hkv, self.d, generator=g, device=self.device,
                        dtype=torch.float32).to(self.dtype)
        return Q, k, v


def _randn(shape, gen, device, dtype):
    """N(0,1) drawn in fp32 slabs over dim 0 then cast, to bound peak memory."""
    out = torch.empty(shape, device=device, dtype=dtype)
    for b in range(shape[0]):
        out[b] = torch.randn(shape[1:], generator=gen, device=device, dtype=torch.float32).to(dtype)
    return out


def retrieval_pairs_stack(n_layers: int, Hkv: int, frac: float, seed: int) -> np.ndarray:
    """Config 5: round(frac * n_layers * Hkv) (layer, kv-head) pairs without replacement."""
    rng = np.random.default_rng(seed)
    total = n_layers * Hkv
    k = int(round(frac * total))
    flat = np.zeros(total, dtype=np.uint8)
    flat[rng.choice(total, size=k, replace=False)] = 1
    return flat.reshape(n_layers, Hkv)


def make_workload(cfg: int, device="cpu", *, context: Optional[int] = None,
                  batch: Optional[int] = None, window: Optional[int] = None,
                  max_new: Optional[int] = None, layer: int = 0,
                  materialize: bool = True, mask: Optional[np.ndarray] = None) -> Workload:
    """Build configuration `cfg` (1..5).  `context` / `batch` / `window` shrink or
    override it for tests; the recipe (distribution, structure, mask rule) stays."""
    device = torch.device(device)
    seed = 1000 * cfg + layer
    rng = np.random.default_rng(seed)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)

    if cfg == 1:
        B, Hq, Hkv, d, N, dt = batch or 1, 8, 8, 64, context or 2048, torch.float32
        win = 256 if window is None else window
        m = np.zeros(Hkv, np.uint8); m[[0, 5]] = 1
        steps, name = 1, "c1 MHA 8x64 fp32"
    elif cfg == 2:
        B, Hq, Hkv, d, N, dt = batch or 1, 32, 32, 128, context or 32768, torch.bfloat16
        win = (N * 20) // 100 if window is None else window
        m = np.zeros(Hkv, np.uint8); m[rng.choice(Hkv, 5, replace=False)] = 1
        steps, name = 64, "c2 Llama-2-7B-shaped MHA 32x128 bf16"
    elif cfg == 3:
        B, Hq, Hkv, d, N, dt = batch or 4, 32, 8, 128, context or 131072, torch.bfloat16
        win = max(4096, (N * 15) // 100) if window is None else window
        m = np.zeros(Hkv, np.uint8); m[rng.choice(Hkv, 2, replace=False)] = 1
        steps, name = 1, "c3 Llama-3-8B-shaped GQA 32/8x128 bf16"
    elif cfg == 4:
        B, Hq, Hkv, d, N, dt = batch or 16, 64, 8, 128, context or 65536, torch.bfloat16
        win = 2048 if window is None else window
        m = np.zeros(Hkv, np.uint8); m[rng.choice(Hkv, max(1, round(0.15 * Hkv)), replace=False)] = 1
        steps, name = 1, "c4 70B-class GQA 64/8x128 bf16 ragged"
    elif cfg == 5:
        B, Hq, Hkv, d, N, dt = batch or 8, 32, 8, 128, context or 131072, torch.bfloat16
        win = max(4096, (N * 15) // 100) if window is None else window
        m = retrieval_pairs_stack(32, Hkv, 0.15, 5000)[layer]
        steps, name = 256, f"c5 8B-shaped stack layer {layer}"
    else:
        raise ValueError(f"unknown config {cfg}")
    if mask is not None:
        m = np.ascontiguousarray(mask, dtype=np.uint8)
        assert m.shape == (Hkv,)

    if cfg == 4:
        lo = max(1, N // 8)
        seq_lens = rng.integers(lo, N + 1, size=B).astype(np.int32)
    else:
        seq_lens = np.full(B, N, dtype=np.int32)

    w = Workload(name=name, cfg=cfg, B=B, Hq=Hq, Hkv=Hkv, d=d, N=N, dtype=dt,
                 seq_lens=seq_lens, mask=m, n_sink=4, window=int(win),
                 max_new=steps if max_new is None else max_new,
                 scale=1.0 / float(np.sqrt(d)), seed=seed, device=device,
                 decode_steps=steps, _gen=gen)
    if not materialize:
        return w

    K = _randn((B, Hkv, N, d), gen, device, dt)
    V = _randn((B, Hkv, N, d), gen, device, dt)
    if cfg == 1:
        K[:, :, :4, :] *= 4            # sink keys draw large logits
    if cfg == 2:
        for t in (K, V):               # 4 outlier channels per (head, tensor), x8
            for h in range(Hkv):
                ch = torch.from_numpy(rng.choice(d, 4, replace=False)).to(device)
                t[:, h, :, ch] *= 8
    w.K, w.V = K, V
    return w


# ----------------------------------------------------------------------------------------------
# Inputs of the head-scoring pass (Sec. 3.3): one prompt of `period` random tokens repeated.

@dataclass
class ScoringWorkload:
    Hq: int
    Hkv: int
    d: int
    N: int                      # tokens in the prompt
    period: int                 # tokens before the prompt repeats
    scale: float
    Q: torch.Tensor             # [Hq, N, d], as after the rotary transformation
    K: torch.Tensor             # [Hkv, N, d]
    tokens: np.ndarray          # int64 [N]
    echo_kv: np.ndarray         # KV heads built to look back at the previous copy of the current token
    induction_kv: np.ndarray    # KV heads built to look at the token after that copy


def make_scoring_workload(device="cpu", *, n_q_heads: int = 32, n_kv_heads: int = 8, head_dim: int = 128,
                          period: int = 2500, n_tokens: Optional[int] = None, n_echo_kv: int = 1,
                          n_induction_kv: int = 1, seed: int = 0,
                          dtype: torch.dtype = torch.bfloat16) -> ScoringWorkload:
    """The paper feeds a trained model 2500 random tokens repeated 4 times and reads its attention
    maps.  There are no weights here, so Q and K are drawn directly with the structure that makes
    such a prompt informative: every token id has a random unit embedding; a query carries the
    embedding of its own token; the keys of an "echo" KV head carry the embedding of their own
    token, those of an "induction" KV head the embedding of the token before them, all other KV
    heads only noise.  Every key head also has one large first key (a sink) along a direction all
    queries share.  Query heads of one group differ in how strongly they carry the token embedding,
    so scores vary inside a group."""
    N = 4 * period if n_tokens is None else n_tokens
    assert n_q_heads % n_kv_heads == 0 and n_echo_kv + n_induction_kv <= n_kv_heads and 1 <= period < N
    dev = torch.device(device)
    g = torch.Generator(device="cpu")
    g.manual_seed(977 * seed + 31)
    first = torch.randint(0, 50000, (period,), generator=g)
    tokens = first.repeat((N + period - 1) // period)[:N]
    ids = torch.unique(tokens, return_inverse=True)[1]                     # dense ids of the tokens used
    emb = torch.randn(int(ids.max()) + 1, head_dim, generator=g)
    emb = emb / emb.norm(dim=1, keepdim=True)
    own = emb[ids]                                                         # [N, d]
    before = torch.cat([torch.zeros(1, head_dim), own[:-1]])               # embedding of the previous token
    sink_dir = torch.randn(head_dim, generator=g)
    sink_dir = sink_dir / sink_dir.norm()
    kinds = torch.randperm(n_kv_heads, generator=g)
    echo_kv = np.sort(kinds[:n_echo_kv].numpy())
    induction_kv = np.sort(kinds[n_echo_kv:n_echo_kv + n_induction_kv].numpy())
    gain = float(head_dim) ** 0.5
    K = 0.5 * torch.randn(n_kv_heads, N, head_dim, generator=g)
    for j in echo_kv:
        K[j] += gain * own
    for j in induction_kv:
        K[j] += gain * before
    K[:, 0] += 4.0 * gain * sink_dir
    strength = 0.3 + 0.7 * torch.rand(n_q_heads, generator=g)               # per query head
    Q = 0.5 * torch.randn(n_q_heads, N, head_dim, generator=g)
    Q += gain * strength[:, None, None] * own[None]
    Q += 0.25 * gain * sink_dir
    return ScoringWorkload(Hq=n_q_heads, Hkv=n_kv_heads, d=head_dim, N=N, period=period,
                           scale=float(head_dim) ** -0.5, Q=Q.to(dtype).to(dev), K=K.to(dtype).to(dev),
                           tokens=tokens.numpy(), echo_kv=echo_kv, induction_kv=induction_kv)
