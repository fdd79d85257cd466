"""Seeded synthetic per-layer Q/K/V tensors shaped like Llama-3-8B / Mistral-7B attention.

Input generation only: no attention arithmetic, no selection, no softmax lives here.  Both the
CPU oracle's tests and the HIP path's tests / benchmark draw their inputs from this module so
that the two sides always consume identical arrays.

Recipe (stands in for real prompts, whose data and model weights are not available):
  * queries: one stationary AR(1) chain per (sequence, query head) over the ``w + T`` positions
    that the method reads (observation window, then ``T`` decode steps):
    ``x_0 ~ N(0, I/(1-rho^2))``, ``x_t = rho x_{t-1} + eps_t``, ``eps_t ~ N(0, I)``.  Nearby
    queries are therefore similar (neighbour cosine ~ rho), which is the paper's observation Q1
    (Sec. 3.1.1).
  * keys / values: iid N(0,1); per (sequence, KV head) ``n_heavy`` distinct prefix positions in
    ``[1, P)`` have their key row scaled x4 (heavy hitters), and position 0's key row is scaled
    x6 (attention sink).
  * values are rounded to the storage dtype (bf16 round-to-nearest-even, or fp32) before anyone
    reads them.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import torch


@dataclasses.dataclass
class Workload:
    """Shapes of one synthetic workload (names follow the paper / problem statement)."""
    name: str
    batch: int                 # sequences (a layer stack is passed as extra batch entries)
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_lens: List[int]        # prompt length n_b per sequence, window included
    window: int                # w
    budget: int                # B, window included
    pool_kernel: int           # k (odd)
    dtype: str                 # "bf16" | "fp32"
    decode_steps: int          # T
    rho: float = 0.9
    n_heavy: int = 8
    theta1: float = 0.7
    theta2: float = 0.85

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32


BASE_SEED = 20250719


def config(idx: int, *, layers: Optional[int] = None, budget: Optional[int] = None,
           batch: Optional[int] = None, decode_steps: Optional[int] = None) -> Workload:
    """The five workload shapes.  ``layers``/``budget``/``batch`` shrink or pick a variant."""
    if idx == 1:
        return Workload("cfg1_small_fp32", 1, 8, 2, 64, [512], 16, 64, 5, "fp32",
                        decode_steps or 16)
    if idx == 2:
        return Workload("cfg2_llama8b_8k", 1, 32, 8, 128, [8192], 32, 512, 7, "bf16",
                        decode_steps or 128)
    if idx == 3:
        L = layers or 32
        return Workload(f"cfg3_llama8b_32k_x{L}layers_B{budget or 512}", L, 32, 8, 128,
                        [32768] * L, 32, budget or 512, 7, "bf16", decode_steps or 256)
    if idx == 4:
        nb = batch or 64
        g = torch.Generator().manual_seed(BASE_SEED + 4000)
        lens = torch.randint(4096, 16384 + 1, (nb,), generator=g).tolist()
        return Workload(f"cfg4_mistral7b_batch{nb}_varlen", nb, 32, 8, 128, lens, 32,
                        budget or 1024, 7, "bf16", decode_steps or 8)
    if idx == 5:
        return Workload("cfg5_long_131k", 1, 32, 8, 128, [131072], 64, budget or 4096, 7,
                        "bf16", decode_steps or 8)
    raise ValueError(f"unknown config {idx}")


def ar1_queries(wl: Workload, steps: int, seed: int, device="cpu") -> torch.Tensor:
    """[steps][batch][Hq][D] fp32 AR(1) chain along the first axis."""
    g = torch.Generator(device=device).manual_seed(seed)
    shape = (wl.batch, wl.n_q_heads, wl.head_dim)
    out = torch.empty((steps,) + shape, dtype=torch.float32, device=device)
    x = torch.randn(shape, generator=g, device=device) / (1.0 - wl.rho ** 2) ** 0.5
    out[0] = x
    for t in range(1, steps):
        x = wl.rho * x + torch.randn(shape, generator=g, device=device)
        out[t] = x
    return out


def make_inputs(wl: Workload, seed: int = BASE_SEED, device="cpu") -> dict:
    """Build every tensor one compress + ``T`` decode steps need.

    Returns a dict of tensors on ``device``:
      q_win  [batch][Hq][w][D]      window queries, storage dtype
      q_dec  [T][batch][Hq][D]      decode queries (AR(1) continuation), storage dtype
      k, v   packed varlen [sum_b Hkv*n_b*D] viewed flat; sequence b starts at token
             seq_offsets[b]; inside a sequence the layout is [Hkv][n_b][D]
      seq_offsets [batch+1] int32
    """
    dt = wl.torch_dtype
    w, T = wl.window, wl.decode_steps
    q = ar1_queries(wl, w + T, seed, device)                     # [w+T][b][Hq][D]
    q_win = q[:w].permute(1, 2, 0, 3).contiguous().to(dt)         # [b][Hq][w][D]
    q_dec = q[w:].contiguous().to(dt)                             # [T][b][Hq][D]

    offs = [0]
    for n in wl.seq_lens:
        offs.append(offs[-1] + n)
    total = offs[-1]
    Hkv, D = wl.n_kv_heads, wl.head_dim
    k = torch.empty(total * Hkv * D, dtype=dt, device=device)
    v = torch.empty(total * Hkv * D, dtype=dt, device=device)
    gk = torch.Generator(device=device)
    gpos = torch.Generator()                                      # positions always drawn on CPU
    for b, n in enumerate(wl.seq_lens):
        gk.manual_seed(seed + 7919 * (b + 1))
        gpos.manual_seed(seed + 104729 * (b + 1))
        lo, hi = offs[b] * Hkv * D, offs[b + 1] * Hkv * D
        kb = torch.randn((Hkv, n, D), generator=gk, device=device, dtype=torch.float32)
        P = n - w
        for g in range(Hkv):
            if P > 1 and wl.n_heavy > 0:
                cnt = min(wl.n_heavy, P - 1)
                pos = (torch.randperm(P - 1, generator=gpos)[:cnt] + 1).to(device)
                kb[g, pos] *= 4.0
            kb[g, 0] *= 6.0
        k[lo:hi] = kb.to(dt).reshape(-1)
        del kb
        vb = torch.randn((Hkv, n, D), generator=gk, device=device, dtype=torch.float32)
        v[lo:hi] = vb.to(dt).reshape(-1)
        del vb
    seq_offsets = torch.tensor(offs, dtype=torch.int32, device=device)
    return dict(q_win=q_win, q_dec=q_dec, k=k, v=v, seq_offsets=seq_offsets)


def seq_view(flat: torch.Tensor, wl: Workload, b: int) -> torch.Tensor:
    """[Hkv][n_b][D] view of sequence ``b`` inside a packed K or V buffer."""
    Hkv, D = wl.n_kv_heads, wl.head_dim
    lo = sum(wl.seq_lens[:b]) * Hkv * D
    n = wl.seq_lens[b]
    return flat[lo:lo + n * Hkv * D].view(Hkv, n, D)


def full_queries(wl: Workload, x: dict, seed: int = BASE_SEED, device="cpu") -> torch.Tensor:
    """Every prompt query (what a strategy that scores with all queries reads), packed like K
    but with Hq heads: sequence b starts at token seq_offsets[b], inside [Hq][n_b][D].  Per
    (sequence, head) a stationary AR(1) chain along the positions (same rho as the window
    chain); the last w positions are exactly x["q_win"], so Q_{-1} is the same query."""
    dt = wl.torch_dtype
    Hq, D, w, rho = wl.n_q_heads, wl.head_dim, wl.window, wl.rho
    C = 64                                                        # positions generated per step
    j = torch.arange(C, device=device, dtype=torch.float32)
    tri = torch.tril(rho ** (j[:, None] - j[None, :]).clamp(min=0.0))        # tri[j][s] = rho^(j-s), s <= j
    carry = (rho ** (j + 1.0))[:, None, None]
    parts = []
    g = torch.Generator(device=device)
    for b, n in enumerate(wl.seq_lens):
        g.manual_seed(seed + 15485863 * (b + 1))
        m = max(n - w, 0)
        chain = torch.empty((m, Hq, D), dtype=torch.float32, device=device)
        prev = torch.randn((Hq, D), generator=g, device=device) / (1.0 - rho ** 2) ** 0.5
        for t0 in range(0, m, C):
            c = min(C, m - t0)
            e = torch.randn((c, Hq, D), generator=g, device=device)
            blk = torch.einsum("js,shd->jhd", tri[:c, :c], e) + carry[:c] * prev
            chain[t0:t0 + c] = blk
            prev = blk[c - 1]
        qb = torch.cat([chain.permute(1, 0, 2).to(dt), x["q_win"][b][:, max(w - n, 0):]], dim=1)   # [Hq][n][D]
        parts.append(qb.reshape(-1))
    return torch.cat(parts)


def seq_view_q(flat: torch.Tensor, wl: Workload, b: int) -> torch.Tensor:
    """[Hq][n_b][D] view of sequence ``b`` inside a packed full-query buffer."""
    Hq, D = wl.n_q_heads, wl.head_dim
    lo = sum(wl.seq_lens[:b]) * Hq * D
    n = wl.seq_lens[b]
    return flat[lo:lo + n * Hq * D].view(Hq, n, D)
