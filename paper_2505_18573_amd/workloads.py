"""Seeded synthetic inputs shaped like the paper's training setup.

This module only *generates inputs* (logits, temperatures, target ids, rewards,
CSR group offsets).  It holds none of the method's arithmetic and imports
neither the HIP binding nor the CPU oracle; both are fed from here so that
they see identical stored values.

Shapes follow the paper's Training Details (Section 5.1): 64 prompts x 8
rollouts per step, a Qwen-family vocabulary of 151,936 entries, rollout
budgets that differ per prompt once the dynamic budget (Algorithm 1) is on.
The paper's datasets are not needed: the cost and the numerics of the
vocabulary pass depend on shapes, dtypes and how peaked the rows are, not on
the text behind them.

All generators take a torch device.  Large configs are generated on the GPU in
bounded chunks; the oracle is handed host copies of the same stored values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch

V_QWEN = 151_936


@dataclass
class Workload:
    """One batch of inputs.  Fields that a config does not use are None."""
    name: str
    seed: int
    logits: torch.Tensor                      # [rows, V] bf16 or fp32, row-major
    tau_rows: Optional[torch.Tensor] = None   # [rows] fp32, or None -> tau_scalar
    tau_scalar: float = 1.0
    target_ids: Optional[torch.Tensor] = None  # [rows] int32
    row_mask: Optional[torch.Tensor] = None    # [rows] uint8
    rewards: Optional[torch.Tensor] = None     # [N] fp32
    group_offsets: Optional[torch.Tensor] = None  # [B+1] int32
    notes: dict = field(default_factory=dict)

    @property
    def rows(self) -> int:
        return int(self.logits.shape[0])

    @property
    def V(self) -> int:
        return int(self.logits.shape[1])


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _normal_rows(rows: int, V: int, sigma: float, dtype, g: torch.Generator, device,
                 chunk_rows: int = 2048) -> torch.Tensor:
    """N(0, sigma^2) logits stored in `dtype`, generated in bounded chunks."""
    out = torch.empty((rows, V), dtype=dtype, device=device)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        x = torch.randn((r1 - r0, V), generator=g, device=device, dtype=torch.float32)
        out[r0:r1] = (x * sigma).to(dtype)
        del x
    return out


def _boost_random_columns(logits: torch.Tensor, k: int, boost: float, g: torch.Generator):
    """Add `boost` to k distinct random columns per row (done in fp32, stored back)."""
    rows, V = logits.shape
    dev = logits.device
    cols = torch.empty((rows, k), dtype=torch.int64, device=dev)
    for r0 in range(0, rows, 4096):
        r1 = min(rows, r0 + 4096)
        # k distinct columns: top-k of uniform noise would cost rows*V; sample with
        # replacement, then repair duplicates by re-drawing (k << V, so this is rare).
        c = torch.randint(0, V, (r1 - r0, k), generator=g, device=dev)
        for _ in range(8):
            s, _idx = torch.sort(c, dim=1)
            dup = torch.zeros_like(c, dtype=torch.bool)
            dup[:, 1:] = s[:, 1:] == s[:, :-1]
            if not bool(dup.any()):
                c = s
                break
            redraw = torch.randint(0, V, c.shape, generator=g, device=dev)
            c = torch.where(dup, redraw, s)
        cols[r0:r1] = c
    vals = torch.gather(logits, 1, cols).float() + boost
    logits.scatter_(1, cols, vals.to(logits.dtype))
    return cols


def tiny(device="cpu", seed: int = 0) -> Workload:
    """Config 1: 8 prompts x 4 rollouts = 32 rows, V = 1024, fp32 N(0, 2^2), tau = 1."""
    g = _gen(seed, device)
    B, G, V = 8, 4, 1024
    logits = _normal_rows(B * G, V, 2.0, torch.float32, g, device)
    rewards = (torch.rand(B * G, generator=g, device=device) < 0.5).float()
    offsets = torch.arange(0, B * G + 1, G, dtype=torch.int32, device=device)
    targets = torch.randint(0, V, (B * G,), generator=g, device=device).to(torch.int32)
    return Workload("tiny", seed, logits, None, 1.0, targets, None, rewards, offsets)


def decode_step(device, seed: int = 1, prompts: int = 64, rollouts: int = 8,
                V: int = V_QWEN) -> Workload:
    """Config 2: prompts x rollouts rows, bf16 N(0, 3^2), 20 random columns per row
    boosted by +8 (a peaked next-token distribution), per-row tau ~ U[0.6, 1.4]."""
    g = _gen(seed, device)
    rows = prompts * rollouts
    logits = _normal_rows(rows, V, 3.0, torch.bfloat16, g, device)
    _boost_random_columns(logits, min(20, V), 8.0, g)
    tau = (0.6 + 0.8 * torch.rand(rows, generator=g, device=device)).float()
    return Workload("decode_step", seed, logits, tau, 1.0)


# group-size mix of config 3: (size, how many groups)
_DYN_MIX = ((2, 32), (4, 32), (8, 40), (16, 16), (32, 8))


def dynamic_budget_groups(device, seed: int = 2, scale: int = 1):
    """CSR offsets and rewards of config 3 (without logits): 128*scale prompts with
    group sizes from {2,4,8,16,32} in a seeded permutation, per-prompt success rate
    p ~ Beta(1/2, 1/2), rewards ~ Bernoulli(p); group 0 forced all-0, group 1 all-1."""
    rng = np.random.Generator(np.random.PCG64(seed))
    sizes = np.concatenate([np.full(cnt * scale, sz, dtype=np.int64) for sz, cnt in _DYN_MIX])
    sizes = sizes[rng.permutation(sizes.size)]
    offsets = np.zeros(sizes.size + 1, dtype=np.int64)
    np.cumsum(sizes, out=offsets[1:])
    p = rng.beta(0.5, 0.5, size=sizes.size)
    rewards = np.empty(int(offsets[-1]), dtype=np.float32)
    for gi in range(sizes.size):
        lo, hi = offsets[gi], offsets[gi + 1]
        rewards[lo:hi] = (rng.random(hi - lo) < p[gi]).astype(np.float32)
    rewards[offsets[0]:offsets[1]] = 0.0
    rewards[offsets[1]:offsets[2]] = 1.0
    return (torch.from_numpy(offsets.astype(np.int32)).to(device),
            torch.from_numpy(rewards).to(device))


def dynamic_budgets(device, seed: int = 2, V: int = V_QWEN) -> Workload:
    """Config 3: one logit row per rollout of `dynamic_budget_groups` (1024 rows)."""
    offsets, rewards = dynamic_budget_groups(device, seed)
    rows = int(offsets[-1].item())
    g = _gen(seed, device)
    logits = _normal_rows(rows, V, 3.0, torch.bfloat16, g, device)
    _boost_random_columns(logits, min(20, V), 8.0, g)
    tau = (0.6 + 0.8 * torch.rand(rows, generator=g, device=device)).float()
    return Workload("dynamic_budgets", seed, logits, tau, 1.0, None, None, rewards, offsets)


def training_pass(device, seed: int = 3, rows: int = 32_768, V: int = V_QWEN,
                  masked_fraction: float = 0.0) -> Workload:
    """Config 4: `rows` response tokens, bf16 N(0, 3^2) with +6 on one uniformly
    random target column per row, scalar tau = 1; target ids = the boosted column.
    `masked_fraction` > 0 additionally masks out that share of rows (padding tokens)."""
    g = _gen(seed, device)
    logits = _normal_rows(rows, V, 3.0, torch.bfloat16, g, device)
    cols = _boost_random_columns(logits, 1, 6.0, g)
    targets = cols[:, 0].to(torch.int32)
    mask = None
    if masked_fraction > 0.0:
        mask = (torch.rand(rows, generator=g, device=device) >= masked_fraction).to(torch.uint8)
    return Workload("training_pass", seed, logits, None, 1.0, targets, mask)


def large_decode(device, seed: int = 4, rows: int = 4096, V: int = V_QWEN) -> Workload:
    """Config 5: as config 2 but tau alternates {0.3, 2.0} by row parity and 10% of
    the rows (seeded choice) get their two largest logits set to within 1e-3 of each
    other before bf16 rounding (so the stored gap is 0 or one bf16 ulp)."""
    g = _gen(seed, device)
    logits = _normal_rows(rows, V, 3.0, torch.bfloat16, g, device)
    _boost_random_columns(logits, min(20, V), 8.0, g)
    tau = torch.where(torch.arange(rows, device=device) % 2 == 0,
                      torch.tensor(0.3, device=device), torch.tensor(2.0, device=device)).float()
    n_tie = max(1, rows // 10)
    tie_rows = torch.randperm(rows, generator=g, device=device)[:n_tie]
    sub = logits[tie_rows].float()
    top2 = torch.topk(sub, 2, dim=1)
    gap = 1e-3 * torch.rand(n_tie, generator=g, device=device)
    new_second = (top2.values[:, 0] - gap).to(torch.bfloat16)
    sub_b = logits[tie_rows]
    sub_b.scatter_(1, top2.indices[:, 1:2], new_second[:, None])
    logits[tie_rows] = sub_b
    w = Workload("large_decode", seed, logits, tau, 1.0)
    w.notes["tie_rows"] = tie_rows
    return w


def delta_model_rows(device, deltas, V: int = V_QWEN, dtype=torch.float32) -> torch.Tensor:
    """Rows of the Appendix-A two-level model: one logit `delta` above V-1 equal ones.
    The dominant column moves with the row index so that every lane position is hit."""
    rows = len(deltas)
    logits = torch.zeros((rows, V), dtype=dtype, device=device)
    for r, d in enumerate(deltas):
        logits[r, (r * 7919) % V] = float(d)
    return logits


def host_bits(t: torch.Tensor) -> np.ndarray:
    """Host copy of a logit tensor as the array the oracle reads: float32 as is,
    bf16 as its uint16 bit patterns (numpy has no bf16)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.numpy()
    raise TypeError(f"unsupported logit dtype {t.dtype}")
