"""ctypes front end of the C oracle (test infrastructure only).

Marshals numpy arrays into e3_oracle.c; no arithmetic of the method lives here.
Logits are passed as float32 arrays or as uint16 arrays of bf16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import build as _build

F32, BF16 = 0, 1

_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        path = _build.build()
        _lib = C.CDLL(path)
        _declare(_lib)
    return _lib


def _declare(L):
    vp, i32, i64, u32, u64, f32, f64 = (C.c_void_p, C.c_int32, C.c_int64, C.c_uint32,
                                        C.c_uint64, C.c_float, C.c_double)
    L.e3o_philox4x32_10.argtypes = [vp, vp, vp]
    L.e3o_philox4x32_10.restype = None
    L.e3o_noise_word.argtypes = [u64, u64, u32, u32]
    L.e3o_noise_word.restype = u32
    L.e3o_uniform.argtypes = [u32]
    L.e3o_uniform.restype = f64
    L.e3o_gumbel.argtypes = [u32]
    L.e3o_gumbel.restype = f64
    L.e3o_num_tiles.argtypes = [i64] * 4
    L.e3o_num_tiles.restype = i64
    L.e3o_tile_of.argtypes = [i64] * 4
    L.e3o_tile_of.restype = i64
    L.e3o_entropy_textbook.argtypes = [vp, C.c_int, i64, f64]
    L.e3o_entropy_textbook.restype = f64
    L.e3o_log_softmax_row.argtypes = [vp, C.c_int, i64, f64, vp]
    L.e3o_log_softmax_row.restype = None
    L.e3o_sample_entropy.argtypes = [vp, C.c_int, i64, i64, i64, vp, f32, u64, u64,
                                     i64, i64, i64, vp, vp, vp, vp, vp, C.c_int]
    L.e3o_sample_entropy.restype = C.c_int
    L.e3o_logprob_entropy.argtypes = [vp, C.c_int, i64, i64, i64, vp, vp, vp, f32,
                                      vp, vp, vp, vp, C.c_int]
    L.e3o_logprob_entropy.restype = C.c_int
    L.e3o_grpo_advantages.argtypes = [vp, vp, i32, i32, f64, vp]
    L.e3o_grpo_advantages.restype = C.c_int
    L.e3o_entropy_target.argtypes = [f64, i64, i64, i64, f64]
    L.e3o_entropy_target.restype = f64
    L.e3o_temperature_update.argtypes = [f64, f64, f64, i64, i64, i64, i64, f64, f64, f64, vp, vp]
    L.e3o_temperature_update.restype = C.c_int
    L.e3o_difficulty_ranks.argtypes = [vp, vp, i64, vp]
    L.e3o_difficulty_ranks.restype = C.c_int
    L.e3o_allocate_budgets.argtypes = [vp, i32, i32, i32, i32, vp]
    L.e3o_allocate_budgets.restype = C.c_int
    L.e3o_budget_bounds.argtypes = [i32, i32, i32, i32, i32, vp, vp]
    L.e3o_budget_bounds.restype = C.c_int
    L.e3o_logit_gaps.argtypes = [vp, C.c_int, i64, i64, i64, vp, f32, vp]
    L.e3o_logit_gaps.restype = C.c_int
    L.e3o_temperature_update_gap.argtypes = [f64, f64, f64, f64, i64, i64, i64, f64, f64, f64, vp, vp]
    L.e3o_temperature_update_gap.restype = C.c_int
    L.e3o_grpo_objective.argtypes = [vp, vp, vp, vp, vp, i32, f64, vp, vp, vp]
    L.e3o_grpo_objective.restype = C.c_int
    L.e3o_sample_restricted.argtypes = [vp, C.c_int, i64, i64, i64, vp, f32, i32, f64, u64, u64,
                                        vp, vp, vp, vp, vp, C.c_int]
    L.e3o_sample_restricted.restype = C.c_int
    L.e3o_max_threads.argtypes = []
    L.e3o_max_threads.restype = C.c_int


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _logits(a: np.ndarray):
    if a.dtype == np.float32:
        dt = F32
    elif a.dtype == np.uint16:
        dt = BF16
    else:
        raise TypeError("logits must be float32 or uint16 (bf16 bit patterns)")
    if a.ndim != 2 or a.strides[1] != a.itemsize or a.strides[0] % a.itemsize:
        raise ValueError("logits must be 2-D with unit column stride")
    return dt, a.shape[0], a.shape[1], a.strides[0] // a.itemsize


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().e3o_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def noise_word(seed: int, row: int, stream: int, index: int) -> int:
    return int(lib().e3o_noise_word(seed, row, stream, index))


def uniform(word: int) -> float:
    return float(lib().e3o_uniform(word))


def gumbel(word: int) -> float:
    return float(lib().e3o_gumbel(word))


def num_tiles(V: int, partition) -> int:
    return int(lib().e3o_num_tiles(V, *partition))


def tile_of(col: int, partition) -> int:
    return int(lib().e3o_tile_of(col, *partition))


def _tau32(tau: float) -> float:
    """Temperatures cross the library boundary as fp32; round the same way here."""
    return float(np.float32(tau))


def entropy_textbook(row: np.ndarray, tau: float) -> float:
    dt, _, V, _ = _logits(row.reshape(1, -1))
    return float(lib().e3o_entropy_textbook(_ptr(row), dt, V, _tau32(tau)))


def log_softmax_row(row: np.ndarray, tau: float) -> np.ndarray:
    dt, _, V, _ = _logits(row.reshape(1, -1))
    out = np.empty(V, dtype=np.float64)
    lib().e3o_log_softmax_row(_ptr(row), dt, V, _tau32(tau), _ptr(out))
    return out


@dataclass
class SampleResult:
    token: np.ndarray      # int32 [rows]
    logp: np.ndarray       # float64 [rows]
    entropy: np.ndarray    # float64 [rows]
    near_tie: np.ndarray   # uint8 [rows]
    diag: np.ndarray       # float64 [rows, 4]: top-two tile scores, top-two column scores


def sample_entropy(logits: np.ndarray, tau_rows: Optional[np.ndarray], tau_scalar: float,
                   seed: int, row_base: int = 0, *, partition,
                   nthreads: int = 1) -> SampleResult:
    """partition = (chunk, lanes, depth) of the sampler's column tiles: columns are cut into
    chunks, chunks dealt round-robin to `lanes` slots, a tile is `depth` successive chunks of
    one slot.  It is part of the definition of the token and has no default here: a caller
    states which sampler it means ((V, 1, 1) and (1, 1, 1) are the flat Gumbel-max)."""
    dt, rows, V, stride = _logits(logits)
    if tau_rows is not None:
        tau_rows = np.ascontiguousarray(tau_rows, dtype=np.float32)
        assert tau_rows.shape == (rows,)
    tok = np.empty(rows, dtype=np.int32)
    logp = np.empty(rows, dtype=np.float64)
    ent = np.empty(rows, dtype=np.float64)
    tie = np.zeros(rows, dtype=np.uint8)
    diag = np.empty((rows, 4), dtype=np.float64)
    rc = lib().e3o_sample_entropy(_ptr(logits), dt, rows, V, stride, _ptr(tau_rows),
                                  tau_scalar, seed, row_base, *partition,
                                  _ptr(tok), _ptr(logp), _ptr(ent), _ptr(tie), _ptr(diag),
                                  nthreads)
    if rc != 0:
        raise RuntimeError(f"e3o_sample_entropy failed: {rc}")
    return SampleResult(tok, logp, ent, tie, diag)


@dataclass
class RestrictedResult:
    token: np.ndarray      # int32 [rows]
    logp: np.ndarray       # float64 [rows], under the truncated and renormalised distribution
    kept: np.ndarray       # int32 [rows], columns that survive the truncation
    near_tie: np.ndarray   # uint8 [rows]
    near_cut: np.ndarray   # uint8 [rows]


def sample_restricted(logits: np.ndarray, tau_rows: Optional[np.ndarray], tau_scalar: float,
                      top_k: int, top_p: float, seed: int, row_base: int = 0,
                      nthreads: int = 1) -> RestrictedResult:
    """top_p crosses the library boundary as fp32 and is rounded the same way here."""
    dt, rows, V, stride = _logits(logits)
    if tau_rows is not None:
        tau_rows = np.ascontiguousarray(tau_rows, dtype=np.float32)
        assert tau_rows.shape == (rows,)
    tok = np.empty(rows, dtype=np.int32)
    logp = np.empty(rows, dtype=np.float64)
    kept = np.empty(rows, dtype=np.int32)
    tie = np.zeros(rows, dtype=np.uint8)
    cut = np.zeros(rows, dtype=np.uint8)
    rc = lib().e3o_sample_restricted(_ptr(logits), dt, rows, V, stride, _ptr(tau_rows), tau_scalar,
                                     int(top_k), float(np.float32(top_p)), seed, row_base,
                                     _ptr(tok), _ptr(logp), _ptr(kept), _ptr(tie), _ptr(cut), nthreads)
    if rc != 0:
        raise RuntimeError(f"e3o_sample_restricted failed: {rc}")
    return RestrictedResult(tok, logp, kept, tie, cut)


@dataclass
class LogprobResult:
    logp: np.ndarray          # float64 [rows]
    entropy: np.ndarray       # float64 [rows]
    entropy_sum: float
    entropy_count: int

    @property
    def entropy_mean(self) -> float:
        return self.entropy_sum / self.entropy_count


def logprob_entropy(logits: np.ndarray, target_ids: Optional[np.ndarray],
                    row_mask: Optional[np.ndarray], tau_rows: Optional[np.ndarray],
                    tau_scalar: float, nthreads: int = 1) -> LogprobResult:
    dt, rows, V, stride = _logits(logits)
    if target_ids is not None:
        target_ids = np.ascontiguousarray(target_ids, dtype=np.int32)
    if row_mask is not None:
        row_mask = np.ascontiguousarray(row_mask, dtype=np.uint8)
    if tau_rows is not None:
        tau_rows = np.ascontiguousarray(tau_rows, dtype=np.float32)
    logp = np.empty(rows, dtype=np.float64)
    ent = np.empty(rows, dtype=np.float64)
    s = C.c_double(0.0)
    n = C.c_int64(0)
    rc = lib().e3o_logprob_entropy(_ptr(logits), dt, rows, V, stride, _ptr(target_ids),
                                   _ptr(row_mask), _ptr(tau_rows), tau_scalar,
                                   _ptr(logp), _ptr(ent), C.addressof(s), C.addressof(n),
                                   nthreads)
    if rc != 0:
        raise RuntimeError(f"e3o_logprob_entropy failed: {rc}")
    return LogprobResult(logp, ent, s.value, n.value)


def grpo_advantages(rewards: np.ndarray, group_offsets: np.ndarray, ddof: int = 0,
                    eps: float = 0.0) -> np.ndarray:
    rewards = np.ascontiguousarray(rewards, dtype=np.float32)
    group_offsets = np.ascontiguousarray(group_offsets, dtype=np.int32)
    out = np.full(rewards.shape[0], np.nan, dtype=np.float64)
    rc = lib().e3o_grpo_advantages(_ptr(rewards), _ptr(group_offsets),
                                   group_offsets.shape[0] - 1, ddof, eps, _ptr(out))
    if rc != 0:
        raise RuntimeError(f"e3o_grpo_advantages failed: {rc}")
    return out


def entropy_target(H_init: float, t: int, t_anneal: int, t_max: int, eta: float) -> float:
    return float(lib().e3o_entropy_target(H_init, t, t_anneal, t_max, eta))


def temperature_update(tau_t: float, H_t: float, H_init: float, vocab: int, t: int = 0,
                       t_anneal: int = -1, t_max: int = 0, eta: float = 1.0,
                       tau_min: float = 0.0, tau_max: float = float("inf")):
    """Returns (status, tau_next, H_target)."""
    nxt = C.c_double(float("nan"))
    tgt = C.c_double(float("nan"))
    rc = lib().e3o_temperature_update(tau_t, H_t, H_init, vocab, t, t_anneal, t_max, eta,
                                      tau_min, tau_max, C.addressof(nxt), C.addressof(tgt))
    return rc, nxt.value, tgt.value


def difficulty_ranks(cum_reward, cum_rollouts):
    """Returns (status, k float64 [n])."""
    r = np.ascontiguousarray(cum_reward, dtype=np.float64)
    n = np.ascontiguousarray(cum_rollouts, dtype=np.int64)
    k = np.full(r.shape[0], np.nan)
    rc = lib().e3o_difficulty_ranks(_ptr(r), _ptr(n), r.shape[0], _ptr(k))
    return rc, k


def allocate_budgets(k, G: int, G_min: int, G_max: int):
    """Returns (status, G_i int32 [B])."""
    k = np.ascontiguousarray(k, dtype=np.float64)
    out = np.full(k.shape[0], -1, dtype=np.int32)
    rc = lib().e3o_allocate_budgets(_ptr(k), k.shape[0], G, G_min, G_max, _ptr(out))
    return rc, out


def budget_bounds(G: int, passes_done: int, step: int, G_min_limit: int, G_max_limit: int):
    """Returns (status, G_min, G_max)."""
    lo, hi = C.c_int32(-1), C.c_int32(-1)
    rc = lib().e3o_budget_bounds(G, passes_done, step, G_min_limit, G_max_limit,
                                 C.addressof(lo), C.addressof(hi))
    return rc, lo.value, hi.value


def logit_gaps(logits: np.ndarray, tau_rows: Optional[np.ndarray], tau_scalar: float) -> np.ndarray:
    dt, rows, V, stride = _logits(logits)
    if tau_rows is not None:
        tau_rows = np.ascontiguousarray(tau_rows, dtype=np.float32)
    out = np.empty(rows, dtype=np.float64)
    rc = lib().e3o_logit_gaps(_ptr(logits), dt, rows, V, stride, _ptr(tau_rows), tau_scalar, _ptr(out))
    if rc != 0:
        raise RuntimeError(f"e3o_logit_gaps failed: {rc}")
    return out


def temperature_update_gap(tau_t: float, H_t: float, H_init: float, delta: float, t: int = 0,
                           t_anneal: int = -1, t_max: int = 0, eta: float = 1.0,
                           tau_min: float = 0.0, tau_max: float = float("inf")):
    """Returns (status, tau_next, H_target)."""
    nxt = C.c_double(float("nan"))
    tgt = C.c_double(float("nan"))
    rc = lib().e3o_temperature_update_gap(tau_t, H_t, H_init, delta, t, t_anneal, t_max, eta,
                                          tau_min, tau_max, C.addressof(nxt), C.addressof(tgt))
    return rc, nxt.value, tgt.value


def grpo_objective(logp_new, logp_old, seq_offsets, adv, group_offsets, clip_eps: float):
    """Returns (J, token_terms float64 [T], seq_means float64 [N])."""
    ln = np.ascontiguousarray(logp_new, dtype=np.float32)
    lo = np.ascontiguousarray(logp_old, dtype=np.float32)
    so = np.ascontiguousarray(seq_offsets, dtype=np.int32)
    ad = np.ascontiguousarray(adv, dtype=np.float32)
    go = np.ascontiguousarray(group_offsets, dtype=np.int32)
    terms = np.full(ln.shape[0], np.nan)
    means = np.full(ad.shape[0], np.nan)
    J = C.c_double(float("nan"))
    rc = lib().e3o_grpo_objective(_ptr(ln), _ptr(lo), _ptr(so), _ptr(ad), _ptr(go), go.shape[0] - 1,
                                  clip_eps, _ptr(terms), _ptr(means), C.addressof(J))
    if rc != 0:
        raise RuntimeError(f"e3o_grpo_objective failed: {rc}")
    return J.value, terms, means


def max_threads() -> int:
    return int(lib().e3o_max_threads())
