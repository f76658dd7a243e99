"""Python binding of libe3.so: argument marshalling only.

Every function has the name and the arguments of the C entry point it calls
(include/e3.h).  Tensors are torch tensors used as device memory; the current
torch stream is handed over as the hipStream_t.  Nothing is computed here, and
there is no fallback: without the built library the import of `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libe3.so")

E3_F32, E3_BF16 = 0, 1
E3_OK = 0
E3_TILE_CHUNK, E3_TILE_LANES, E3_TILE_DEPTH = 8, 64, 8
E3_NOALLOC_MAX_ROWS = 1024

EXPORTS = ("e3_strerror", "e3_workspace_bytes", "e3_sample_entropy", "e3_sample_entropy_noalloc",
           "e3_sample_restricted",
           "e3_logprob_entropy", "e3_logprob_entropy_advantages",
           "e3_grpo_advantages", "e3_temperature_update", "e3_difficulty_ranks",
           "e3_allocate_budgets", "e3_budget_bounds", "e3_logprob_entropy_gap",
           "e3_temperature_update_gap", "e3_grpo_objective", "e3_read_probe",
           "e3_time_next_launch")

_lib: Optional[C.CDLL] = None


class E3Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {e3_strerror(status)} (status {status})")


def lib() -> C.CDLL:
    """Load libe3.so (built in-tree by paper_2505_18573_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2505_18573_amd.build` "
                              "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u64, f32, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_double
        L.e3_strerror.argtypes = [C.c_int]
        L.e3_strerror.restype = C.c_char_p
        L.e3_workspace_bytes.argtypes = [i64, i64]
        L.e3_workspace_bytes.restype = C.c_size_t
        L.e3_sample_entropy.argtypes = [vp, C.c_int, i64, i64, i64, vp, f32, u64, u64,
                                        vp, vp, vp, vp, C.c_size_t, vp]
        L.e3_sample_entropy.restype = C.c_int
        L.e3_sample_entropy_noalloc.argtypes = [vp, C.c_int, i64, i64, i64, vp, f32, u64, u64, vp, vp, vp, vp]
        L.e3_sample_entropy_noalloc.restype = C.c_int
        L.e3_sample_restricted.argtypes = [vp, C.c_int, i64, i64, i64, vp, f32, i32, f32, u64, u64,
                                           vp, vp, vp, vp]
        L.e3_sample_restricted.restype = C.c_int
        L.e3_time_next_launch.argtypes = [vp, vp]
        L.e3_time_next_launch.restype = C.c_int
        L.e3_read_probe.argtypes = [vp, i64, vp, vp]
        L.e3_read_probe.restype = C.c_int
        L.e3_logprob_entropy.argtypes = [vp, C.c_int, i64, i64, i64, vp, vp, vp, f32,
                                         vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.e3_logprob_entropy.restype = C.c_int
        L.e3_logprob_entropy_advantages.argtypes = [vp, C.c_int, i64, i64, i64, vp, vp, vp, f32,
                                                    vp, vp, vp, vp, vp, vp, i32, i32, f32, vp,
                                                    vp, C.c_size_t, vp]
        L.e3_logprob_entropy_advantages.restype = C.c_int
        L.e3_logprob_entropy_gap.argtypes = [vp, C.c_int, i64, i64, i64, vp, vp, vp, f32,
                                             vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.e3_logprob_entropy_gap.restype = C.c_int
        L.e3_temperature_update_gap.argtypes = [f64, f64, f64, f64, i64, i64, i64, f64, f64, f64, vp, vp]
        L.e3_temperature_update_gap.restype = C.c_int
        L.e3_grpo_objective.argtypes = [vp, vp, vp, vp, i32, vp, i32, f32, vp, vp, vp, vp]
        L.e3_grpo_objective.restype = C.c_int
        L.e3_grpo_advantages.argtypes = [vp, vp, i32, i32, f32, vp, vp]
        L.e3_grpo_advantages.restype = C.c_int
        L.e3_temperature_update.argtypes = [f64, f64, f64, i64, i64, i64, i64, f64, f64, f64, vp, vp]
        L.e3_temperature_update.restype = C.c_int
        L.e3_difficulty_ranks.argtypes = [vp, vp, i64, vp]
        L.e3_difficulty_ranks.restype = C.c_int
        L.e3_allocate_budgets.argtypes = [vp, i32, i32, i32, i32, vp, vp]
        L.e3_allocate_budgets.restype = C.c_int
        L.e3_budget_bounds.argtypes = [i32, i32, i32, i32, i32, vp, vp]
        L.e3_budget_bounds.restype = C.c_int
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(device) -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def _logits_meta(logits: torch.Tensor) -> Tuple[int, int, int, int]:
    if logits.dim() != 2 or (logits.shape[1] > 1 and logits.stride(1) != 1):
        raise ValueError("logits must be [rows, V] with unit column stride")
    if not logits.is_cuda:
        raise ValueError("logits must live on the GPU")
    if logits.dtype == torch.bfloat16:
        dt = E3_BF16
    elif logits.dtype == torch.float32:
        dt = E3_F32
    else:
        raise TypeError(f"unsupported logit dtype {logits.dtype}")
    rows, V = logits.shape
    stride = logits.stride(0) if rows > 1 else max(V, logits.stride(0))
    return dt, rows, V, stride


def _check(t: Optional[torch.Tensor], dtype, n: int, name: str, device):
    if t is None:
        return
    if t.dtype != dtype or t.dim() != 1 or t.shape[0] != n or not t.is_contiguous() \
            or t.device != device:
        raise ValueError(f"{name} must be a contiguous {dtype} tensor of {n} elements on {device}")


def _check_scalar_out(t: Optional[torch.Tensor], dtype, name: str, device):
    """A one-element output that one thread stores once: device memory, or pinned host
    memory (which the device addresses through the same pointer)."""
    if t is not None and t.device.type == "cpu":
        if not t.is_pinned():
            raise ValueError(f"{name}: a host tensor must be pinned")
        device = t.device
    _check(t, dtype, 1, name, device)


def e3_strerror(status: int) -> str:
    return lib().e3_strerror(int(status)).decode()


def e3_workspace_bytes(rows: int, V: int) -> int:
    return int(lib().e3_workspace_bytes(rows, V))


def new_workspace(rows: int, V: int, device) -> Optional[torch.Tensor]:
    """Allocate a workspace for a [rows, V] problem (None when none is needed)."""
    need = e3_workspace_bytes(rows, V)
    if need == 0:
        return None
    return torch.empty((need + 3) // 4, dtype=torch.int32, device=device)


def _workspace(rows: int, V: int, workspace, device):
    """workspace: a tensor to use, None to allocate one of e3_workspace_bytes(), or False to
    pass NULL (every row then stays in one workgroup)."""
    if workspace is False:
        return None, 0
    if workspace is None:
        workspace = new_workspace(rows, V, device)
    if workspace is None:
        return None, 0
    return workspace, workspace.numel() * workspace.element_size()


def e3_sample_entropy(logits: torch.Tensor, tau_rows: Optional[torch.Tensor], tau_scalar: float,
                      seed: int, row_base: int = 0,
                      token_out: Optional[torch.Tensor] = None,
                      logp_out: Optional[torch.Tensor] = None,
                      entropy_out: Optional[torch.Tensor] = None,
                      workspace=None):
    """Returns (token int32 [rows], logp fp32 [rows], entropy fp32 [rows])."""
    dt, rows, V, stride = _logits_meta(logits)
    dev = logits.device
    if token_out is None:
        token_out = torch.empty(rows, dtype=torch.int32, device=dev)
    if logp_out is None:
        logp_out = torch.empty(rows, dtype=torch.float32, device=dev)
    if entropy_out is None:
        entropy_out = torch.empty(rows, dtype=torch.float32, device=dev)
    _check(tau_rows, torch.float32, rows, "tau_rows", dev)
    _check(token_out, torch.int32, rows, "token_out", dev)
    _check(logp_out, torch.float32, rows, "logp_out", dev)
    _check(entropy_out, torch.float32, rows, "entropy_out", dev)
    ws, ws_bytes = _workspace(rows, V, workspace, dev)
    rc = lib().e3_sample_entropy(_ptr(logits), dt, rows, V, stride, _ptr(tau_rows),
                                 float(tau_scalar), int(seed), int(row_base),
                                 _ptr(token_out), _ptr(logp_out), _ptr(entropy_out),
                                 _ptr(ws), ws_bytes, _stream(dev))
    if rc != E3_OK:
        raise E3Error(rc, "e3_sample_entropy")
    return token_out, logp_out, entropy_out


def e3_sample_entropy_noalloc(logits: torch.Tensor, tau_rows: Optional[torch.Tensor], tau_scalar: float,
                              seed: int, row_base: int, token_out: torch.Tensor,
                              logp_out: Optional[torch.Tensor], entropy_out: Optional[torch.Tensor]):
    """The allocation-free entry point: the caller passes every output (nothing is allocated
    here either).  Returns (token_out, logp_out, entropy_out)."""
    dt, rows, V, stride = _logits_meta(logits)
    dev = logits.device
    _check(tau_rows, torch.float32, rows, "tau_rows", dev)
    _check(token_out, torch.int32, rows, "token_out", dev)
    _check(logp_out, torch.float32, rows, "logp_out", dev)
    _check(entropy_out, torch.float32, rows, "entropy_out", dev)
    rc = lib().e3_sample_entropy_noalloc(_ptr(logits), dt, rows, V, stride, _ptr(tau_rows),
                                         float(tau_scalar), int(seed), int(row_base),
                                         _ptr(token_out), _ptr(logp_out), _ptr(entropy_out), _stream(dev))
    if rc != E3_OK:
        raise E3Error(rc, "e3_sample_entropy_noalloc")
    return token_out, logp_out, entropy_out


def e3_sample_restricted(logits: torch.Tensor, tau_rows: Optional[torch.Tensor], tau_scalar: float,
                         top_k: int, top_p: float, seed: int, row_base: int = 0,
                         token_out: Optional[torch.Tensor] = None,
                         logp_out: Optional[torch.Tensor] = None,
                         kept_out: Optional[torch.Tensor] = None):
    """Returns (token int32 [rows], logp fp32 [rows], kept int32 [rows]).  bf16 rows: any
    top_k / top_p; fp32 rows: 1 <= top_k <= 256 (E3_ERR_VALUE otherwise)."""
    dt, rows, V, stride = _logits_meta(logits)
    dev = logits.device
    if token_out is None:
        token_out = torch.empty(rows, dtype=torch.int32, device=dev)
    if logp_out is None:
        logp_out = torch.empty(rows, dtype=torch.float32, device=dev)
    if kept_out is None:
        kept_out = torch.empty(rows, dtype=torch.int32, device=dev)
    _check(tau_rows, torch.float32, rows, "tau_rows", dev)
    _check(token_out, torch.int32, rows, "token_out", dev)
    _check(logp_out, torch.float32, rows, "logp_out", dev)
    _check(kept_out, torch.int32, rows, "kept_out", dev)
    rc = lib().e3_sample_restricted(_ptr(logits), dt, rows, V, stride, _ptr(tau_rows),
                                    float(tau_scalar), int(top_k), float(top_p), int(seed),
                                    int(row_base), _ptr(token_out), _ptr(logp_out), _ptr(kept_out),
                                    _stream(dev))
    if rc != E3_OK:
        raise E3Error(rc, "e3_sample_restricted")
    return token_out, logp_out, kept_out


E3_READ_PROBE_SUMS = 2048


def e3_time_next_launch(start_event: Optional[int], stop_event: Optional[int]) -> None:
    """start_event / stop_event: hipEvent_t handles as integers (or None)."""
    lib().e3_time_next_launch(C.c_void_p(start_event), C.c_void_p(stop_event))


def e3_read_probe(buf: torch.Tensor, sums_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Reads the (contiguous) tensor once; returns the E3_READ_PROBE_SUMS xor checksums (int32)."""
    if not buf.is_cuda or not buf.is_contiguous():
        raise ValueError("buf must be a contiguous GPU tensor")
    dev = buf.device
    if sums_out is None:
        sums_out = torch.empty(E3_READ_PROBE_SUMS, dtype=torch.int32, device=dev)
    _check(sums_out, torch.int32, E3_READ_PROBE_SUMS, "sums_out", dev)
    rc = lib().e3_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sums_out), _stream(dev))
    if rc != E3_OK:
        raise E3Error(rc, "e3_read_probe")
    return sums_out


def e3_logprob_entropy(logits: torch.Tensor, target_ids: Optional[torch.Tensor],
                       row_mask: Optional[torch.Tensor], tau_rows: Optional[torch.Tensor],
                       tau_scalar: float,
                       logp_out: Optional[torch.Tensor] = None,
                       entropy_out: Optional[torch.Tensor] = None,
                       entropy_sum_out: Optional[torch.Tensor] = None,
                       entropy_count_out: Optional[torch.Tensor] = None,
                       workspace=None, want_sum: bool = True):
    """Returns (logp fp32 [rows] or None, entropy fp32 [rows], entropy_sum fp64 [1] or None,
    entropy_count int64 [1] or None); the sum and count stay on the device unless pinned host
    tensors are passed for them."""
    dt, rows, V, stride = _logits_meta(logits)
    dev = logits.device
    if logp_out is None and target_ids is not None:
        logp_out = torch.empty(rows, dtype=torch.float32, device=dev)
    if entropy_out is None:
        entropy_out = torch.empty(rows, dtype=torch.float32, device=dev)
    if want_sum and entropy_sum_out is None:
        entropy_sum_out = torch.empty(1, dtype=torch.float64, device=dev)
    if want_sum and entropy_count_out is None:
        entropy_count_out = torch.empty(1, dtype=torch.int64, device=dev)
    _check(target_ids, torch.int32, rows, "target_ids", dev)
    _check(row_mask, torch.uint8, rows, "row_mask", dev)
    _check(tau_rows, torch.float32, rows, "tau_rows", dev)
    _check(logp_out, torch.float32, rows, "logp_out", dev)
    _check(entropy_out, torch.float32, rows, "entropy_out", dev)
    _check_scalar_out(entropy_sum_out, torch.float64, "entropy_sum_out", dev)
    _check_scalar_out(entropy_count_out, torch.int64, "entropy_count_out", dev)
    ws, ws_bytes = _workspace(rows, V, workspace, dev)
    rc = lib().e3_logprob_entropy(_ptr(logits), dt, rows, V, stride, _ptr(target_ids),
                                  _ptr(row_mask), _ptr(tau_rows), float(tau_scalar),
                                  _ptr(logp_out), _ptr(entropy_out),
                                  _ptr(entropy_sum_out), _ptr(entropy_count_out),
                                  _ptr(ws), ws_bytes, _stream(dev))
    if rc != E3_OK:
        raise E3Error(rc, "e3_logprob_entropy")
    return logp_out, entropy_out, entropy_sum_out, entropy_count_out


def e3_logprob_entropy_advantages(logits: torch.Tensor, target_ids: Optional[torch.Tensor],
                                  row_mask: Optional[torch.Tensor], tau_rows: Optional[torch.Tensor],
                                  tau_scalar: float, rewards: torch.Tensor, group_offsets: torch.Tensor,
                                  ddof: int = 0, eps: float = 0.0,
                                  logp_out: Optional[torch.Tensor] = None,
                                  entropy_out: Optional[torch.Tensor] = None,
                                  entropy_sum_out: Optional[torch.Tensor] = None,
                                  entropy_count_out: Optional[torch.Tensor] = None,
                                  adv_out: Optional[torch.Tensor] = None,
                                  workspace=None, want_sum: bool = True):
    """e3_logprob_entropy and e3_grpo_advantages in one call.  Returns (logp, entropy,
    entropy_sum, entropy_count, adv)."""
    dt, rows, V, stride = _logits_meta(logits)
    dev = logits.device
    n = rewards.shape[0]
    num_groups = group_offsets.shape[0] - 1
    if logp_out is None and target_ids is not None:
        logp_out = torch.empty(rows, dtype=torch.float32, device=dev)
    if entropy_out is None:
        entropy_out = torch.empty(rows, dtype=torch.float32, device=dev)
    if want_sum and entropy_sum_out is None:
        entropy_sum_out = torch.empty(1, dtype=torch.float64, device=dev)
    if want_sum and entropy_count_out is None:
        entropy_count_out = torch.empty(1, dtype=torch.int64, device=dev)
    if adv_out is None:
        adv_out = torch.empty(n, dtype=torch.float32, device=dev)
    _check(target_ids, torch.int32, rows, "target_ids", dev)
    _check(row_mask, torch.uint8, rows, "row_mask", dev)
    _check(tau_rows, torch.float32, rows, "tau_rows", dev)
    _check(logp_out, torch.float32, rows, "logp_out", dev)
    _check(entropy_out, torch.float32, rows, "entropy_out", dev)
    _check_scalar_out(entropy_sum_out, torch.float64, "entropy_sum_out", dev)
    _check_scalar_out(entropy_count_out, torch.int64, "entropy_count_out", dev)
    _check(rewards, torch.float32, n, "rewards", dev)
    _check(group_offsets, torch.int32, num_groups + 1, "group_offsets", dev)
    _check(adv_out, torch.float32, n, "adv_out", dev)
    ws, ws_bytes = _workspace(rows, V, workspace, dev)
    rc = lib().e3_logprob_entropy_advantages(_ptr(logits), dt, rows, V, stride, _ptr(target_ids),
                                             _ptr(row_mask), _ptr(tau_rows), float(tau_scalar),
                                             _ptr(logp_out), _ptr(entropy_out),
                                             _ptr(entropy_sum_out), _ptr(entropy_count_out),
                                             _ptr(rewards), _ptr(group_offsets), num_groups, int(ddof),
                                             float(eps), _ptr(adv_out), _ptr(ws), ws_bytes, _stream(dev))
    if rc != E3_OK:
        raise E3Error(rc, "e3_logprob_entropy_advantages")
    return logp_out, entropy_out, entropy_sum_out, entropy_count_out, adv_out


def e3_grpo_advantages(rewards: torch.Tensor, group_offsets: torch.Tensor, ddof: int = 0,
                       eps: float = 0.0, adv_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Returns adv fp32 [N].  group_offsets is int32 [B+1] on the same device."""
    dev = rewards.device
    if not rewards.is_cuda:
        raise ValueError("rewards must live on the GPU")
    n = rewards.shape[0]
    num_groups = group_offsets.shape[0] - 1
    _check(rewards, torch.float32, n, "rewards", dev)
    _check(group_offsets, torch.int32, num_groups + 1, "group_offsets", dev)
    if adv_out is None:
        adv_out = torch.empty(n, dtype=torch.float32, device=dev)
    _check(adv_out, torch.float32, n, "adv_out", dev)
    rc = lib().e3_grpo_advantages(_ptr(rewards), _ptr(group_offsets), num_groups, int(ddof),
                                  float(eps), _ptr(adv_out), _stream(dev))
    if rc != E3_OK:
        raise E3Error(rc, "e3_grpo_advantages")
    return adv_out


def e3_temperature_update(tau_t: float, H_t: float, H_init: float, vocab: int, t: int = 0,
                          t_anneal: int = -1, t_max: int = 0, eta: float = 1.0,
                          tau_min: float = 0.0, tau_max: float = float("inf")):
    """Host-only scheduler step.  Returns (tau_next, H_target)."""
    nxt, tgt = C.c_double(float("nan")), C.c_double(float("nan"))
    rc = lib().e3_temperature_update(float(tau_t), float(H_t), float(H_init), int(vocab), int(t),
                                     int(t_anneal), int(t_max), float(eta), float(tau_min),
                                     float(tau_max), C.addressof(nxt), C.addressof(tgt))
    if rc != E3_OK:
        raise E3Error(rc, "e3_temperature_update")
    return nxt.value, tgt.value


def e3_difficulty_ranks(cum_reward, cum_rollouts):
    """Host-only.  Returns k (numpy float64 [num_questions])."""
    import numpy as np
    r = np.ascontiguousarray(cum_reward, dtype=np.float64)
    n = np.ascontiguousarray(cum_rollouts, dtype=np.int64)
    if r.shape != n.shape or r.ndim != 1:
        raise ValueError("cum_reward and cum_rollouts must be 1-D and of equal length")
    k = np.empty(r.shape[0], dtype=np.float64)
    rc = lib().e3_difficulty_ranks(r.ctypes.data, n.ctypes.data, r.shape[0], k.ctypes.data)
    if rc != E3_OK:
        raise E3Error(rc, "e3_difficulty_ranks")
    return k


def e3_allocate_budgets(k, G: int, G_min: int, G_max: int):
    """Host-only.  Returns (G_i int32 [B], offsets int32 [B+1]) as numpy arrays."""
    import numpy as np
    k = np.ascontiguousarray(k, dtype=np.float64)
    B = k.shape[0]
    g = np.empty(B, dtype=np.int32)
    off = np.empty(B + 1, dtype=np.int32)
    rc = lib().e3_allocate_budgets(k.ctypes.data, B, int(G), int(G_min), int(G_max),
                                   g.ctypes.data, off.ctypes.data)
    if rc != E3_OK:
        raise E3Error(rc, "e3_allocate_budgets")
    return g, off


def e3_budget_bounds(G: int, passes_done: int, step: int, G_min_limit: int, G_max_limit: int):
    """Host-only.  Returns (G_min, G_max)."""
    lo, hi = C.c_int32(-1), C.c_int32(-1)
    rc = lib().e3_budget_bounds(int(G), int(passes_done), int(step), int(G_min_limit),
                                int(G_max_limit), C.addressof(lo), C.addressof(hi))
    if rc != E3_OK:
        raise E3Error(rc, "e3_budget_bounds")
    return lo.value, hi.value


def e3_logprob_entropy_gap(logits: torch.Tensor, target_ids: Optional[torch.Tensor],
                           row_mask: Optional[torch.Tensor], tau_rows: Optional[torch.Tensor],
                           tau_scalar: float, workspace=None):
    """Returns (logp or None, entropy, gap, entropy_sum fp64 [1], gap_sum fp64 [1], count int64 [1]),
    all on the device."""
    dt, rows, V, stride = _logits_meta(logits)
    dev = logits.device
    logp = torch.empty(rows, dtype=torch.float32, device=dev) if target_ids is not None else None
    ent = torch.empty(rows, dtype=torch.float32, device=dev)
    gap = torch.empty(rows, dtype=torch.float32, device=dev)
    hs = torch.empty(1, dtype=torch.float64, device=dev)
    gs = torch.empty(1, dtype=torch.float64, device=dev)
    cnt = torch.empty(1, dtype=torch.int64, device=dev)
    _check(target_ids, torch.int32, rows, "target_ids", dev)
    _check(row_mask, torch.uint8, rows, "row_mask", dev)
    _check(tau_rows, torch.float32, rows, "tau_rows", dev)
    ws, ws_bytes = _workspace(rows, V, workspace, dev)
    rc = lib().e3_logprob_entropy_gap(_ptr(logits), dt, rows, V, stride, _ptr(target_ids),
                                      _ptr(row_mask), _ptr(tau_rows), float(tau_scalar),
                                      _ptr(logp), _ptr(ent), _ptr(gap), _ptr(hs), _ptr(gs), _ptr(cnt),
                                      _ptr(ws), ws_bytes, _stream(dev))
    if rc != E3_OK:
        raise E3Error(rc, "e3_logprob_entropy_gap")
    return logp, ent, gap, hs, gs, cnt


def e3_temperature_update_gap(tau_t: float, H_t: float, H_init: float, gap: float, t: int = 0,
                              t_anneal: int = -1, t_max: int = 0, eta: float = 1.0,
                              tau_min: float = 0.0, tau_max: float = float("inf")):
    """Host-only scheduler step with a measured gap.  Returns (tau_next, H_target)."""
    nxt, tgt = C.c_double(float("nan")), C.c_double(float("nan"))
    rc = lib().e3_temperature_update_gap(float(tau_t), float(H_t), float(H_init), float(gap), int(t),
                                         int(t_anneal), int(t_max), float(eta), float(tau_min),
                                         float(tau_max), C.addressof(nxt), C.addressof(tgt))
    if rc != E3_OK:
        raise E3Error(rc, "e3_temperature_update_gap")
    return nxt.value, tgt.value


def e3_grpo_objective(logp_new: torch.Tensor, logp_old: torch.Tensor, seq_offsets: torch.Tensor,
                      adv: torch.Tensor, group_offsets: torch.Tensor, clip_eps: float,
                      want_token_terms: bool = False):
    """Returns (objective fp64 [1], seq_mean fp64 [N], token_terms fp32 [T] or None), on the device."""
    dev = logp_new.device
    if not logp_new.is_cuda:
        raise ValueError("logp_new must live on the GPU")
    T = logp_new.shape[0]
    N = adv.shape[0]
    B = group_offsets.shape[0] - 1
    _check(logp_new, torch.float32, T, "logp_new", dev)
    _check(logp_old, torch.float32, T, "logp_old", dev)
    _check(seq_offsets, torch.int32, N + 1, "seq_offsets", dev)
    _check(adv, torch.float32, N, "adv", dev)
    _check(group_offsets, torch.int32, B + 1, "group_offsets", dev)
    terms = torch.empty(T, dtype=torch.float32, device=dev) if want_token_terms else None
    seq_mean = torch.empty(N, dtype=torch.float64, device=dev)
    J = torch.empty(1, dtype=torch.float64, device=dev)
    rc = lib().e3_grpo_objective(_ptr(logp_new), _ptr(logp_old), _ptr(seq_offsets), _ptr(adv), N,
                                 _ptr(group_offsets), B, float(clip_eps), _ptr(terms),
                                 _ptr(seq_mean), _ptr(J), _stream(dev))
    if rc != E3_OK:
        raise E3Error(rc, "e3_grpo_objective")
    return J, seq_mean, terms
