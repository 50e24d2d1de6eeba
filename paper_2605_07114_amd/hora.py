"""Python binding of the HORA C-ABI library (``include/hora.h``).

Argument marshalling only: every function here passes device pointers of torch
tensors, sizes and the current HIP stream to the entry point of the same name
in ``libhora.so``; all arithmetic runs in the library's kernels.  There is no
CPU fallback: a missing library raises.

``Session`` is a convenience holder for the buffers a caller keeps alive across
calls (workspace, device status word) and allocates outputs with torch.
"""
from __future__ import annotations

import ctypes
import os
import threading
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhora.so")

OK = 0
ERR_INVALID_ARG, ERR_INFEASIBLE, ERR_WORKSPACE, ERR_RANGE = -1, -2, -3, -4
ERR_HIP, ERR_UNSUPPORTED = -5, -6
MAX_DEPTH = 1 << 20
ADV_GRPO, ADV_RLOO, ADV_CENTER = 0, 1, 2
F32, F64 = 0, 1
I32, I64 = 0, 1
ALLOC_AUTO, ALLOC_CLASS, ALLOC_BISECT = 0, 1, 2
RULE_UNIFORM, RULE_HARD_FIRST = 0, 1
CLASS_MAX_G0 = 63

EXPORTS = (
    "hora_status_string", "hora_version", "hora_marginal_gains", "hora_allocate_workspace_bytes",
    "hora_allocate", "hora_allocate_posterior", "hora_group_advantage", "hora_token_broadcast",
    "hora_token_broadcast_workspace_bytes", "hora_allocate_sharded", "hora_allocate_sharded_workspace_bytes",
    "hora_response_weights", "hora_allocate_baseline", "hora_pass_at_k", "hora_pass_at_k_workspace_bytes",
    "hora_allocate_static", "hora_token_broadcast2", "hora_token_broadcast2_workspace_bytes",
    "hora_allocation_shares",
)


class HoraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Loads libhora.so and declares the signatures of include/hora.h."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build it with `python -m paper_2605_07114_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    p, i32, i64, f64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_size_t
    lib.hora_status_string.argtypes = [ctypes.c_int]
    lib.hora_status_string.restype = ctypes.c_char_p
    lib.hora_version.argtypes = []
    lib.hora_version.restype = ctypes.c_int
    lib.hora_marginal_gains.argtypes = [i64, p, p, i32, p, p, p]
    lib.hora_marginal_gains.restype = ctypes.c_int
    lib.hora_allocate_workspace_bytes.argtypes = [i64, i32]
    lib.hora_allocate_workspace_bytes.restype = sz
    lib.hora_allocate.argtypes = [i64, i32, p, f64, f64, i64, i32, i32, p, p, p, i32, p, p, p, sz, p]
    lib.hora_allocate.restype = ctypes.c_int
    lib.hora_allocate_static.argtypes = [i64, i32, p, f64, f64, i64, i32, i32, p, p, p, i32, p, p, p]
    lib.hora_allocate_static.restype = ctypes.c_int
    lib.hora_allocation_shares.argtypes = [i64, i32, p, p, p, p, p, p]
    lib.hora_allocation_shares.restype = ctypes.c_int
    lib.hora_allocate_baseline.argtypes = [i64, i32, p, f64, f64, i64, i32, i32, p, p, p, i32, p, p, p, sz, p]
    lib.hora_allocate_baseline.restype = ctypes.c_int
    lib.hora_allocate_posterior.argtypes = [i64, i32, p, p, i64, i32, p, p, p, i32, p, p, p, sz, p]
    lib.hora_allocate_posterior.restype = ctypes.c_int
    lib.hora_allocate_sharded_workspace_bytes.argtypes = [i64]
    lib.hora_allocate_sharded_workspace_bytes.restype = sz
    lib.hora_allocate_sharded.argtypes = [i64, i32, p, f64, f64, i64, p, p, i32, p, p, p, i32, p, p, p, sz, p]
    lib.hora_allocate_sharded.restype = ctypes.c_int
    lib.hora_group_advantage.argtypes = [i64, p, i32, i64, p, p, i32, i32, f64, i32, p, p]
    lib.hora_group_advantage.restype = ctypes.c_int
    lib.hora_pass_at_k_workspace_bytes.argtypes = [i64, i32]
    lib.hora_pass_at_k_workspace_bytes.restype = sz
    lib.hora_pass_at_k.argtypes = [i64, p, p, i32, p, p, p, p, p, sz, p]
    lib.hora_pass_at_k.restype = ctypes.c_int
    lib.hora_response_weights.argtypes = [i64, p, i32, i64, p, i32, f64, p, i32, p, p]
    lib.hora_response_weights.restype = ctypes.c_int
    lib.hora_token_broadcast_workspace_bytes.argtypes = [i64, i32]
    lib.hora_token_broadcast_workspace_bytes.restype = sz
    lib.hora_token_broadcast.argtypes = [i64, p, i32, p, i32, p, i32, i64, p, p, sz, p]
    lib.hora_token_broadcast.restype = ctypes.c_int
    lib.hora_token_broadcast2_workspace_bytes.argtypes = [i64, i32]
    lib.hora_token_broadcast2_workspace_bytes.restype = sz
    lib.hora_token_broadcast2.argtypes = [i64, p, p, i32, p, i32, p, p, i32, i64, p, p, sz, p]
    lib.hora_token_broadcast2.restype = ctypes.c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().hora_status_string(int(status)).decode()


def version() -> int:
    return int(load_library().hora_version())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


# (torch.cuda.current_stream() builds a Stream object, ~3 us per call; the raw handle is what is passed on)
_raw_current_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream(stream, like: Optional[torch.Tensor] = None) -> Optional[int]:
    """The HIP stream handle to pass on: `stream` (a torch stream), or the current stream of
    the device that `like` lives on."""
    if stream is None:
        if _raw_current_stream is not None and like is not None and like.is_cuda:
            return _raw_current_stream(like.device.index) or None
        stream = torch.cuda.current_stream(like.device if like is not None and like.is_cuda else None)
    return stream.cuda_stream or None


def _ftype(t: torch.Tensor) -> int:
    return {torch.float32: F32, torch.float64: F64}[t.dtype]


def _itype(t: torch.Tensor) -> int:
    return {torch.int32: I32, torch.int64: I64}[t.dtype]


def _check(status: int, where: str) -> None:
    if status != OK:
        raise HoraError(status, where)


_recording = threading.local()


def _call(name: str, *args) -> None:
    """Calls entry point `name` with marshalled arguments (or notes the call down for `prepared`)."""
    f = getattr(load_library(), name)
    notes = getattr(_recording, "notes", None)
    if notes is not None:
        notes.append((f, args, name))
        return
    _check(f(*args), name)


def prepared(binding, *args, **kwargs):
    """Marshals once, calls many times.  Runs `binding` (one of the hora_* functions below that
    launch work) with the given arguments up to, but not including, the call into the library,
    and returns a function without arguments that makes that call each time: the same device
    buffers (the tensors stay referenced by the returned function), sizes and stream.  For
    loops that repeat a small call: the checks and conversions above cost several microseconds,
    more than the kernels of a call on a few dozen prompts."""
    if getattr(_recording, "notes", None) is not None:
        raise RuntimeError("prepared() calls do not nest")
    _recording.notes = []
    try:
        binding(*args, **kwargs)
        notes = _recording.notes
    finally:
        _recording.notes = None
    if len(notes) != 1:
        raise ValueError("prepared() expects a binding that makes exactly one library call")
    f, cargs, name = notes[0]

    def run() -> None:
        status = f(*cargs)
        if status != OK:
            raise HoraError(status, name)

    run.keeps = (args, kwargs)
    return run


def _expect(t: Optional[torch.Tensor], dtype, numel: int, name: str) -> None:
    if t is None:
        return
    if t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if t.numel() < numel:
        raise ValueError(f"{name}: {t.numel()} elements, expected at least {numel}")


# ----------------------------------------------------------------------------
# Entry points, one per function of include/hora.h
# ----------------------------------------------------------------------------
def hora_allocate_workspace_bytes(n: int, g0: int) -> int:
    return int(load_library().hora_allocate_workspace_bytes(int(n), int(g0)))


def hora_marginal_gains(alpha: torch.Tensor, beta: torch.Tensor, count: int,
                        gains: Optional[torch.Tensor], util: Optional[torch.Tensor], stream=None) -> None:
    n = alpha.numel()
    _expect(alpha, torch.float64, n, "alpha")
    _expect(beta, torch.float64, n, "beta")
    _expect(gains, torch.float64, n * count, "gains")
    _expect(util, torch.float64, n * count, "util")
    _call("hora_marginal_gains", n, _ptr(alpha), _ptr(beta), int(count), _ptr(gains), _ptr(util),
          _stream(stream, alpha))


def hora_allocate(c: torch.Tensor, g0: int, budget: int, delta: torch.Tensor, dev_status: torch.Tensor,
                  workspace: torch.Tensor, *, alpha0: float = 1.0, beta0: float = 1.0, delta_max: int = 0,
                  method: int = ALLOC_AUTO, util: Optional[torch.Tensor] = None,
                  group_off: Optional[torch.Tensor] = None, summary: Optional[torch.Tensor] = None,
                  stream=None) -> None:
    n = c.numel()
    _expect(c, torch.int32, n, "c")
    _expect(delta, torch.int32, n, "delta")
    _expect(util, torch.float64, n, "util")
    _expect(dev_status, torch.int32, 1, "dev_status")
    _expect(summary, torch.int64, 4, "summary")
    if group_off is not None and group_off.numel() < n + 1:
        raise ValueError("group_off needs n + 1 elements")
    _call("hora_allocate", n, int(g0), _ptr(c), float(alpha0), float(beta0), int(budget), int(delta_max), int(method),
          _ptr(delta), _ptr(util), _ptr(group_off), _itype(group_off) if group_off is not None else I32,
          _ptr(summary), _ptr(dev_status), _ptr(workspace), workspace.numel() * workspace.element_size(),
          _stream(stream, c))


def hora_allocate_static(c: torch.Tensor, g0: int, budget: int, delta: torch.Tensor, dev_status: torch.Tensor, *,
                         alpha0: float = 1.0, beta0: float = 1.0, delta_max: int = 0, method: int = ALLOC_AUTO,
                         util: Optional[torch.Tensor] = None, group_off: Optional[torch.Tensor] = None,
                         summary: Optional[torch.Tensor] = None, stream=None) -> None:
    n = c.numel()
    _expect(c, torch.int32, n, "c")
    _expect(delta, torch.int32, n, "delta")
    _expect(util, torch.float64, n, "util")
    _expect(dev_status, torch.int32, 1, "dev_status")
    _expect(summary, torch.int64, 4, "summary")
    if group_off is not None and group_off.numel() < n + 1:
        raise ValueError("group_off needs n + 1 elements")
    _call("hora_allocate_static", n, int(g0), _ptr(c), float(alpha0), float(beta0), int(budget), int(delta_max), int(method),
          _ptr(delta), _ptr(util), _ptr(group_off), _itype(group_off) if group_off is not None else I32,
          _ptr(summary), _ptr(dev_status), _stream(stream, c))


def hora_allocation_shares(c: torch.Tensor, delta: torch.Tensor, g0: int, class_count: torch.Tensor,
                           class_budget: torch.Tensor, dev_status: torch.Tensor, stream=None) -> None:
    n = c.numel()
    _expect(c, torch.int32, n, "c")
    _expect(delta, torch.int32, n, "delta")
    _expect(class_count, torch.int64, g0 + 1, "class_count")
    _expect(class_budget, torch.int64, g0 + 1, "class_budget")
    _expect(dev_status, torch.int32, 1, "dev_status")
    _call("hora_allocation_shares", n, int(g0), _ptr(c), _ptr(delta), _ptr(class_count),
          _ptr(class_budget), _ptr(dev_status), _stream(stream, c))


def hora_allocate_baseline(c: torch.Tensor, g0: int, budget: int, rule: int, delta: torch.Tensor,
                           dev_status: torch.Tensor, workspace: torch.Tensor, *, alpha0: float = 1.0,
                           beta0: float = 1.0, delta_max: int = 0, util: Optional[torch.Tensor] = None,
                           group_off: Optional[torch.Tensor] = None, summary: Optional[torch.Tensor] = None,
                           stream=None) -> None:
    n = c.numel()
    _expect(c, torch.int32, n, "c")
    _expect(delta, torch.int32, n, "delta")
    _expect(util, torch.float64, n, "util")
    _expect(dev_status, torch.int32, 1, "dev_status")
    _expect(summary, torch.int64, 4, "summary")
    if group_off is not None and group_off.numel() < n + 1:
        raise ValueError("group_off needs n + 1 elements")
    _call("hora_allocate_baseline", n, int(g0), _ptr(c), float(alpha0), float(beta0), int(budget), int(delta_max), int(rule),
          _ptr(delta), _ptr(util), _ptr(group_off), _itype(group_off) if group_off is not None else I32,
          _ptr(summary), _ptr(dev_status), _ptr(workspace), workspace.numel() * workspace.element_size(),
          _stream(stream, c))


def hora_allocate_posterior(alpha: torch.Tensor, beta: torch.Tensor, g0: int, budget: int, delta: torch.Tensor,
                            dev_status: torch.Tensor, workspace: torch.Tensor, *, delta_max: int = 0,
                            util: Optional[torch.Tensor] = None, group_off: Optional[torch.Tensor] = None,
                            summary: Optional[torch.Tensor] = None, stream=None) -> None:
    n = alpha.numel()
    _expect(alpha, torch.float64, n, "alpha")
    _expect(beta, torch.float64, n, "beta")
    _expect(delta, torch.int32, n, "delta")
    _expect(util, torch.float64, n, "util")
    _expect(dev_status, torch.int32, 1, "dev_status")
    _expect(summary, torch.int64, 4, "summary")
    if group_off is not None and group_off.numel() < n + 1:
        raise ValueError("group_off needs n + 1 elements")
    _call("hora_allocate_posterior", n, int(g0), _ptr(alpha), _ptr(beta), int(budget), int(delta_max), _ptr(delta), _ptr(util),
          _ptr(group_off), _itype(group_off) if group_off is not None else I32, _ptr(summary),
          _ptr(dev_status), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream, alpha))


def hora_allocate_sharded_workspace_bytes(n_shards: int) -> int:
    return int(load_library().hora_allocate_sharded_workspace_bytes(int(n_shards)))


def hora_allocate_sharded(c: torch.Tensor, g0: int, shard_off: torch.Tensor, shard_budget: torch.Tensor,
                          delta: torch.Tensor, dev_status: torch.Tensor, workspace: Optional[torch.Tensor], *,
                          alpha0: float = 1.0, beta0: float = 1.0, delta_max: int = 0,
                          util: Optional[torch.Tensor] = None, group_off: Optional[torch.Tensor] = None,
                          summary: Optional[torch.Tensor] = None, stream=None) -> None:
    n = c.numel()
    n_shards = shard_budget.numel()
    _expect(c, torch.int32, n, "c")
    _expect(shard_off, torch.int64, n_shards + 1, "shard_off")
    _expect(shard_budget, torch.int64, n_shards, "shard_budget")
    _expect(delta, torch.int32, n, "delta")
    _expect(util, torch.float64, n, "util")
    _expect(dev_status, torch.int32, 1, "dev_status")
    _expect(summary, torch.int64, 4 * n_shards, "summary")
    if group_off is not None and group_off.numel() < n + 1:
        raise ValueError("group_off needs n + 1 elements")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _call("hora_allocate_sharded", n, int(g0), _ptr(c), float(alpha0), float(beta0), n_shards, _ptr(shard_off), _ptr(shard_budget),
          int(delta_max), _ptr(delta), _ptr(util), _ptr(group_off),
          _itype(group_off) if group_off is not None else I32, _ptr(summary), _ptr(dev_status), _ptr(workspace),
          ws_bytes, _stream(stream, c))


def hora_group_advantage(group_off: torch.Tensor, reward: torch.Tensor, adv: torch.Tensor, mode: int,
                         dev_status: torch.Tensor, *, eps: float = 0.0, ddof: int = 0, stream=None) -> None:
    n_groups = group_off.numel() - 1
    n_resp = reward.numel()
    if adv.dtype != reward.dtype or adv.numel() < n_resp:
        raise ValueError("adv must match reward in dtype and size")
    _expect(dev_status, torch.int32, 1, "dev_status")
    _call("hora_group_advantage", n_groups, _ptr(group_off), _itype(group_off), n_resp, _ptr(reward), _ptr(adv), _ftype(reward),
          int(mode), float(eps), int(ddof), _ptr(dev_status), _stream(stream, group_off))


def hora_response_weights(group_off: torch.Tensor, tok_off: torch.Tensor, weight: torch.Tensor,
                          dev_status: torch.Tensor, *, length_const: float = 0.0, stream=None) -> None:
    n_groups = group_off.numel() - 1
    n_resp = tok_off.numel() - 1
    if weight.numel() < n_resp:
        raise ValueError("weight too small")
    _expect(dev_status, torch.int32, 1, "dev_status")
    _call("hora_response_weights", n_groups, _ptr(group_off), _itype(group_off), n_resp, _ptr(tok_off), _itype(tok_off), float(length_const),
          _ptr(weight), _ftype(weight), _ptr(dev_status), _stream(stream, group_off))


def hora_pass_at_k(n_samples: torch.Tensor, correct: torch.Tensor, ks, mean: torch.Tensor,
                   dev_status: torch.Tensor, workspace: torch.Tensor, *, per_problem: Optional[torch.Tensor] = None,
                   stream=None) -> None:
    n = n_samples.numel()
    ks = [int(k) for k in ks]
    _expect(n_samples, torch.int32, n, "n_samples")
    _expect(correct, torch.int32, n, "correct")
    _expect(mean, torch.float64, len(ks), "mean")
    _expect(per_problem, torch.float64, len(ks) * n, "per_problem")
    _expect(dev_status, torch.int32, 1, "dev_status")
    host_ks = (ctypes.c_int32 * max(len(ks), 1))(*ks)
    _call("hora_pass_at_k", n, _ptr(n_samples), _ptr(correct), len(ks), ctypes.cast(host_ks, ctypes.c_void_p), _ptr(per_problem),
          _ptr(mean), _ptr(dev_status), _ptr(workspace), workspace.numel() * workspace.element_size(),
          _stream(stream, n_samples))


def hora_pass_at_k_workspace_bytes(n_problems: int, n_k: int) -> int:
    return int(load_library().hora_pass_at_k_workspace_bytes(int(n_problems), int(n_k)))


def hora_token_broadcast_workspace_bytes(n_tokens: int, out_dtype: torch.dtype = torch.float32) -> int:
    t = {torch.float32: F32, torch.float64: F64}[out_dtype]
    return int(load_library().hora_token_broadcast_workspace_bytes(int(n_tokens), t))


def hora_token_broadcast(adv: torch.Tensor, tok_off: torch.Tensor, tok_adv: torch.Tensor, n_tokens: int,
                         dev_status: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    n_resp = adv.numel()
    if tok_off.numel() != n_resp + 1:
        raise ValueError("tok_off needs n_resp + 1 elements")
    if tok_adv.numel() < n_tokens:
        raise ValueError("tok_adv too small")
    _expect(dev_status, torch.int32, 1, "dev_status")
    _call("hora_token_broadcast", n_resp, _ptr(adv), _ftype(adv), _ptr(tok_off), _itype(tok_off), _ptr(tok_adv), _ftype(tok_adv),
          int(n_tokens), _ptr(dev_status), _ptr(workspace), workspace.numel() * workspace.element_size(),
          _stream(stream, adv))


def hora_token_broadcast2_workspace_bytes(n_tokens: int, out_dtype: torch.dtype = torch.float32) -> int:
    t = {torch.float32: F32, torch.float64: F64}[out_dtype]
    return int(load_library().hora_token_broadcast2_workspace_bytes(int(n_tokens), t))


def hora_token_broadcast2(adv_a: torch.Tensor, adv_b: torch.Tensor, tok_off: torch.Tensor, tok_a: torch.Tensor,
                          tok_b: torch.Tensor, n_tokens: int, dev_status: torch.Tensor, workspace: torch.Tensor,
                          stream=None) -> None:
    n_resp = adv_a.numel()
    if adv_b.numel() != n_resp or adv_b.dtype != adv_a.dtype:
        raise ValueError("adv_b must match adv_a in dtype and size")
    if tok_off.numel() != n_resp + 1:
        raise ValueError("tok_off needs n_resp + 1 elements")
    if tok_a.numel() < n_tokens or tok_b.numel() < n_tokens or tok_a.dtype != tok_b.dtype:
        raise ValueError("tok_a / tok_b too small or of different types")
    _expect(dev_status, torch.int32, 1, "dev_status")
    _call("hora_token_broadcast2", n_resp, _ptr(adv_a), _ptr(adv_b), _ftype(adv_a), _ptr(tok_off), _itype(tok_off), _ptr(tok_a), _ptr(tok_b),
          _ftype(tok_a), int(n_tokens), _ptr(dev_status), _ptr(workspace),
          workspace.numel() * workspace.element_size(), _stream(stream, adv_a))


# ----------------------------------------------------------------------------
# Buffer holder
# ----------------------------------------------------------------------------
@dataclass
class Allocation:
    delta: torch.Tensor
    util: Optional[torch.Tensor]
    group_off: Optional[torch.Tensor]
    summary: Optional[torch.Tensor]   # int64[4]: bits of tau, count_gt, tie_units, tie_prompts


class Session:
    """Owns the workspace and the sticky device status word of one caller."""

    def __init__(self, device: str = "cuda:0"):
        self.device = torch.device(device)
        self.dev_status = torch.zeros(1, dtype=torch.int32, device=self.device)
        self._workspace = torch.zeros(0, dtype=torch.uint8, device=self.device)
        self._bcast_workspace = torch.empty(0, dtype=torch.uint8, device=self.device)
        self._shard_workspace = torch.empty(0, dtype=torch.uint8, device=self.device)

    def workspace(self, n: int, g0: int) -> torch.Tensor:
        need = hora_allocate_workspace_bytes(n, g0)
        if self._workspace.numel() < need:
            self._workspace = torch.zeros(need, dtype=torch.uint8, device=self.device)
        return self._workspace

    def allocate(self, c: torch.Tensor, g0: int, budget: int, *, alpha0: float = 1.0, beta0: float = 1.0,
                 delta_max: int = 0, method: int = ALLOC_AUTO, want_util: bool = True,
                 off_dtype: Optional[torch.dtype] = torch.int64, want_summary: bool = True) -> Allocation:
        n = c.numel()
        out = Allocation(
            delta=torch.empty(n, dtype=torch.int32, device=self.device),
            util=torch.empty(n, dtype=torch.float64, device=self.device) if want_util else None,
            group_off=torch.empty(n + 1, dtype=off_dtype, device=self.device) if off_dtype else None,
            summary=torch.zeros(4, dtype=torch.int64, device=self.device) if want_summary else None)
        hora_allocate(c, g0, budget, out.delta, self.dev_status, self.workspace(n, g0), alpha0=alpha0,
                      beta0=beta0, delta_max=delta_max, method=method, util=out.util, group_off=out.group_off,
                      summary=out.summary)
        return out

    def allocate_baseline(self, c: torch.Tensor, g0: int, budget: int, rule: int, *, delta_max: int = 0,
                          off_dtype: Optional[torch.dtype] = torch.int64) -> Allocation:
        n = c.numel()
        out = Allocation(
            delta=torch.empty(n, dtype=torch.int32, device=self.device),
            util=torch.empty(n, dtype=torch.float64, device=self.device),
            group_off=torch.empty(n + 1, dtype=off_dtype, device=self.device) if off_dtype else None,
            summary=torch.zeros(4, dtype=torch.int64, device=self.device))
        hora_allocate_baseline(c, g0, budget, rule, out.delta, self.dev_status, self.workspace(n, g0),
                               delta_max=delta_max, util=out.util, group_off=out.group_off, summary=out.summary)
        return out

    def allocate_sharded(self, c: torch.Tensor, g0: int, shard_off: torch.Tensor, shard_budget: torch.Tensor, *,
                         alpha0: float = 1.0, beta0: float = 1.0, delta_max: int = 0, want_util: bool = True,
                         off_dtype: Optional[torch.dtype] = torch.int64,
                         want_summary: bool = True) -> Allocation:
        n, n_shards = c.numel(), shard_budget.numel()
        out = Allocation(
            delta=torch.empty(n, dtype=torch.int32, device=self.device),
            util=torch.empty(n, dtype=torch.float64, device=self.device) if want_util else None,
            group_off=torch.empty(n + 1, dtype=off_dtype, device=self.device) if off_dtype else None,
            summary=torch.zeros(4 * n_shards, dtype=torch.int64, device=self.device) if want_summary else None)
        need = hora_allocate_sharded_workspace_bytes(n_shards)
        if self._shard_workspace.numel() < need:
            self._shard_workspace = torch.zeros(need, dtype=torch.uint8, device=self.device)
        hora_allocate_sharded(c, g0, shard_off, shard_budget, out.delta, self.dev_status, self._shard_workspace,
                              alpha0=alpha0, beta0=beta0, delta_max=delta_max, util=out.util,
                              group_off=out.group_off, summary=out.summary)
        return out

    def allocate_posterior(self, alpha: torch.Tensor, beta: torch.Tensor, g0: int, budget: int, *,
                           delta_max: int = 0, want_util: bool = True,
                           off_dtype: Optional[torch.dtype] = torch.int64,
                           want_summary: bool = True) -> Allocation:
        n = alpha.numel()
        out = Allocation(
            delta=torch.empty(n, dtype=torch.int32, device=self.device),
            util=torch.empty(n, dtype=torch.float64, device=self.device) if want_util else None,
            group_off=torch.empty(n + 1, dtype=off_dtype, device=self.device) if off_dtype else None,
            summary=torch.zeros(4, dtype=torch.int64, device=self.device) if want_summary else None)
        hora_allocate_posterior(alpha, beta, g0, budget, out.delta, self.dev_status, self.workspace(n, g0),
                                delta_max=delta_max, util=out.util, group_off=out.group_off,
                                summary=out.summary)
        return out

    def group_advantage(self, group_off: torch.Tensor, reward: torch.Tensor, mode: int, *, eps: float = 0.0,
                        ddof: int = 0) -> torch.Tensor:
        adv = torch.empty_like(reward)
        hora_group_advantage(group_off, reward, adv, mode, self.dev_status, eps=eps, ddof=ddof)
        return adv

    def broadcast_workspace(self, n_tokens: int, out_dtype: torch.dtype = torch.float32) -> torch.Tensor:
        need = hora_token_broadcast_workspace_bytes(n_tokens, out_dtype)
        if self._bcast_workspace.numel() < need:
            self._bcast_workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._bcast_workspace

    def token_broadcast(self, adv: torch.Tensor, tok_off: torch.Tensor, n_tokens: int,
                        out_dtype: torch.dtype = torch.float32,
                        out: Optional[torch.Tensor] = None) -> torch.Tensor:
        tok_adv = out if out is not None else torch.empty(n_tokens, dtype=out_dtype, device=self.device)
        hora_token_broadcast(adv, tok_off, tok_adv, n_tokens, self.dev_status,
                             self.broadcast_workspace(n_tokens, tok_adv.dtype))
        return tok_adv

    def token_broadcast2(self, adv_a: torch.Tensor, adv_b: torch.Tensor, tok_off: torch.Tensor, n_tokens: int,
                         out_dtype: torch.dtype = torch.float32, out=None):
        if out is None:
            out = (torch.empty(n_tokens, dtype=out_dtype, device=self.device),
                   torch.empty(n_tokens, dtype=out_dtype, device=self.device))
        need = hora_token_broadcast2_workspace_bytes(n_tokens, out[0].dtype)
        if self._bcast_workspace.numel() < need:
            self._bcast_workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        hora_token_broadcast2(adv_a, adv_b, tok_off, out[0], out[1], n_tokens, self.dev_status,
                              self._bcast_workspace)
        return out

    def status(self) -> int:
        """Synchronises and returns the sticky device status (0 = no data error so far)."""
        return int(self.dev_status.item())

    def check(self) -> None:
        s = self.status()
        if s != OK:
            self.dev_status.zero_()
            raise HoraError(s, "device status")
