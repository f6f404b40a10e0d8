"""Thin ctypes binding of libtlora.so: argument marshalling only.

The functions mirror the C ABI declared in include/tlora.h (same names).  `LayerProblem` is a
convenience holder that keeps the host arrays and torch tensors of one problem alive and builds the
`tlora_problem_t` struct from them.  Every step of the layer runs inside the library's kernels;
there is no fallback: a missing library or a failed call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

TLORA_F32, TLORA_BF16 = 0, 1
TLORA_BWD_REUSE_S = 1
TLORA_BWD_REUSE_WT = 2
TLORA_BWD_ACCUMULATE = 4
TLORA_OK, TLORA_EINVAL, TLORA_ENULL, TLORA_EDTYPE, TLORA_EWORKSPACE, TLORA_EARCH, TLORA_EHIP, TLORA_EALIGN = 0, -1, -2, -3, -4, -5, -6, -7
TLORA_ESCRATCH = -8
TLORA_NOALLOC_SCRATCH_BYTES = 16 << 20

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("TLORA_LIB") or os.path.join(_HERE, "libtlora.so")
_lib = None


class TloraError(RuntimeError):
    pass


class tlora_problem_t(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("num_jobs", ctypes.c_int32),
                ("d_in", ctypes.c_int32), ("d_out", ctypes.c_int32),
                ("ranks", ctypes.POINTER(ctypes.c_int32)), ("offsets", ctypes.POINTER(ctypes.c_int64)),
                ("scales", ctypes.POINTER(ctypes.c_float)),
                ("X", ctypes.c_void_p), ("W", ctypes.c_void_p),
                ("A", ctypes.POINTER(ctypes.c_void_p)), ("B", ctypes.POINTER(ctypes.c_void_p))]


class tlora_aimd_t(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("alpha", ctypes.c_int32), ("n_max", ctypes.c_int32),
                ("have_prev", ctypes.c_int32), ("beta", ctypes.c_double), ("tau_rel", ctypes.c_double),
                ("t_prev", ctypes.c_double)]


class tlora_mlp_t(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("num_jobs", ctypes.c_int32), ("d_model", ctypes.c_int32),
                ("d_ff", ctypes.c_int32), ("ranks", ctypes.POINTER(ctypes.c_int32)),
                ("offsets", ctypes.POINTER(ctypes.c_int64)), ("scales", ctypes.POINTER(ctypes.c_float)),
                ("X", ctypes.c_void_p), ("gamma", ctypes.c_void_p), ("eps", ctypes.c_float),
                ("W_gate", ctypes.c_void_p), ("W_up", ctypes.c_void_p), ("W_down", ctypes.c_void_p),
                ("A_gate", ctypes.POINTER(ctypes.c_void_p)), ("B_gate", ctypes.POINTER(ctypes.c_void_p)),
                ("A_up", ctypes.POINTER(ctypes.c_void_p)), ("B_up", ctypes.POINTER(ctypes.c_void_p)),
                ("A_down", ctypes.POINTER(ctypes.c_void_p)), ("B_down", ctypes.POINTER(ctypes.c_void_p))]


class tlora_attn_t(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("num_jobs", ctypes.c_int32), ("d_model", ctypes.c_int32),
                ("n_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("rope_base", ctypes.c_float), ("eps", ctypes.c_float), ("ranks", ctypes.POINTER(ctypes.c_int32)),
                ("offsets", ctypes.POINTER(ctypes.c_int64)), ("scales", ctypes.POINTER(ctypes.c_float)),
                ("num_seqs", ctypes.c_int32), ("seq_offsets", ctypes.POINTER(ctypes.c_int64)),
                ("X", ctypes.c_void_p), ("gamma", ctypes.c_void_p),
                ("W_q", ctypes.c_void_p), ("W_k", ctypes.c_void_p), ("W_v", ctypes.c_void_p), ("W_o", ctypes.c_void_p),
                ("A_q", ctypes.POINTER(ctypes.c_void_p)), ("B_q", ctypes.POINTER(ctypes.c_void_p)),
                ("A_k", ctypes.POINTER(ctypes.c_void_p)), ("B_k", ctypes.POINTER(ctypes.c_void_p)),
                ("A_v", ctypes.POINTER(ctypes.c_void_p)), ("B_v", ctypes.POINTER(ctypes.c_void_p)),
                ("A_o", ctypes.POINTER(ctypes.c_void_p)), ("B_o", ctypes.POINTER(ctypes.c_void_p))]


class tlora_layer_t(ctypes.Structure):
    _fields_ = [("attn", tlora_attn_t), ("mlp", tlora_mlp_t)]


class tlora_sched_model_t(ctypes.Structure):
    _fields_ = [("n_points", ctypes.c_int32), ("tokens", ctypes.POINTER(ctypes.c_double)),
                ("ms", ctypes.POINTER(ctypes.c_double)), ("ms_per_token_rank", ctypes.c_double),
                ("ms_per_job", ctypes.c_double)]


class tlora_sched_job_t(ctypes.Structure):
    _fields_ = [("tokens", ctypes.c_int64), ("rank", ctypes.c_int32), ("steps", ctypes.c_int32),
                ("urgency", ctypes.c_double), ("max_slowdown", ctypes.c_double)]


class tlora_adamw_tensor_t(ctypes.Structure):
    _fields_ = [("param", ctypes.c_void_p), ("master", ctypes.c_void_p), ("grad", ctypes.c_void_p),
                ("m", ctypes.c_void_p), ("v", ctypes.c_void_p), ("n", ctypes.c_int64),
                ("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("step", ctypes.c_int32)]


EXPORTS = ["tlora_workspace_bytes", "tlora_fwd", "tlora_fwd_noalloc", "tlora_bwd", "tlora_adamw_workspace_bytes", "tlora_adamw_step",
           "tlora_mlp_workspace_bytes", "tlora_mlp_fwd", "tlora_mlp_bwd",
           "tlora_attention_workspace_bytes", "tlora_rope", "tlora_attention_fwd", "tlora_attention_bwd",
           "tlora_attn_workspace_bytes", "tlora_attn_fwd", "tlora_attn_bwd",
           "tlora_layer_workspace_bytes", "tlora_layer_fwd", "tlora_layer_bwd",
           "tlora_sched_step_ms", "tlora_sched_partition", "tlora_sched_simulate",
           "tlora_indexed_workspace_bytes", "tlora_fwd_indexed", "tlora_bwd_indexed",
           "tlora_aimd_init", "tlora_aimd_update",
           "tlora_nano_split", "tlora_nano_workspace_bytes", "tlora_fwd_nano", "tlora_bwd_nano",
           "tlora_plan_dump", "tlora_plan_check", "tlora_set_option",
           "tlora_profile", "tlora_profile_read", "tlora_profile_clock", "tlora_strerror", "tlora_last_hip_error",
           "tlora_version"]
KERNEL_CLASSES = ["pack", "shrink", "gemm_fwd", "gemm_bwd", "rank_grad", "grad_reduce", "f32", "w_transpose", "optimizer", "glue", "permute",
                  "attn_fwd", "attn_bwd", "rope"]


def lib() -> ctypes.CDLL:
    """Load libtlora.so; it is built first if it is missing or older than one of its sources (an explicit
    TLORA_LIB path is taken as it is)."""
    global _lib
    if _lib is not None:
        return _lib
    # One HIP runtime per process: PyTorch ships its own copy of libamdhip64 and loads it by path, so if this library
    # (linked against the system's copy) came first the process would hold two runtimes, and the second one finds
    # no device.  With torch loaded first the dynamic loader hands this library the copy that is already there.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.environ.get("TLORA_LIB"):
        from . import build as _build
        if _build.is_stale():
            _build.build()
    L = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(tlora_problem_t)
    L.tlora_workspace_bytes.restype = ctypes.c_size_t
    L.tlora_workspace_bytes.argtypes = [P]
    L.tlora_fwd.restype = ctypes.c_int
    L.tlora_fwd.argtypes = [P, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.tlora_fwd_noalloc.restype = ctypes.c_int
    L.tlora_fwd_noalloc.argtypes = [P, ctypes.c_void_p, ctypes.c_void_p]
    L.tlora_bwd.restype = ctypes.c_int
    L.tlora_bwd.argtypes = [P, ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p),
                            ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                            ctypes.c_void_p]
    PM = ctypes.POINTER(tlora_mlp_t)
    VPP = ctypes.POINTER(ctypes.c_void_p)
    PA = ctypes.POINTER(tlora_attn_t)
    I64P, VP, I32, SZ = ctypes.POINTER(ctypes.c_int64), ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    L.tlora_attention_workspace_bytes.restype = SZ
    L.tlora_attention_workspace_bytes.argtypes = [I32, I64P, I32]
    L.tlora_rope.restype = ctypes.c_int
    L.tlora_rope.argtypes = [VP, I32, I64P, I32, I32, ctypes.c_float, I32, VP, SZ, VP]
    L.tlora_attention_fwd.restype = ctypes.c_int
    L.tlora_attention_fwd.argtypes = [VP, VP, VP, VP, VP, I32, I64P, I32, I32, I32, VP, SZ, VP]
    L.tlora_attention_bwd.restype = ctypes.c_int
    L.tlora_attention_bwd.argtypes = [VP] * 9 + [I32, I64P, I32, I32, I32, VP, SZ, VP]
    L.tlora_attn_workspace_bytes.restype = SZ
    L.tlora_attn_workspace_bytes.argtypes = [PA]
    L.tlora_attn_fwd.restype = ctypes.c_int
    L.tlora_attn_fwd.argtypes = [PA, VP, VP, SZ, VP]
    L.tlora_attn_bwd.restype = ctypes.c_int
    L.tlora_attn_bwd.argtypes = [PA, VP, VP, ctypes.POINTER(VPP), ctypes.POINTER(VPP), ctypes.c_int, VP, SZ, VP]
    PSM, PSJ = ctypes.POINTER(tlora_sched_model_t), ctypes.POINTER(tlora_sched_job_t)
    I32P, DP = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)
    L.tlora_sched_step_ms.restype = ctypes.c_int
    L.tlora_sched_step_ms.argtypes = [PSM, I32, PSJ, I32P, I32, DP]
    L.tlora_sched_partition.restype = ctypes.c_int
    L.tlora_sched_partition.argtypes = [PSM, I32, PSJ, I32P, I32P]
    L.tlora_sched_simulate.restype = ctypes.c_int
    L.tlora_sched_simulate.argtypes = [PSM, I32, PSJ, I32, DP, DP, I32P, I32P, I32P, I64P, ctypes.c_int64]
    PL = ctypes.POINTER(tlora_layer_t)
    L.tlora_layer_workspace_bytes.restype = SZ
    L.tlora_layer_workspace_bytes.argtypes = [PL]
    L.tlora_layer_fwd.restype = ctypes.c_int
    L.tlora_layer_fwd.argtypes = [PL, VP, VP, SZ, VP]
    L.tlora_layer_bwd.restype = ctypes.c_int
    L.tlora_layer_bwd.argtypes = [PL, VP, VP, ctypes.POINTER(VPP), ctypes.POINTER(VPP), ctypes.c_int, VP, SZ, VP]
    L.tlora_mlp_workspace_bytes.restype = ctypes.c_size_t
    L.tlora_mlp_workspace_bytes.argtypes = [PM]
    L.tlora_mlp_fwd.restype = ctypes.c_int
    L.tlora_mlp_fwd.argtypes = [PM, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.tlora_mlp_bwd.restype = ctypes.c_int
    L.tlora_mlp_bwd.argtypes = [PM, ctypes.c_void_p, ctypes.c_void_p, VPP, VPP, VPP, VPP, VPP, VPP, ctypes.c_int,
                                ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.tlora_indexed_workspace_bytes.restype = ctypes.c_size_t
    L.tlora_indexed_workspace_bytes.argtypes = [P]
    L.tlora_fwd_indexed.restype = ctypes.c_int
    L.tlora_fwd_indexed.argtypes = [P, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.tlora_bwd_indexed.restype = ctypes.c_int
    L.tlora_bwd_indexed.argtypes = [P, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, VPP, VPP, ctypes.c_int,
                                    ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.tlora_adamw_workspace_bytes.restype = ctypes.c_size_t
    L.tlora_adamw_workspace_bytes.argtypes = [ctypes.c_int32]
    L.tlora_adamw_step.restype = ctypes.c_int
    L.tlora_adamw_step.argtypes = [ctypes.POINTER(tlora_adamw_tensor_t), ctypes.c_int32, ctypes.c_int32,
                                   ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.tlora_aimd_init.restype = ctypes.c_int
    L.tlora_aimd_init.argtypes = [ctypes.POINTER(tlora_aimd_t), ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                  ctypes.c_double, ctypes.c_int32]
    L.tlora_aimd_update.restype = ctypes.c_int
    L.tlora_aimd_update.argtypes = [ctypes.POINTER(tlora_aimd_t), ctypes.c_double, ctypes.POINTER(ctypes.c_int32)]
    L.tlora_nano_split.restype = ctypes.c_int
    L.tlora_nano_split.argtypes = [P, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64),
                                   ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]
    L.tlora_nano_workspace_bytes.restype = ctypes.c_size_t
    L.tlora_nano_workspace_bytes.argtypes = [P, ctypes.c_int32, ctypes.c_int64]
    L.tlora_fwd_nano.restype = ctypes.c_int
    L.tlora_fwd_nano.argtypes = [P, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                 ctypes.c_void_p]
    L.tlora_bwd_nano.restype = ctypes.c_int
    L.tlora_bwd_nano.argtypes = [P, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                 ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
                                 ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.tlora_plan_dump.restype = ctypes.c_int
    L.tlora_plan_dump.argtypes = [P, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64),
                                  ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64),
                                  ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32),
                                  ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)]
    L.tlora_plan_check.restype = ctypes.c_int
    L.tlora_plan_check.argtypes = [P, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    L.tlora_set_option.restype = ctypes.c_int
    L.tlora_set_option.argtypes = [ctypes.c_char_p, ctypes.c_int64]
    L.tlora_profile.restype = ctypes.c_int
    L.tlora_profile.argtypes = [ctypes.c_int]
    L.tlora_profile_read.restype = ctypes.c_int
    L.tlora_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    L.tlora_profile_clock.restype = ctypes.c_int
    L.tlora_profile_clock.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    L.tlora_strerror.restype = ctypes.c_char_p
    L.tlora_strerror.argtypes = [ctypes.c_int]
    L.tlora_last_hip_error.restype = ctypes.c_char_p
    L.tlora_last_hip_error.argtypes = []
    L.tlora_version.restype = ctypes.c_char_p
    L.tlora_version.argtypes = []
    _lib = L
    return L


def tlora_strerror(status: int) -> str:
    return lib().tlora_strerror(int(status)).decode()


def tlora_version() -> str:
    return lib().tlora_version().decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        detail = f": {lib().tlora_last_hip_error().decode()}" if status == TLORA_EHIP else ""
        raise TloraError(f"{what} failed: {status} ({tlora_strerror(status)}{detail})")


def tlora_set_option(name: str, value: int) -> None:
    _check(lib().tlora_set_option(name.encode(), int(value)), f"tlora_set_option({name})")


def tlora_profile(enable) -> None:
    """False / 0: off; True / 1: bracket every kernel launch with events; 2: only the segmented GEMMs."""
    _check(lib().tlora_profile(int(enable)), "tlora_profile")


def tlora_profile_read() -> dict:
    """{kernel class name: (total milliseconds, launches)} since profiling was enabled."""
    out = {}
    for i, name in enumerate(KERNEL_CLASSES):
        ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
        _check(lib().tlora_profile_read(i, ctypes.byref(ms), ctypes.byref(n)), "tlora_profile_read")
        out[name] = (float(ms.value), int(n.value))
    return out


def tlora_profile_clock():
    """(GHz seen by the last profiled forward GEMM, GHz seen by the last profiled dX GEMM); 0.0 = none yet."""
    a, b = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib().tlora_profile_clock(ctypes.byref(a), ctypes.byref(b)), "tlora_profile_clock")
    return float(a.value), float(b.value)


def make_problem(dtype: int, d_in: int, d_out: int, ranks: Sequence[int], offsets: Sequence[int],
                 scales: Sequence[float], X_ptr: int, W_ptr: int, A_ptrs: Sequence[int],
                 B_ptrs: Sequence[int]):
    """Build a tlora_problem_t from plain integers; returns (struct, keepalive list)."""
    J = len(ranks)
    c_ranks = (ctypes.c_int32 * J)(*[int(r) for r in ranks])
    c_off = (ctypes.c_int64 * (J + 1))(*[int(o) for o in offsets])
    c_scales = (ctypes.c_float * J)(*[float(s) for s in scales])
    c_A = (ctypes.c_void_p * J)(*[ctypes.c_void_p(int(p)) if p else None for p in A_ptrs])
    c_B = (ctypes.c_void_p * J)(*[ctypes.c_void_p(int(p)) if p else None for p in B_ptrs])
    prob = tlora_problem_t(int(dtype), J, int(d_in), int(d_out), c_ranks, c_off, c_scales,
                           ctypes.c_void_p(int(X_ptr)) if X_ptr else None,
                           ctypes.c_void_p(int(W_ptr)) if W_ptr else None, c_A, c_B)
    return prob, [c_ranks, c_off, c_scales, c_A, c_B]


def tlora_workspace_bytes(prob: tlora_problem_t) -> int:
    return int(lib().tlora_workspace_bytes(ctypes.byref(prob)))


def tlora_fwd(prob: tlora_problem_t, Y_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(lib().tlora_fwd(ctypes.byref(prob), ctypes.c_void_p(Y_ptr), ctypes.c_void_p(ws_ptr),
                           ctypes.c_size_t(ws_bytes), ctypes.c_void_p(stream)), "tlora_fwd")


def tlora_fwd_noalloc(prob: tlora_problem_t, Y_ptr: int, stream: int = 0) -> None:
    _check(lib().tlora_fwd_noalloc(ctypes.byref(prob), ctypes.c_void_p(Y_ptr), ctypes.c_void_p(stream)),
           "tlora_fwd_noalloc")


def tlora_bwd(prob: tlora_problem_t, dY_ptr: int, dX_ptr: int, dA_ptrs: Optional[Sequence[int]],
              dB_ptrs: Optional[Sequence[int]], flags: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    J = prob.num_jobs
    if dA_ptrs is None:
        c_dA = c_dB = None
    else:
        c_dA = (ctypes.c_void_p * J)(*[ctypes.c_void_p(int(p)) if p else None for p in dA_ptrs])
        c_dB = (ctypes.c_void_p * J)(*[ctypes.c_void_p(int(p)) if p else None for p in dB_ptrs])
    _check(lib().tlora_bwd(ctypes.byref(prob), ctypes.c_void_p(dY_ptr), ctypes.c_void_p(dX_ptr) if dX_ptr else None,
                           c_dA, c_dB, int(flags), ctypes.c_void_p(ws_ptr), ctypes.c_size_t(ws_bytes),
                           ctypes.c_void_p(stream)), "tlora_bwd")


def _grad_ptr_arrays(J, dA_ptrs, dB_ptrs):
    if dA_ptrs is None:
        return None, None
    return ((ctypes.c_void_p * J)(*[ctypes.c_void_p(int(p)) if p else None for p in dA_ptrs]),
            (ctypes.c_void_p * J)(*[ctypes.c_void_p(int(p)) if p else None for p in dB_ptrs]))


def tlora_adamw_workspace_bytes(count: int) -> int:
    return int(lib().tlora_adamw_workspace_bytes(int(count)))


def tlora_adamw_step(tensors: Sequence[dict], dtype: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    """tensors: dicts with integer device pointers param / master / grad / m / v, n and the hyper-parameters."""
    arr = (tlora_adamw_tensor_t * len(tensors))()
    for a, t in zip(arr, tensors):
        a.param, a.master, a.grad, a.m, a.v = (t["param"] or None, t.get("master") or None, t["grad"] or None,
                                               t["m"] or None, t["v"] or None)
        a.n = int(t["n"])
        a.lr, a.beta1, a.beta2 = float(t["lr"]), float(t.get("beta1", 0.9)), float(t.get("beta2", 0.999))
        a.eps, a.weight_decay, a.step = float(t.get("eps", 1e-8)), float(t.get("weight_decay", 0.0)), int(t["step"])
    _check(lib().tlora_adamw_step(arr, len(tensors), int(dtype), ctypes.c_void_p(ws_ptr), ctypes.c_size_t(ws_bytes),
                                  ctypes.c_void_p(stream)), "tlora_adamw_step")


def tlora_aimd_init(n0: int, alpha: int = 4, beta: float = 0.5, tau_rel: float = 0.02, n_max: int = 0) -> tlora_aimd_t:
    c = tlora_aimd_t()
    _check(lib().tlora_aimd_init(ctypes.byref(c), int(n0), int(alpha), float(beta), float(tau_rel), int(n_max)),
           "tlora_aimd_init")
    return c


def tlora_aimd_update(c: tlora_aimd_t, t_step: float) -> int:
    n = ctypes.c_int32(0)
    _check(lib().tlora_aimd_update(ctypes.byref(c), float(t_step), ctypes.byref(n)), "tlora_aimd_update")
    return int(n.value)


def tlora_nano_split(prob: tlora_problem_t, n_nano: int, granule: int, n: int):
    """(row0, row1, sub-offsets) of nano-batch n."""
    r0, r1 = ctypes.c_int64(0), ctypes.c_int64(0)
    sub = (ctypes.c_int64 * (prob.num_jobs + 1))()
    _check(lib().tlora_nano_split(ctypes.byref(prob), int(n_nano), int(granule), int(n), ctypes.byref(r0),
                                  ctypes.byref(r1), sub), "tlora_nano_split")
    return int(r0.value), int(r1.value), list(sub)


def tlora_nano_workspace_bytes(prob: tlora_problem_t, n_nano: int, granule: int) -> int:
    return int(lib().tlora_nano_workspace_bytes(ctypes.byref(prob), int(n_nano), int(granule)))


def tlora_fwd_nano(prob: tlora_problem_t, n_nano: int, granule: int, Y_ptr: int, ws_ptr: int, ws_bytes: int,
                   stream: int = 0) -> None:
    _check(lib().tlora_fwd_nano(ctypes.byref(prob), int(n_nano), int(granule), ctypes.c_void_p(Y_ptr),
                                ctypes.c_void_p(ws_ptr), ctypes.c_size_t(ws_bytes), ctypes.c_void_p(stream)),
           "tlora_fwd_nano")


def tlora_bwd_nano(prob: tlora_problem_t, n_nano: int, granule: int, dY_ptr: int, dX_ptr: int,
                   dA_ptrs: Optional[Sequence[int]], dB_ptrs: Optional[Sequence[int]], flags: int, ws_ptr: int,
                   ws_bytes: int, stream: int = 0) -> None:
    c_dA, c_dB = _grad_ptr_arrays(prob.num_jobs, dA_ptrs, dB_ptrs)
    _check(lib().tlora_bwd_nano(ctypes.byref(prob), int(n_nano), int(granule), ctypes.c_void_p(dY_ptr),
                                ctypes.c_void_p(dX_ptr) if dX_ptr else None, c_dA, c_dB, int(flags),
                                ctypes.c_void_p(ws_ptr), ctypes.c_size_t(ws_bytes), ctypes.c_void_p(stream)),
           "tlora_bwd_nano")


def tlora_indexed_workspace_bytes(prob: tlora_problem_t) -> int:
    return int(lib().tlora_indexed_workspace_bytes(ctypes.byref(prob)))


def tlora_fwd_indexed(prob: tlora_problem_t, index_ptr: int, Y_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(lib().tlora_fwd_indexed(ctypes.byref(prob), ctypes.c_void_p(index_ptr), ctypes.c_void_p(Y_ptr),
                                   ctypes.c_void_p(ws_ptr), ctypes.c_size_t(ws_bytes), ctypes.c_void_p(stream)),
           "tlora_fwd_indexed")


def tlora_bwd_indexed(prob: tlora_problem_t, index_ptr: int, dY_ptr: int, dX_ptr: int,
                      dA_ptrs: Optional[Sequence[int]], dB_ptrs: Optional[Sequence[int]], flags: int, ws_ptr: int,
                      ws_bytes: int, stream: int = 0) -> None:
    c_dA, c_dB = _grad_ptr_arrays(prob.num_jobs, dA_ptrs, dB_ptrs)
    _check(lib().tlora_bwd_indexed(ctypes.byref(prob), ctypes.c_void_p(index_ptr), ctypes.c_void_p(dY_ptr),
                                   ctypes.c_void_p(dX_ptr) if dX_ptr else None, c_dA, c_dB, int(flags),
                                   ctypes.c_void_p(ws_ptr), ctypes.c_size_t(ws_bytes), ctypes.c_void_p(stream)),
           "tlora_bwd_indexed")


def tlora_plan_dump(prob: tlora_problem_t) -> dict:
    """The plan's integer bookkeeping as Python lists."""
    J = prob.num_jobs
    L = lib()
    n = ctypes.c_int64(0)
    rpad = (ctypes.c_int32 * J)()
    soff = (ctypes.c_int64 * (J + 1))()
    tile_rows = ctypes.c_int32(0)
    _check(L.tlora_plan_dump(ctypes.byref(prob), rpad, soff, ctypes.byref(tile_rows), None, None, None, None,
                             ctypes.byref(n)), "tlora_plan_dump")
    nt = max(int(n.value), 1)
    row0 = (ctypes.c_int64 * nt)()
    nrows = (ctypes.c_int32 * nt)()
    jf = (ctypes.c_int32 * nt)()
    jl = (ctypes.c_int32 * nt)()
    n2 = ctypes.c_int64(nt)
    _check(L.tlora_plan_dump(ctypes.byref(prob), None, None, None, row0, nrows, jf, jl, ctypes.byref(n2)),
           "tlora_plan_dump")
    k = int(n.value)
    return {"rpad": list(rpad), "soff": list(soff), "tile_rows": int(tile_rows.value),
            "tiles": [(int(row0[i]), int(nrows[i]), int(jf[i]), int(jl[i])) for i in range(k)]}


def tlora_plan_check(prob: tlora_problem_t, fwd_only: bool = False):
    """(status, number of the first failed consistency check or 0) for a freshly built plan of `prob`."""
    bad = ctypes.c_int32(0)
    rc = lib().tlora_plan_check(ctypes.byref(prob), 1 if fwd_only else 0, ctypes.byref(bad))
    return int(rc), int(bad.value)


# ---- torch-backed convenience holder ---------------------------------------------------------------------
class LayerProblem:
    """Device tensors of one fused-layer problem plus the marshalled struct.

    Torch only owns the device memory and supplies the stream; all computation is in libtlora.so."""

    def __init__(self, dtype: str, d_in: int, d_out: int, ranks, offsets, scales, X, W, A: List, B: List):
        import torch
        self.torch = torch
        self.dtype = dtype
        self.code = TLORA_BF16 if dtype == "bf16" else TLORA_F32
        self.d_in, self.d_out = int(d_in), int(d_out)
        self.ranks = [int(r) for r in ranks]
        self.offsets = [int(o) for o in offsets]
        self.scales = [float(s) for s in scales]
        self.X, self.W, self.A, self.B = X, W, list(A), list(B)
        self.T = self.offsets[-1]
        self.prob, self._keep = make_problem(
            self.code, d_in, d_out, self.ranks, self.offsets, self.scales, X.data_ptr(), W.data_ptr(),
            [a.data_ptr() if a is not None and a.numel() else 0 for a in self.A],
            [b.data_ptr() if b is not None and b.numel() else 0 for b in self.B])
        self.ws_bytes = tlora_workspace_bytes(self.prob)
        if self.ws_bytes == 0:
            raise TloraError("tlora_workspace_bytes: invalid problem")
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=X.device)

    @classmethod
    def from_numpy(cls, p, device="cuda"):
        """Upload a workloads.Problem (float32 numpy arrays) in its dtype."""
        import torch
        tdt = torch.bfloat16 if p.dtype == "bf16" else torch.float32

        def up(a):
            return torch.from_numpy(a).to(device=device, dtype=tdt).contiguous()
        return cls(p.dtype, p.d_in, p.d_out, p.ranks, p.offsets, p.scales, up(p.X), up(p.W),
                   [up(a) for a in p.A], [up(b) for b in p.B])

    def _stream(self) -> int:
        return int(self.torch.cuda.current_stream().cuda_stream)

    def new_outputs(self):
        t = self.torch
        tdt = t.bfloat16 if self.dtype == "bf16" else t.float32
        dev = self.X.device
        Y = t.empty((self.T, self.d_out), dtype=tdt, device=dev)
        dX = t.empty((self.T, self.d_in), dtype=tdt, device=dev)
        dA = [t.empty((self.d_in, r), dtype=t.float32, device=dev) for r in self.ranks]
        dB = [t.empty((r, self.d_out), dtype=t.float32, device=dev) for r in self.ranks]
        return Y, dX, dA, dB

    def fwd(self, Y) -> None:
        tlora_fwd(self.prob, Y.data_ptr(), self.ws.data_ptr(), self.ws_bytes, self._stream())

    def bwd(self, dY, dX, dA, dB, reuse_S: bool = False, flags: int = 0) -> None:
        tlora_bwd(self.prob, dY.data_ptr(), dX.data_ptr() if dX is not None else 0,
                  None if dA is None else [a.data_ptr() if a.numel() else 0 for a in dA],
                  None if dB is None else [b.data_ptr() if b.numel() else 0 for b in dB],
                  (TLORA_BWD_REUSE_S if reuse_S else 0) | flags, self.ws.data_ptr(), self.ws_bytes, self._stream())

    def _nano_ws(self, n_nano: int, granule: int) -> None:
        """Grow the workspace to what this partition needs (its tiles start at other rows than the whole batch's, so a
        tile may hold more jobs and its K-extension operand may be wider)."""
        need = tlora_nano_workspace_bytes(self.prob, n_nano, granule)
        if need == 0:
            raise TloraError("tlora_nano_workspace_bytes: invalid problem or partition")
        if need > self.ws_bytes:
            self.ws = self.torch.empty(need, dtype=self.torch.uint8, device=self.X.device)
            self.ws_bytes = need

    def fwd_nano(self, n_nano: int, granule: int, Y) -> None:
        """Forward over n_nano nano-batches."""
        self._nano_ws(n_nano, granule)
        tlora_fwd_nano(self.prob, n_nano, granule, Y.data_ptr(), self.ws.data_ptr(), self.ws_bytes, self._stream())

    def bwd_nano(self, n_nano: int, granule: int, dY, dX, dA, dB, flags: int = 0) -> None:
        self._nano_ws(n_nano, granule)
        tlora_bwd_nano(self.prob, n_nano, granule, dY.data_ptr(), dX.data_ptr() if dX is not None else 0,
                       None if dA is None else [a.data_ptr() if a.numel() else 0 for a in dA],
                       None if dB is None else [b.data_ptr() if b.numel() else 0 for b in dB],
                       flags, self.ws.data_ptr(), self.ws_bytes, self._stream())

    def job_slice(self, j: int) -> "LayerProblem":
        """Job j alone as a one-job problem over views of the same tensors (the per-job loop baseline)."""
        lo, hi = self.offsets[j], self.offsets[j + 1]
        return LayerProblem(self.dtype, self.d_in, self.d_out, [self.ranks[j]], [0, hi - lo], [self.scales[j]],
                            self.X[lo:hi], self.W, [self.A[j]], [self.B[j]])


class MlpBlock:
    """Holder of one MLP-block problem (torch tensors) marshalling pointers to tlora_mlp_fwd / tlora_mlp_bwd.
    `layers` = {"gate": (W, [A_j], [B_j]), "up": (...), "down": (...)}."""

    def __init__(self, dtype: str, d_model: int, d_ff: int, ranks, offsets, scales, X, gamma, eps: float, layers):
        import torch
        self.torch, self.dtype, self.d_model, self.d_ff = torch, dtype, int(d_model), int(d_ff)
        self.ranks, self.offsets = [int(r) for r in ranks], [int(o) for o in offsets]
        self.T, J = self.offsets[-1], len(self.ranks)
        self.X, self.gamma, self.layers = X, gamma, layers
        self._keep = [(ctypes.c_int32 * J)(*self.ranks), (ctypes.c_int64 * (J + 1))(*self.offsets),
                      (ctypes.c_float * J)(*[float(x) for x in scales])]

        def ptrs(ts):
            a = (ctypes.c_void_p * J)(*[ctypes.c_void_p(t.data_ptr()) if t.numel() else None for t in ts])
            self._keep.append(a)
            return a
        self.prob = tlora_mlp_t(TLORA_BF16 if dtype == "bf16" else TLORA_F32, J, self.d_model, self.d_ff,
                                self._keep[0], self._keep[1], self._keep[2],
                                ctypes.c_void_p(X.data_ptr()) if self.T else None, ctypes.c_void_p(gamma.data_ptr()),
                                float(eps), ctypes.c_void_p(layers["gate"][0].data_ptr()),
                                ctypes.c_void_p(layers["up"][0].data_ptr()), ctypes.c_void_p(layers["down"][0].data_ptr()),
                                ptrs(layers["gate"][1]), ptrs(layers["gate"][2]), ptrs(layers["up"][1]),
                                ptrs(layers["up"][2]), ptrs(layers["down"][1]), ptrs(layers["down"][2]))
        self.ws_bytes = int(lib().tlora_mlp_workspace_bytes(ctypes.byref(self.prob)))
        if self.ws_bytes == 0:
            raise TloraError("tlora_mlp_workspace_bytes: invalid problem")
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=X.device)

    def _stream(self) -> int:
        return int(self.torch.cuda.current_stream().cuda_stream)

    def new_grads(self):
        t = self.torch
        dev = self.X.device
        out = {}
        for name, (W, A, B) in self.layers.items():
            out[name] = ([t.empty(a.shape, dtype=t.float32, device=dev) for a in A],
                         [t.empty(b.shape, dtype=t.float32, device=dev) for b in B])
        return out

    def fwd(self, Out) -> None:
        _check(lib().tlora_mlp_fwd(ctypes.byref(self.prob), ctypes.c_void_p(Out.data_ptr()) if self.T else None,
                                   ctypes.c_void_p(self.ws.data_ptr()), ctypes.c_size_t(self.ws_bytes),
                                   ctypes.c_void_p(self._stream())), "tlora_mlp_fwd")

    def bwd(self, dOut, dX, grads, flags: int = 0) -> None:
        J = len(self.ranks)

        def arr(ts):
            return (ctypes.c_void_p * J)(*[ctypes.c_void_p(t.data_ptr()) if t.numel() else None for t in ts])
        a = [arr(grads[n][k]) for n in ("gate", "up", "down") for k in (0, 1)]
        _check(lib().tlora_mlp_bwd(ctypes.byref(self.prob), ctypes.c_void_p(dOut.data_ptr()) if self.T else None,
                                   ctypes.c_void_p(dX.data_ptr()) if self.T else None, *a, int(flags),
                                   ctypes.c_void_p(self.ws.data_ptr()), ctypes.c_size_t(self.ws_bytes),
                                   ctypes.c_void_p(self._stream())), "tlora_mlp_bwd")


class Attention:
    """Rotary embedding and causal grouped-query attention over token rows cut into sequences by `seq_offsets`
    (argument marshalling for tlora_rope / tlora_attention_fwd / tlora_attention_bwd; bf16, head size 128)."""

    def __init__(self, seq_offsets, n_heads: int, n_kv_heads: int, device, head_dim: int = 128):
        import torch
        self.torch = torch
        self.seq = [int(o) for o in seq_offsets]
        self.S, self.T = len(self.seq) - 1, self.seq[-1]
        self.n_heads, self.n_kv, self.hd = int(n_heads), int(n_kv_heads), int(head_dim)
        self._seq = (ctypes.c_int64 * (self.S + 1))(*self.seq)
        self.ws_bytes = int(lib().tlora_attention_workspace_bytes(self.S, self._seq, self.n_heads))
        if self.ws_bytes == 0:
            raise TloraError("tlora_attention_workspace_bytes: invalid problem")
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)

    def _tail(self):
        return (ctypes.c_void_p(self.ws.data_ptr()), ctypes.c_size_t(self.ws_bytes),
                ctypes.c_void_p(int(self.torch.cuda.current_stream().cuda_stream)))

    @staticmethod
    def _p(t):
        return ctypes.c_void_p(t.data_ptr()) if t.numel() else None

    def rope(self, X, heads: int, base: float, inverse: bool = False) -> None:
        _check(lib().tlora_rope(self._p(X), self.S, self._seq, int(heads), self.hd, float(base), int(bool(inverse)),
                                *self._tail()), "tlora_rope")

    def fwd(self, Q, K, V, O, lse) -> None:
        p = self._p
        _check(lib().tlora_attention_fwd(p(Q), p(K), p(V), p(O), p(lse), self.S, self._seq, self.n_heads, self.n_kv,
                                         self.hd, *self._tail()), "tlora_attention_fwd")

    def bwd(self, Q, K, V, O, dO, lse, dQ, dK, dV) -> None:
        p = self._p
        _check(lib().tlora_attention_bwd(p(Q), p(K), p(V), p(O), p(dO), p(lse), p(dQ), p(dK), p(dV), self.S, self._seq,
                                         self.n_heads, self.n_kv, self.hd, *self._tail()), "tlora_attention_bwd")


class AttnBlock:
    """Holder of one attention-block problem (torch tensors) marshalling pointers to tlora_attn_fwd / tlora_attn_bwd.
    `layers` = {"q": (W, [A_j], [B_j]), "k": (...), "v": (...), "o": (...)}."""
    NAMES = ("q", "k", "v", "o")

    def __init__(self, d_model: int, n_heads: int, n_kv_heads: int, rope_base: float, ranks, offsets, scales,
                 seq_offsets, X, gamma, eps: float, layers, head_dim: int = 128):
        import torch
        self.torch, self.d_model = torch, int(d_model)
        self.ranks, self.offsets = [int(r) for r in ranks], [int(o) for o in offsets]
        self.seq = [int(o) for o in seq_offsets]
        self.T, J = self.offsets[-1], len(self.ranks)
        self.X, self.gamma, self.layers = X, gamma, layers
        self._keep = [(ctypes.c_int32 * J)(*self.ranks), (ctypes.c_int64 * (J + 1))(*self.offsets),
                      (ctypes.c_float * J)(*[float(x) for x in scales]), (ctypes.c_int64 * len(self.seq))(*self.seq)]

        def ptrs(ts):
            a = (ctypes.c_void_p * J)(*[ctypes.c_void_p(t.data_ptr()) if t.numel() else None for t in ts])
            self._keep.append(a)
            return a
        ab = [ptrs(layers[n][k]) for n in self.NAMES for k in (1, 2)]
        self.prob = tlora_attn_t(TLORA_BF16, J, self.d_model, int(n_heads), int(n_kv_heads), int(head_dim),
                                 float(rope_base), float(eps), self._keep[0], self._keep[1], self._keep[2],
                                 len(self.seq) - 1, self._keep[3],
                                 ctypes.c_void_p(X.data_ptr()) if self.T else None, ctypes.c_void_p(gamma.data_ptr()),
                                 *[ctypes.c_void_p(layers[n][0].data_ptr()) for n in self.NAMES], *ab)
        self.ws_bytes = int(lib().tlora_attn_workspace_bytes(ctypes.byref(self.prob)))
        if self.ws_bytes == 0:
            raise TloraError("tlora_attn_workspace_bytes: invalid problem")
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=X.device)

    def _stream(self) -> int:
        return int(self.torch.cuda.current_stream().cuda_stream)

    def new_grads(self):
        t = self.torch
        dev = self.X.device
        return {n: ([t.empty(a.shape, dtype=t.float32, device=dev) for a in A],
                    [t.empty(b.shape, dtype=t.float32, device=dev) for b in B]) for n, (W, A, B) in self.layers.items()}

    def fwd(self, Out) -> None:
        _check(lib().tlora_attn_fwd(ctypes.byref(self.prob), ctypes.c_void_p(Out.data_ptr()) if self.T else None,
                                    ctypes.c_void_p(self.ws.data_ptr()), ctypes.c_size_t(self.ws_bytes),
                                    ctypes.c_void_p(self._stream())), "tlora_attn_fwd")

    def bwd(self, dOut, dX, grads, flags: int = 0) -> None:
        J = len(self.ranks)
        VPP = ctypes.POINTER(ctypes.c_void_p)

        def arr(ts):
            return (ctypes.c_void_p * J)(*[ctypes.c_void_p(t.data_ptr()) if t.numel() else None for t in ts])
        da = [arr(grads[n][0]) for n in self.NAMES]
        db = [arr(grads[n][1]) for n in self.NAMES]
        dA = (VPP * 4)(*[ctypes.cast(a, VPP) for a in da])
        dB = (VPP * 4)(*[ctypes.cast(a, VPP) for a in db])
        _check(lib().tlora_attn_bwd(ctypes.byref(self.prob), ctypes.c_void_p(dOut.data_ptr()) if self.T else None,
                                    ctypes.c_void_p(dX.data_ptr()) if self.T else None, dA, dB, int(flags),
                                    ctypes.c_void_p(self.ws.data_ptr()), ctypes.c_size_t(self.ws_bytes),
                                    ctypes.c_void_p(self._stream())), "tlora_attn_bwd")


class DecoderLayer:
    """Holder of one decoder-layer problem (torch tensors) marshalling pointers to tlora_layer_fwd / tlora_layer_bwd.
    `layers` maps "q", "k", "v", "o", "gate", "up", "down" to (W, [A_j], [B_j]); gamma_attn / gamma_mlp are the two
    RMSNorm weights."""
    NAMES = ("q", "k", "v", "o", "gate", "up", "down")

    def __init__(self, d_model: int, d_ff: int, n_heads: int, n_kv_heads: int, rope_base: float, ranks, offsets, scales,
                 seq_offsets, X, gamma_attn, gamma_mlp, eps: float, layers, head_dim: int = 128):
        import torch
        self.torch, self.d_model, self.d_ff = torch, int(d_model), int(d_ff)
        self.ranks, self.offsets = [int(r) for r in ranks], [int(o) for o in offsets]
        self.seq = [int(o) for o in seq_offsets]
        self.T, J = self.offsets[-1], len(self.ranks)
        self.X, self.layers = X, layers
        self._keep = [(ctypes.c_int32 * J)(*self.ranks), (ctypes.c_int64 * (J + 1))(*self.offsets),
                      (ctypes.c_float * J)(*[float(x) for x in scales]), (ctypes.c_int64 * len(self.seq))(*self.seq),
                      gamma_attn, gamma_mlp]

        def ptrs(ts):
            a = (ctypes.c_void_p * J)(*[ctypes.c_void_p(t.data_ptr()) if t.numel() else None for t in ts])
            self._keep.append(a)
            return a
        w = lambda n: ctypes.c_void_p(layers[n][0].data_ptr())
        ab = {n: (ptrs(layers[n][1]), ptrs(layers[n][2])) for n in self.NAMES}
        xp = ctypes.c_void_p(X.data_ptr()) if self.T else None
        attn = tlora_attn_t(TLORA_BF16, J, self.d_model, int(n_heads), int(n_kv_heads), int(head_dim), float(rope_base),
                            float(eps), self._keep[0], self._keep[1], self._keep[2], len(self.seq) - 1, self._keep[3],
                            xp, ctypes.c_void_p(gamma_attn.data_ptr()), w("q"), w("k"), w("v"), w("o"),
                            *[ab[n][k] for n in ("q", "k", "v", "o") for k in (0, 1)])
        mlp = tlora_mlp_t(TLORA_BF16, J, self.d_model, self.d_ff, self._keep[0], self._keep[1], self._keep[2], None,
                          ctypes.c_void_p(gamma_mlp.data_ptr()), float(eps), w("gate"), w("up"), w("down"),
                          *[ab[n][k] for n in ("gate", "up", "down") for k in (0, 1)])
        self.prob = tlora_layer_t(attn, mlp)
        self.ws_bytes = int(lib().tlora_layer_workspace_bytes(ctypes.byref(self.prob)))
        if self.ws_bytes == 0:
            raise TloraError("tlora_layer_workspace_bytes: invalid problem")
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=X.device)

    def _stream(self) -> int:
        return int(self.torch.cuda.current_stream().cuda_stream)

    def new_grads(self):
        t = self.torch
        dev = self.X.device
        return {n: ([t.empty(a.shape, dtype=t.float32, device=dev) for a in A],
                    [t.empty(b.shape, dtype=t.float32, device=dev) for b in B]) for n, (W, A, B) in self.layers.items()}

    def fwd(self, Out) -> None:
        _check(lib().tlora_layer_fwd(ctypes.byref(self.prob), ctypes.c_void_p(Out.data_ptr()) if self.T else None,
                                     ctypes.c_void_p(self.ws.data_ptr()), ctypes.c_size_t(self.ws_bytes),
                                     ctypes.c_void_p(self._stream())), "tlora_layer_fwd")

    def bwd(self, dOut, dX, grads, flags: int = 0) -> None:
        J = len(self.ranks)
        VPP = ctypes.POINTER(ctypes.c_void_p)

        def arr(ts):
            return (ctypes.c_void_p * J)(*[ctypes.c_void_p(t.data_ptr()) if t.numel() else None for t in ts])
        da = [arr(grads[n][0]) for n in self.NAMES]
        db = [arr(grads[n][1]) for n in self.NAMES]
        dA = (VPP * 7)(*[ctypes.cast(a, VPP) for a in da])
        dB = (VPP * 7)(*[ctypes.cast(a, VPP) for a in db])
        _check(lib().tlora_layer_bwd(ctypes.byref(self.prob), ctypes.c_void_p(dOut.data_ptr()) if self.T else None,
                                     ctypes.c_void_p(dX.data_ptr()) if self.T else None, dA, dB, int(flags),
                                     ctypes.c_void_p(self.ws.data_ptr()), ctypes.c_size_t(self.ws_bytes),
                                     ctypes.c_void_p(self._stream())), "tlora_layer_bwd")


class Scheduler:
    """Argument marshalling for the host-side adapter scheduler (tlora_sched_*).  model = dict(tokens=[..], ms=[..],
    rho=ms per token and rank unit, kappa=ms per additional job); jobs = dicts with tokens, rank and optionally steps, urgency, max_slowdown."""

    def __init__(self, model, jobs):
        n = len(model["tokens"])
        self._x = (ctypes.c_double * n)(*[float(v) for v in model["tokens"]])
        self._y = (ctypes.c_double * n)(*[float(v) for v in model["ms"]])
        self.model = tlora_sched_model_t(n, self._x, self._y, float(model["rho"]), float(model.get("kappa", 0.0)))
        self.n = len(jobs)
        self.jobs = (tlora_sched_job_t * max(self.n, 1))(*[
            tlora_sched_job_t(int(j["tokens"]), int(j["rank"]), int(j.get("steps", 0)), float(j.get("urgency", 1.0)),
                              float(j.get("max_slowdown", 1e300))) for j in jobs])

    def step_ms(self, members) -> float:
        m = (ctypes.c_int32 * max(len(members), 1))(*[int(v) for v in members])
        out = ctypes.c_double(0.0)
        _check(lib().tlora_sched_step_ms(ctypes.byref(self.model), self.n, self.jobs, m, len(members), ctypes.byref(out)),
               "tlora_sched_step_ms")
        return float(out.value)

    def partition(self):
        """Groups in the order they were finalized, each a sorted list of job indices."""
        group_of = (ctypes.c_int32 * max(self.n, 1))()
        ng = ctypes.c_int32(0)
        _check(lib().tlora_sched_partition(ctypes.byref(self.model), self.n, self.jobs, group_of, ctypes.byref(ng)),
               "tlora_sched_partition")
        return [[j for j in range(self.n) if group_of[j] == g] for g in range(ng.value)]

    def simulate(self, horizon: int, trace_capacity: int = 4096):
        """(trace, jct, makespan): trace = [(group, steps)] of the first trace_capacity rounds."""
        jct = (ctypes.c_double * max(self.n, 1))()
        mk, nr = ctypes.c_double(0.0), ctypes.c_int64(0)
        tm = (ctypes.c_int32 * max(trace_capacity * self.n, 1))()
        tsz, tst = (ctypes.c_int32 * max(trace_capacity, 1))(), (ctypes.c_int32 * max(trace_capacity, 1))()
        _check(lib().tlora_sched_simulate(ctypes.byref(self.model), self.n, self.jobs, int(horizon), jct, ctypes.byref(mk),
                                          tm, tsz, tst, ctypes.byref(nr), trace_capacity), "tlora_sched_simulate")
        trace, at = [], 0
        for i in range(min(int(nr.value), trace_capacity)):
            trace.append(([int(tm[at + k]) for k in range(tsz[i])], int(tst[i])))
            at += tsz[i]
        return trace, [float(jct[j]) for j in range(self.n)], float(mk.value)
