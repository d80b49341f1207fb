"""ctypes binding of libvarlen_attn.so (argument marshalling only).

Function names and argument order follow include/varlen_attn.h.  Tensor arguments may be
torch tensors (their ``data_ptr()`` is passed) or raw integer device addresses.  PyTorch is
used by callers for device memory and streams; no arithmetic happens on this side, and
there is no fallback: a missing library is an ImportError-like failure at first use.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libvarlen_attn.so")
BENCH_LIB_PATH = os.path.join(HERE, "libvarlen_attn_bench.so")   # measurement probes, bench.py only

TILE_ROWS = 128
STEP_ROWS = 64
OK = 0
INVALID_ARG = -1
UNSUPPORTED = -2
WORKSPACE_TOO_SMALL = -3
LAUNCH_FAILED = -4
BAD_CU_SEQLENS = -5
PLAN_OVERFLOW = -6
STATIC_TOO_LARGE = -7
STATIC_SCRATCH_BYTES = 40 << 20
FLAG_REUSE_PLAN = 1
FLAG_NO_SPLIT = 2
FLAG_PLAN_LARGE = 8
FLAG_FUSED_BWD = 16
FLAG_PLAN_FIRST = 32


def flag_group_heads(n: int) -> int:
    """VARLEN_ATTN_FLAG_GROUP_HEADS(n): q heads per column unit under GQA (0 = plan decides)."""
    return (int(n) & 0xF) << 24


def flag_chunk_steps(row: int, col: int) -> int:
    """VARLEN_ATTN_FLAG_CHUNK_STEPS(row, col): longest chunk of a row / column chain (0 = plan decides)."""
    return ((int(row) & 0xFF) << 8) | ((int(col) & 0xFF) << 16)


class Params(ctypes.Structure):
    _fields_ = [("total_tokens", ctypes.c_int32), ("num_docs", ctypes.c_int32),
                ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("flags", ctypes.c_int32)]


class PlanHeader(ctypes.Structure):
    _fields_ = [("status", ctypes.c_int32), ("n_row_units", ctypes.c_int32),
                ("n_col_units", ctypes.c_int32), ("n_row_combine", ctypes.c_int32),
                ("n_col_combine", ctypes.c_int32), ("row_chunk_steps", ctypes.c_int32),
                ("col_chunk_steps", ctypes.c_int32), ("n_row_slots", ctypes.c_int32),
                ("n_col_slots", ctypes.c_int32), ("row_class_shift", ctypes.c_int32),
                ("col_heads_per_unit", ctypes.c_int32), ("col_class_shift", ctypes.c_int32),
                ("reserved", ctypes.c_int32 * 2),
                ("pairs", ctypes.c_int64)]


class Unit(ctypes.Structure):
    _fields_ = [("row0", ctypes.c_int32), ("doc_start", ctypes.c_int32),
                ("doc_end", ctypes.c_int32), ("step_begin", ctypes.c_int32),
                ("step_end", ctypes.c_int32), ("slot", ctypes.c_int32),
                ("cost", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class CombineItem(ctypes.Structure):
    _fields_ = [("row0", ctypes.c_int32), ("doc_end", ctypes.c_int32),
                ("slot0", ctypes.c_int32), ("n_chunks", ctypes.c_int32)]


class WorkspaceLayout(ctypes.Structure):
    _fields_ = [("row_units_offset", ctypes.c_size_t), ("col_units_offset", ctypes.c_size_t),
                ("row_combine_offset", ctypes.c_size_t), ("col_combine_offset", ctypes.c_size_t),
                ("dsum_offset", ctypes.c_size_t), ("row_partials_offset", ctypes.c_size_t),
                ("col_partials_offset", ctypes.c_size_t), ("dq_accumulator_offset", ctypes.c_size_t),
                ("total_bytes", ctypes.c_size_t),
                ("max_units", ctypes.c_int32), ("max_combine", ctypes.c_int32),
                ("max_row_slots", ctypes.c_int32), ("max_col_slots", ctypes.c_int32)]


class KernelTime(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("launches", ctypes.c_int32),
                ("total_ms", ctypes.c_float)]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2605_06374_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, pp = ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(Params)
        L.varlen_attn_workspace_bytes.restype = sz
        L.varlen_attn_workspace_bytes.argtypes = [pp]
        L.varlen_attn_workspace_regions.restype = ctypes.c_int
        L.varlen_attn_workspace_regions.argtypes = [pp, ctypes.POINTER(WorkspaceLayout)]
        L.varlen_attn_plan.restype = ctypes.c_int
        L.varlen_attn_plan.argtypes = [pp, vp, vp, sz, vp]
        L.varlen_attn_fwd.restype = ctypes.c_int
        L.varlen_attn_fwd.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.varlen_attn_fwd_static.restype = ctypes.c_int
        L.varlen_attn_fwd_static.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.varlen_attn_bwd.restype = ctypes.c_int
        L.varlen_attn_bwd.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.varlen_attn_check.restype = ctypes.c_int
        L.varlen_attn_check.argtypes = [vp, vp]
        L.varlen_attn_status_string.restype = ctypes.c_char_p
        L.varlen_attn_status_string.argtypes = [ctypes.c_int]
        L.varlen_attn_profile.restype = ctypes.c_int
        L.varlen_attn_profile.argtypes = [ctypes.c_int]
        L.varlen_attn_profile_read.restype = ctypes.c_int
        L.varlen_attn_profile_read.argtypes = [ctypes.POINTER(KernelTime), ctypes.c_int]
        _lib = L
    return _lib


_bench_lib = None


def bench_lib() -> ctypes.CDLL:
    """libvarlen_attn_bench.so (include/varlen_attn_bench.h): rate probes for benchmarks."""
    global _bench_lib
    if _bench_lib is None:
        if not os.path.exists(BENCH_LIB_PATH):
            raise RuntimeError(f"{BENCH_LIB_PATH} is missing: build it with "
                               "`python -m paper_2605_06374_amd.build`")
        L = ctypes.CDLL(BENCH_LIB_PATH)
        vp = ctypes.c_void_p
        for name in ("varlen_attn_bench_mfma_rate", "varlen_attn_bench_lds_rate"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [ctypes.c_int, ctypes.c_int, vp, vp,
                                         ctypes.POINTER(ctypes.c_float)]
        L.varlen_attn_bench_overlap.restype = ctypes.c_int
        L.varlen_attn_bench_overlap.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp,
                                                ctypes.POINTER(ctypes.c_float)]
        L.varlen_attn_bench_atomic_rate.restype = ctypes.c_int
        L.varlen_attn_bench_atomic_rate.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                    vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_float)]
        L.varlen_attn_bench_copy.restype = ctypes.c_int
        L.varlen_attn_bench_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        _bench_lib = L
    return _bench_lib


def make_params(total_tokens, num_docs, num_q_heads, num_kv_heads, head_dim, softmax_scale,
                flags=0) -> Params:
    return Params(int(total_tokens), int(num_docs), int(num_q_heads), int(num_kv_heads),
                  int(head_dim), float(softmax_scale), int(flags))


def _addr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _nbytes(x, given) -> int:
    if given is not None:
        return int(given)
    return int(x.numel() * x.element_size())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def varlen_attn_workspace_bytes(params: Params) -> int:
    return int(lib().varlen_attn_workspace_bytes(ctypes.byref(params)))


def varlen_attn_workspace_regions(params: Params) -> WorkspaceLayout:
    out = WorkspaceLayout()
    check(int(lib().varlen_attn_workspace_regions(ctypes.byref(params), ctypes.byref(out))))
    return out


def varlen_attn_plan(params, cu_seqlens, workspace, workspace_bytes=None, stream=None) -> int:
    return int(lib().varlen_attn_plan(ctypes.byref(params), _addr(cu_seqlens), _addr(workspace),
                                      _nbytes(workspace, workspace_bytes), _stream(stream)))


def varlen_attn_fwd(params, q, k, v, cu_seqlens, o, lse, workspace, workspace_bytes=None,
                    stream=None) -> int:
    return int(lib().varlen_attn_fwd(ctypes.byref(params), _addr(q), _addr(k), _addr(v),
                                     _addr(cu_seqlens), _addr(o), _addr(lse), _addr(workspace),
                                     _nbytes(workspace, workspace_bytes), _stream(stream)))


def varlen_attn_fwd_static(params, q, k, v, cu_seqlens, o, lse, plan_status=None, stream=None) -> int:
    return int(lib().varlen_attn_fwd_static(ctypes.byref(params), _addr(q), _addr(k), _addr(v),
                                            _addr(cu_seqlens), _addr(o), _addr(lse),
                                            _addr(plan_status), _stream(stream)))


def varlen_attn_bwd(params, q, k, v, o, lse, d_o, cu_seqlens, dq, dk, dv, workspace,
                    workspace_bytes=None, stream=None) -> int:
    return int(lib().varlen_attn_bwd(ctypes.byref(params), _addr(q), _addr(k), _addr(v), _addr(o),
                                     _addr(lse), _addr(d_o), _addr(cu_seqlens), _addr(dq),
                                     _addr(dk), _addr(dv), _addr(workspace),
                                     _nbytes(workspace, workspace_bytes), _stream(stream)))


def varlen_attn_check(workspace, stream=None) -> int:
    return int(lib().varlen_attn_check(_addr(workspace), _stream(stream)))


def varlen_attn_profile(enable: bool) -> int:
    return int(lib().varlen_attn_profile(1 if enable else 0))


def varlen_attn_profile_read():
    """{kernel name: (launches, total_ms)} of the launches recorded since profiling was enabled."""
    buf = (KernelTime * 16)()
    n = int(lib().varlen_attn_profile_read(buf, 16))
    check(min(n, 0))
    return {buf[i].name.decode(): (int(buf[i].launches), float(buf[i].total_ms)) for i in range(n)}


def varlen_attn_bench_mfma_rate(random_operands: bool, iterations: int, device_scratch, stream=None) -> float:
    """TFLOP/s of a pure bf16 MFMA 32x32x16 kernel (see the header); blocks the host."""
    out = ctypes.c_float(0.0)
    check(bench_lib().varlen_attn_bench_mfma_rate(int(bool(random_operands)), int(iterations),
                                      ctypes.c_void_p(int(device_scratch)),
                                      ctypes.c_void_p(int(stream or 0)), ctypes.byref(out)))
    return float(out.value)


def varlen_attn_bench_lds_rate(transposed: bool, iterations: int, device_scratch, stream=None) -> float:
    """LDS fragment-read rate in bytes per nominal clock per CU (see the header); blocks the host."""
    out = ctypes.c_float(0.0)
    check(bench_lib().varlen_attn_bench_lds_rate(int(bool(transposed)), int(iterations),
                                     ctypes.c_void_p(int(device_scratch)),
                                     ctypes.c_void_p(int(stream or 0)), ctypes.byref(out)))
    return float(out.value)


def varlen_attn_bench_overlap(work_a: int, work_b: int, iterations: int, scratch_ptr: int, stream=None) -> float:
    """Nominal clocks per iteration of the matrix / vector overlap probe; see the bench header."""
    out = ctypes.c_float(0.0)
    check(bench_lib().varlen_attn_bench_overlap(int(work_a), int(work_b), int(iterations),
                                                ctypes.c_void_p(int(scratch_ptr)), _stream(stream),
                                                ctypes.byref(out)))
    return float(out.value)


def varlen_attn_bench_atomic_rate(mode: int, stages: int, regions: int, stride: int, buffer, stream=None) -> float:
    """GB/s of fp32 atomic adds (mode 0) or plain stores (mode 1); see the bench header."""
    out = ctypes.c_float(0.0)
    check(bench_lib().varlen_attn_bench_atomic_rate(int(mode), int(stages), int(regions), int(stride),
                                                    _addr(buffer), _nbytes(buffer, None), _stream(stream),
                                                    ctypes.byref(out)))
    return float(out.value)


def varlen_attn_bench_copy(src, dst, nbytes: int, stream=None) -> None:
    """Plain device copy of known size (kernel bench_copy_kernel); see the bench header."""
    check(bench_lib().varlen_attn_bench_copy(_addr(src), _addr(dst), int(nbytes), _stream(stream)))


def varlen_attn_status_string(status: int) -> str:
    return lib().varlen_attn_status_string(int(status)).decode()


def check(status: int) -> None:
    if status != OK:
        raise RuntimeError(f"varlen_attn: {varlen_attn_status_string(status)} ({status})")
