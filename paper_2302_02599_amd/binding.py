"""ctypes binding of include/ckpt_dp.h.  Argument marshalling only.

PyTorch supplies device memory and the stream; no arithmetic of the method
happens in this file.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

CKPT_INF = 1 << 30
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libckpt_dp.so")
_lib = None


class CkptError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = load_library().ckpt_strerror(code).decode()
        extra = f" (hipError {load_library().ckpt_last_hip_error()})" if code == -5 else ""
        super().__init__(f"{where}: {msg}{extra} [{code}]")


class _Chains(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("uf", "ub", "wa", "wabar", "wdelta", "of", "ob")]


class _Op(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_uint8), ("stage", ctypes.c_uint8)]


class _SolveOpts(ctypes.Structure):
    _fields_ = [("groups", ctypes.c_int), ("side_streams", ctypes.c_void_p * 3), ("list_split", ctypes.c_int),
                ("row_launches", ctypes.c_int), ("stagger", ctypes.c_int), ("frontier", ctypes.c_int), ("spin_limit", ctypes.c_int),
                ("reserved", ctypes.c_int * 3)]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the in-tree HIP library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python paper_2302_02599_amd/build.py` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    # PyTorch ships its own HIP runtime and supplies the device memory and streams used here:
    # it has to be loaded first, so that this library binds to that runtime and not to a second one.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    sz, i, vp = ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p
    lib.ckpt_row_pitch.restype, lib.ckpt_row_pitch.argtypes = sz, [i]
    lib.ckpt_table_rows.restype, lib.ckpt_table_rows.argtypes = sz, [i]
    lib.ckpt_row_index.restype, lib.ckpt_row_index.argtypes = ctypes.c_long, [i, i, i]
    lib.ckpt_table_elems.restype, lib.ckpt_table_elems.argtypes = sz, [i, i, i]
    lib.ckpt_workspace_bytes.restype, lib.ckpt_workspace_bytes.argtypes = sz, [i, i, i]
    lib.ckpt_solve_batched.restype = i
    lib.ckpt_solve_batched.argtypes = [ctypes.POINTER(_Chains), i, i, i, vp, vp, vp, vp]
    lib.ckpt_init.restype, lib.ckpt_init.argtypes = i, [i]
    lib.ckpt_solve_batched_opts.restype = i
    lib.ckpt_solve_batched_opts.argtypes = [ctypes.POINTER(_Chains), i, i, i, vp, vp, vp, vp,
                                            ctypes.POINTER(_SolveOpts)]
    lib.ckpt_solve_batched_noalloc.restype = i
    lib.ckpt_solve_batched_noalloc.argtypes = [ctypes.POINTER(_Chains), i, i, i, vp, vp, vp]
    lib.ckpt_block_indices.restype = i
    lib.ckpt_block_indices.argtypes = [ctypes.POINTER(_Op), i, i, vp]
    lib.ckpt_block_indices_batched.restype = i
    lib.ckpt_block_indices_batched.argtypes = [vp, i, vp, i, i, vp, vp, vp]
    lib.ckpt_solve_profiled.restype = i
    lib.ckpt_solve_profiled.argtypes = [ctypes.POINTER(_Chains), i, i, i, vp, vp, vp, vp, vp, vp, vp]
    lib.ckpt_kernel_name.restype, lib.ckpt_kernel_name.argtypes = ctypes.c_char_p, [i]
    lib.ckpt_check_inputs.restype = i
    lib.ckpt_check_inputs.argtypes = [vp, i, i, i, vp, vp]
    lib.ckpt_schedule.restype = i
    lib.ckpt_schedule.argtypes = [vp, vp, vp, i, i, i, i, i, ctypes.POINTER(_Op), i]
    lib.ckpt_select_plan.restype = i
    lib.ckpt_select_plan.argtypes = [vp, i, i, i, vp, vp, vp]
    lib.ckpt_discretize.restype = i
    lib.ckpt_discretize.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, vp, ctypes.POINTER(_Chains)]
    lib.ckpt_budget_sweep.restype = i
    lib.ckpt_budget_sweep.argtypes = [ctypes.c_int64, i, i, i, vp]
    lib.ckpt_discretize_sweep.restype = i
    lib.ckpt_discretize_sweep.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int64, i, i, i, i, i, vp, vp,
                                          ctypes.POINTER(_Chains)]
    lib.ckpt_schedule_batched.restype = i
    lib.ckpt_schedule_batched.argtypes = [vp, vp, vp, i, i, i, vp, vp, vp, i, vp, vp]
    lib.ckpt_schedule_workspace_bytes.restype, lib.ckpt_schedule_workspace_bytes.argtypes = sz, [i, i]
    lib.ckpt_simulate_batched.restype = i
    lib.ckpt_simulate_batched.argtypes = [ctypes.POINTER(_Chains), i, i, vp, i, vp, vp, vp, vp, vp]
    lib.ckpt_linearize.restype = i
    lib.ckpt_linearize.argtypes = [i, vp, vp, vp, vp, vp]
    lib.ckpt_last_hip_error.restype, lib.ckpt_last_hip_error.argtypes = i, []
    lib.ckpt_strerror.restype, lib.ckpt_strerror.argtypes = ctypes.c_char_p, [i]
    _lib = lib
    return lib


def ckpt_row_pitch(M: int) -> int:
    return load_library().ckpt_row_pitch(M)


def ckpt_table_rows(L: int) -> int:
    return load_library().ckpt_table_rows(L)


def ckpt_row_index(L: int, s: int, t: int) -> int:
    return load_library().ckpt_row_index(L, s, t)


def ckpt_table_elems(L: int, M: int, B: int) -> int:
    return load_library().ckpt_table_elems(L, M, B)


def ckpt_workspace_bytes(L: int, M: int, B: int) -> int:
    return load_library().ckpt_workspace_bytes(L, M, B)


def _dev_ptr(t, name, shape):
    import torch
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous int32 device tensor")
    if tuple(t.shape) != shape:
        raise ValueError(f"{name}: shape {tuple(t.shape)} != {shape}")
    return t.data_ptr()


def _marshal(uf, ub, wa, wabar, L, M, B, cost, arg, workspace, wdelta, of, ob, stream):
    import torch
    ch = _Chains(_dev_ptr(uf, "uf", (B, L)), _dev_ptr(ub, "ub", (B, L)), _dev_ptr(wa, "wa", (B, L + 1)),
                 _dev_ptr(wabar, "wabar", (B, L)), _dev_ptr(wdelta, "wdelta", (B, L + 1)),
                 _dev_ptr(of, "of", (B, L)), _dev_ptr(ob, "ob", (B, L)))
    n = ckpt_table_elems(L, M, B)
    if n and (cost.numel() < n or arg.numel() < n or cost.dtype != torch.int32 or arg.dtype != torch.uint8):
        raise ValueError("cost/arg tables too small or of the wrong dtype")
    if n and workspace.numel() * workspace.element_size() < ckpt_workspace_bytes(L, M, B):
        raise ValueError("workspace too small")
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    return ch, ctypes.c_void_p(st)


def ckpt_solve_profiled(uf, ub, wa, wabar, L, M, B, cost, arg, workspace, *, wdelta=None, of=None, ob=None,
                        stream=None, count_bytes=False):
    """Same fill on one stream with per-kernel-kind timing; returns {kernel name: (total ms, launches)},
    with count_bytes {kernel name: (total ms, launches, bytes loaded, bytes stored)}.  Synchronises."""
    lib = load_library()
    ch, st = _marshal(uf, ub, wa, wabar, L, M, B, cost, arg, workspace, wdelta, of, ob, stream)
    n = 0
    while lib.ckpt_kernel_name(n) is not None:
        n += 1
    ms = (ctypes.c_float * n)()
    cnt = (ctypes.c_int * n)()
    nbytes = (ctypes.c_double * (2 * n))()
    rc = lib.ckpt_solve_profiled(ctypes.byref(ch), L, M, B, st, cost.data_ptr(), arg.data_ptr(),
                                 workspace.data_ptr(), ms, cnt, nbytes if count_bytes else None)
    if rc != 0:
        raise CkptError(rc, "ckpt_solve_profiled")
    if count_bytes:
        return {lib.ckpt_kernel_name(k).decode(): (float(ms[k]), int(cnt[k]), nbytes[2 * k], nbytes[2 * k + 1])
                for k in range(n)}
    return {lib.ckpt_kernel_name(k).decode(): (float(ms[k]), int(cnt[k])) for k in range(n)}


def ckpt_solve_batched(uf, ub, wa, wabar, L, M, B, cost, arg, workspace, *, wdelta=None, of=None, ob=None,
                       stream=None) -> None:
    """Enqueue the table fill on ``stream`` (default: torch's current stream).

    uf, ub, wabar, of, ob: int32 device tensors [B, L]; wa, wdelta: [B, L+1];
    cost: int32 device tensor of ckpt_table_elems elements; arg: uint8, same count;
    workspace: uint8 device tensor of at least ckpt_workspace_bytes bytes.
    """
    ch, st = _marshal(uf, ub, wa, wabar, L, M, B, cost, arg, workspace, wdelta, of, ob, stream)
    rc = load_library().ckpt_solve_batched(ctypes.byref(ch), L, M, B, st, cost.data_ptr(), arg.data_ptr(),
                                           workspace.data_ptr())
    if rc != 0:
        raise CkptError(rc, "ckpt_solve_batched")


def ckpt_init(device: int = -1) -> None:
    """Create the library's per-device helper streams and events (device < 0: the current one)."""
    rc = load_library().ckpt_init(device)
    if rc != 0:
        raise CkptError(rc, "ckpt_init")


def ckpt_solve_batched_opts(uf, ub, wa, wabar, L, M, B, cost, arg, workspace, *, groups=0, side_streams=None,
                            list_split=0, row_launches=0, stagger=0, frontier=0, spin_limit=0, wdelta=None, of=None, ob=None, stream=None) -> None:
    """ckpt_solve_batched with the schedule chosen by the caller: number of chain groups (1 = no
    helper streams), caller-owned side streams (raw hipStream_t values), waves per work list."""
    ch, st = _marshal(uf, ub, wa, wabar, L, M, B, cost, arg, workspace, wdelta, of, ob, stream)
    opts = _SolveOpts()
    opts.groups, opts.list_split, opts.row_launches, opts.stagger = groups, list_split, row_launches, stagger
    opts.frontier, opts.spin_limit = frontier, spin_limit
    for k, h in enumerate(side_streams or []):
        opts.side_streams[k] = h
    rc = load_library().ckpt_solve_batched_opts(ctypes.byref(ch), L, M, B, st, cost.data_ptr(), arg.data_ptr(),
                                                workspace.data_ptr(), ctypes.byref(opts))
    if rc != 0:
        raise CkptError(rc, "ckpt_solve_batched_opts")


def ckpt_solve_batched_noalloc(uf, ub, wa, wabar, L, M, B, cost, arg, *, wdelta=None, of=None, ob=None,
                               stream=None) -> None:
    """ckpt_solve_batched on the library's static per-GPU workspace: allocates nothing."""
    import torch
    ch = _Chains(_dev_ptr(uf, "uf", (B, L)), _dev_ptr(ub, "ub", (B, L)), _dev_ptr(wa, "wa", (B, L + 1)),
                 _dev_ptr(wabar, "wabar", (B, L)), _dev_ptr(wdelta, "wdelta", (B, L + 1)),
                 _dev_ptr(of, "of", (B, L)), _dev_ptr(ob, "ob", (B, L)))
    n = ckpt_table_elems(L, M, B)
    if n and (cost.numel() < n or arg.numel() < n or cost.dtype != torch.int32 or arg.dtype != torch.uint8):
        raise ValueError("cost/arg tables too small or of the wrong dtype")
    rc = load_library().ckpt_solve_batched_noalloc(ctypes.byref(ch), L, M, B, _stream(stream), cost.data_ptr(),
                                                   arg.data_ptr())
    if rc != 0:
        raise CkptError(rc, "ckpt_solve_batched_noalloc")


def ckpt_check_inputs(workspace, L, M, B, *, stream=None) -> np.ndarray:
    """Synchronise and return the per-chain input flags (all zero = fine); raises on nonzero.
    workspace None: the static workspace of ckpt_solve_batched_noalloc."""
    import torch
    flags = np.zeros(B, np.int32)
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    rc = load_library().ckpt_check_inputs(None if workspace is None else workspace.data_ptr(), L, M, B, ctypes.c_void_p(st),
                                          flags.ctypes.data)
    if rc not in (0, -6):
        raise CkptError(rc, "ckpt_check_inputs")
    return flags


def ckpt_schedule(arg_host: np.ndarray, wa: np.ndarray, wabar: np.ndarray, L: int, M: int, s: int, t: int,
                  m_budget: int, ops_cap: Optional[int] = None):
    """Operation list [(kind, stage), ...] of cell (s, t, m_budget) of one chain (host only)."""
    arg_host = np.ascontiguousarray(arg_host, dtype=np.uint8)
    wa = np.ascontiguousarray(wa, dtype=np.int32)
    wabar = np.ascontiguousarray(wabar, dtype=np.int32)
    if arg_host.size < ckpt_table_rows(L) * ckpt_row_pitch(M) or wa.size < L + 1 or wabar.size < L:
        raise ValueError("ckpt_schedule: array too small")
    cap = L * (L + 1) // 2 + L if ops_cap is None else ops_cap
    ops = (_Op * max(cap, 1))()
    rc = load_library().ckpt_schedule(arg_host.ctypes.data, wa.ctypes.data, wabar.ctypes.data, L, M, s, t,
                                      m_budget, ops, cap)
    if rc < 0:
        raise CkptError(rc, "ckpt_schedule")
    return [(ops[i].kind, ops[i].stage) for i in range(rc)]


def ckpt_block_indices(ops, L):
    """Host: checkpoint block index of every stage from a whole-chain operation list
    [(kind, stage), ...]; returns (list of L indices, number of blocks)."""
    arr = (_Op * max(len(ops), 1))()
    for k, (kind, stage) in enumerate(ops):
        arr[k].kind, arr[k].stage = kind, stage
    out = np.empty(max(L, 1), np.int32)
    rc = load_library().ckpt_block_indices(arr, len(ops), L, out.ctypes.data)
    if rc < 0:
        raise CkptError(rc, "ckpt_block_indices")
    return out[:L].tolist(), rc


def _stream(stream):
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream if stream is None else stream)


def _dev(t, name, dtype, numel):
    import torch
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous() and t.numel() >= numel):
        raise TypeError(f"{name}: expected a contiguous {dtype} device tensor of at least {numel} elements")
    return t.data_ptr()


def ckpt_select_plan(cost, L, M, B, m_budget, out, *, stream=None) -> None:
    """out[0] <- best chain (or -1), out[1] <- its cost.  All tensors on the device."""
    import torch
    rc = load_library().ckpt_select_plan(_dev(cost, "cost", torch.int32, ckpt_table_elems(L, M, B)), L, M, B,
                                         _dev(m_budget, "m_budget", torch.int32, B), _stream(stream),
                                         _dev(out, "out", torch.int32, 2))
    if rc != 0:
        raise CkptError(rc, "ckpt_select_plan")


def ckpt_discretize(bytes_wa, bytes_wabar, budget_bytes, L, M, B, wa, wabar, *, bytes_wdelta=None, bytes_of=None,
                    bytes_ob=None, wdelta=None, of=None, ob=None, stream=None) -> None:
    """int64 byte sizes [B, ...] -> int32 slot sizes, slots = ceil(bytes * M / budget_bytes[b])."""
    import torch
    i64, i32 = torch.int64, torch.int32
    outs = _Chains(None, None, _dev(wa, "wa", i32, B * (L + 1)), _dev(wabar, "wabar", i32, B * L),
                   _dev(wdelta, "wdelta", i32, B * (L + 1)), _dev(of, "of", i32, B * L), _dev(ob, "ob", i32, B * L))
    rc = load_library().ckpt_discretize(_dev(bytes_wa, "bytes_wa", i64, B * (L + 1)),
                                        _dev(bytes_wabar, "bytes_wabar", i64, B * L),
                                        _dev(bytes_wdelta, "bytes_wdelta", i64, B * (L + 1)),
                                        _dev(bytes_of, "bytes_of", i64, B * L), _dev(bytes_ob, "bytes_ob", i64, B * L),
                                        _dev(budget_bytes, "budget_bytes", i64, B), L, M, B, _stream(stream),
                                        ctypes.byref(outs))
    if rc != 0:
        raise CkptError(rc, "ckpt_discretize")


def ckpt_budget_sweep(base_budget: int, alpha_num: int, alpha_den: int, count: int) -> list:
    """Host: budgets floor(base * (1 + alpha_num/alpha_den)^n), n = 0..count-1."""
    out = np.zeros(max(count, 1), np.int64)
    rc = load_library().ckpt_budget_sweep(base_budget, alpha_num, alpha_den, count, out.ctypes.data)
    if rc != 0:
        raise CkptError(rc, "ckpt_budget_sweep")
    return out[:count].tolist()


def ckpt_discretize_sweep(bytes_wa, bytes_wabar, base_budget, alpha_num, alpha_den, count, L, M, wa, wabar, *,
                          bytes_wdelta=None, bytes_of=None, bytes_ob=None, wdelta=None, of=None, ob=None,
                          budgets_out=None, stream=None) -> None:
    """One profile (int64 byte sizes of one chain) -> int32 slot sizes of `count` chains, chain n under
    the n-th budget of the sweep."""
    import torch
    i64, i32 = torch.int64, torch.int32
    B = max(count, 0)
    outs = _Chains(None, None, _dev(wa, "wa", i32, B * (L + 1)), _dev(wabar, "wabar", i32, B * L),
                   _dev(wdelta, "wdelta", i32, B * (L + 1)), _dev(of, "of", i32, B * L), _dev(ob, "ob", i32, B * L))
    rc = load_library().ckpt_discretize_sweep(
        _dev(bytes_wa, "bytes_wa", i64, L + 1), _dev(bytes_wabar, "bytes_wabar", i64, L),
        _dev(bytes_wdelta, "bytes_wdelta", i64, L + 1), _dev(bytes_of, "bytes_of", i64, L),
        _dev(bytes_ob, "bytes_ob", i64, L), base_budget, alpha_num, alpha_den, count, L, M, _stream(stream),
        _dev(budgets_out, "budgets_out", i64, B), ctypes.byref(outs))
    if rc != 0:
        raise CkptError(rc, "ckpt_discretize_sweep")


def ckpt_schedule_workspace_bytes(L: int, B: int) -> int:
    return load_library().ckpt_schedule_workspace_bytes(L, B)


def ckpt_schedule_batched(arg, wa, wabar, L, M, B, m_budget, ops, ops_cap, n_ops, workspace, *, stream=None) -> None:
    """Device walk of every chain: ops uint8 [B, ops_cap, 2] (kind, stage), n_ops int32 [B]."""
    import torch
    rc = load_library().ckpt_schedule_batched(
        _dev(arg, "arg", torch.uint8, ckpt_table_elems(L, M, B)), _dev(wa, "wa", torch.int32, B * (L + 1)),
        _dev(wabar, "wabar", torch.int32, B * L), L, M, B, _dev(m_budget, "m_budget", torch.int32, B), _stream(stream),
        _dev(ops, "ops", torch.uint8, B * ops_cap * 2), ops_cap, _dev(n_ops, "n_ops", torch.int32, B),
        _dev(workspace, "workspace", torch.uint8, ckpt_schedule_workspace_bytes(L, B)))
    if rc != 0:
        raise CkptError(rc, "ckpt_schedule_batched")


def ckpt_block_indices_batched(ops, ops_cap, n_ops, L, B, block_of_stage, n_blocks, *, stream=None) -> None:
    """Device: block_of_stage int32 [B, L], n_blocks int32 [B] from the lists of ckpt_schedule_batched."""
    import torch
    rc = load_library().ckpt_block_indices_batched(
        _dev(ops, "ops", torch.uint8, B * ops_cap * 2), ops_cap, _dev(n_ops, "n_ops", torch.int32, B), L, B,
        _stream(stream), _dev(block_of_stage, "block_of_stage", torch.int32, B * L),
        _dev(n_blocks, "n_blocks", torch.int32, B))
    if rc != 0:
        raise CkptError(rc, "ckpt_block_indices_batched")


def ckpt_simulate_batched(uf, ub, wa, wabar, L, B, ops, ops_cap, n_ops, time_out, peak_out, status, *, wdelta=None,
                          of=None, ob=None, stream=None) -> None:
    """Device execution of every chain's operation list under the memory model of Table 1:
    time_out / peak_out int64 [B], status int32 [B]."""
    import torch
    i32 = torch.int32
    chains = _Chains(_dev(uf, "uf", i32, B * L), _dev(ub, "ub", i32, B * L), _dev(wa, "wa", i32, B * (L + 1)),
                     _dev(wabar, "wabar", i32, B * L), _dev(wdelta, "wdelta", i32, B * (L + 1)),
                     _dev(of, "of", i32, B * L), _dev(ob, "ob", i32, B * L))
    rc = load_library().ckpt_simulate_batched(
        ctypes.byref(chains), L, B, _dev(ops, "ops", torch.uint8, B * ops_cap * 2), ops_cap,
        _dev(n_ops, "n_ops", i32, B), _stream(stream), _dev(time_out, "time_out", torch.int64, B),
        _dev(peak_out, "peak_out", torch.int64, B), _dev(status, "status", i32, B))
    if rc != 0:
        raise CkptError(rc, "ckpt_simulate_batched")


def ckpt_linearize(children, flags):
    """Host linearisation of a DAG given as per-node child lists in topological order.
    Returns (group index per node, common flag per node, number of groups)."""
    n = len(children)
    ptr = np.zeros(n + 1, np.int32)
    ptr[1:] = np.cumsum([len(c) for c in children])
    idx = np.array([c for cs in children for c in cs], np.int32)
    fl = np.ascontiguousarray(flags, dtype=np.uint8)
    group = np.empty(max(n, 1), np.int32)
    common = np.empty(max(n, 1), np.uint8)
    rc = load_library().ckpt_linearize(n, ptr.ctypes.data, idx.ctypes.data if idx.size else None, fl.ctypes.data,
                                       group.ctypes.data, common.ctypes.data)
    if rc < 0:
        raise CkptError(rc, "ckpt_linearize")
    return group[:n].tolist(), [bool(c) for c in common[:n]], rc


@dataclass
class Solution:
    """Device tables of one solve, with the logical [B, rows, pitch] views."""
    L: int
    M: int
    B: int
    cost: "object"      # int32 [B, rows, pitch] device tensor
    arg: "object"       # uint8 [B, rows, pitch] device tensor
    workspace: "object"


def solve(batch, device="cuda:0", check=True, **opts) -> Solution:
    """Convenience wrapper: upload a workloads.ChainBatch-like object, allocate tables, solve.
    Keyword options (groups, side_streams, list_split) go to ckpt_solve_batched_opts."""
    import torch
    dev = torch.device(device)
    L, M, B = batch.L, batch.M, batch.B

    def up(a):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)

    rows, pitch = ckpt_table_rows(L), ckpt_row_pitch(M)
    with torch.cuda.device(dev):
        cost = torch.empty((B, rows, pitch), dtype=torch.int32, device=dev)
        arg = torch.empty((B, rows, pitch), dtype=torch.uint8, device=dev)
        ws = torch.empty(ckpt_workspace_bytes(L, M, B), dtype=torch.uint8, device=dev)
        fill = ckpt_solve_batched_opts if opts else ckpt_solve_batched
        fill(up(batch.uf), up(batch.ub), up(batch.wa), up(batch.wabar), L, M, B, cost, arg, ws,
             wdelta=up(batch.wdelta), of=up(batch.of), ob=up(batch.ob), **opts)
        if check:
            flags = ckpt_check_inputs(ws, L, M, B)
            if flags.any():
                raise CkptError(-6, f"solve (flags {flags.tolist()})")
    return Solution(L, M, B, cost, arg, ws)
