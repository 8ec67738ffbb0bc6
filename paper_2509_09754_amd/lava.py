"""ctypes binding over liblava.so: the same entry points as include/lava.h, taking torch tensors.

Argument marshalling only — every step of the path runs in the HIP kernels.  PyTorch supplies
device memory and the current stream.  If the library has not been built the import fails
loudly; there is no fallback implementation.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# LAVA_LIBRARY names another build of the same library (the host-sanitizer build of build.py --sanitize);
# it is read by this binding only, never by the library itself
LIB_PATH = os.environ.get("LAVA_LIBRARY") or os.path.join(_HERE, "liblava.so")

LAVA_OK, LAVA_ERR_INVALID_ARG, LAVA_ERR_SHAPE, LAVA_ERR_BUDGET, LAVA_ERR_WORKSPACE, LAVA_ERR_HIP = range(6)
LAVA_F32, LAVA_BF16 = 0, 1
LAVA_SCORE_LAVA, LAVA_SCORE_ATTENTION, LAVA_SCORE_TOKEN_NORM = 0, 1, 2

EXPORTS = [
    "lava_status_string", "lava_set_tuning", "lava_get_tuning", "lava_window_scores_workspace_bytes", "lava_window_scores",
    "lava_window_scores_primed", "lava_select_topk_primed", "lava_window_scores_planned",
    "lava_layer_budgets", "lava_select_workspace_bytes", "lava_select_topk", "lava_select_status",
    "lava_select_topk_static",
    "lava_select_batch_workspace_bytes", "lava_select_topk_batch", "lava_select_batch_status",
    "lava_compact_kv", "lava_compact_packed", "lava_compact_batch",
    "lava_cascade_workspace_bytes", "lava_cascade_step",
    "lava_decode_workspace_bytes", "lava_decode_attention",
    "lava_prof_kernel_count", "lava_prof_kernel_name", "lava_prof_enable", "lava_prof_reset",
    "lava_prof_read", "lava_probe_stream",
]


class LayerDesc(ctypes.Structure):
    """Mirror of lava_layer_desc."""
    _fields_ = [
        ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("window", ctypes.c_int32), ("pool_kernel", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float), ("score_kind", ctypes.c_int32),
    ]

    @classmethod
    def make(cls, n_q_heads, n_kv_heads, head_dim, window, dtype, pool_kernel=7, softmax_scale=0.0,
             score_kind=LAVA_SCORE_LAVA):
        code = {"f32": LAVA_F32, "bf16": LAVA_BF16, LAVA_F32: LAVA_F32, LAVA_BF16: LAVA_BF16}[dtype]
        return cls(n_q_heads, n_kv_heads, head_dim, window, pool_kernel, code, softmax_scale, score_kind)

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == LAVA_BF16 else torch.float32


class Tuning(ctypes.Structure):
    """Mirror of lava_tuning (zero = the library's own choice)."""
    _fields_ = [
        ("sweep_shape", ctypes.c_int32), ("sweep_workgroups", ctypes.c_int32), ("sweep_schedule", ctypes.c_int32),
        ("decode_rows_per_unit", ctypes.c_int32), ("barrier_spin_limit", ctypes.c_int32),
        ("sweep_orphan_units", ctypes.c_int32), ("reserved", ctypes.c_int32 * 2),
    ]


class BudgetPlan(ctypes.Structure):
    """Mirror of lava_budget_plan (device pointers; see make_budget_plan)."""
    _fields_ = [("n_layers", ctypes.c_int32), ("layer", ctypes.c_int32), ("e", ctypes.c_void_p),
                ("total", ctypes.c_void_p), ("lo", ctypes.c_void_p), ("hi", ctypes.c_void_p),
                ("budgets", ctypes.c_void_p)]


LAVA_PLAN_MAX_LAYERS = 128
SWEEP_SHAPES = {"auto": 0, "wide": 1, "narrow": 2}
SWEEP_SCHEDULES = {"auto": 0, "separate": 1, "persistent": 2, "prepass": 3}


class LavaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2509_09754_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    dp = ctypes.POINTER(LayerDesc)
    lib.lava_status_string.restype = ctypes.c_char_p
    lib.lava_status_string.argtypes = [i32]
    lib.lava_set_tuning.restype = i32
    lib.lava_set_tuning.argtypes = [ctypes.POINTER(Tuning)]
    lib.lava_get_tuning.restype = i32
    lib.lava_get_tuning.argtypes = [ctypes.POINTER(Tuning)]
    lib.lava_window_scores_workspace_bytes.restype = sz
    lib.lava_window_scores_workspace_bytes.argtypes = [dp, i32, i64]
    lib.lava_window_scores.restype = i32
    lib.lava_window_scores.argtypes = [dp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lava_window_scores_primed.restype = i32
    lib.lava_window_scores_primed.argtypes = [dp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, sz, vp]
    lib.lava_window_scores_planned.restype = i32
    lib.lava_window_scores_planned.argtypes = [dp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, sz, vp, vp]
    lib.lava_select_topk_primed.restype = i32
    lib.lava_select_topk_primed.argtypes = [i32, vp, i64, i64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lava_layer_budgets.restype = i32
    lib.lava_layer_budgets.argtypes = [i32, i32, vp, vp, vp, vp, vp, i32, vp]
    lib.lava_select_workspace_bytes.restype = sz
    lib.lava_select_workspace_bytes.argtypes = [i64]
    lib.lava_select_topk.restype = i32
    lib.lava_select_topk.argtypes = [i32, vp, vp, i64, i64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lava_select_topk_static.restype = i32
    lib.lava_select_topk_static.argtypes = [i32, vp, vp, i64, i64, vp, vp, vp, vp, vp, vp]
    lib.lava_select_status.restype = i32
    lib.lava_select_status.argtypes = [vp, i64, vp]
    lib.lava_compact_kv.restype = i32
    lib.lava_compact_kv.argtypes = [dp, i64, vp, vp, vp, vp, i64, vp, vp, vp]
    lib.lava_compact_packed.restype = i32
    lib.lava_compact_packed.argtypes = [dp, vp, i64, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp]
    lib.lava_cascade_workspace_bytes.restype = sz
    lib.lava_cascade_workspace_bytes.argtypes = [dp, i64, i32, i64]
    lib.lava_select_batch_workspace_bytes.restype = sz
    lib.lava_select_batch_workspace_bytes.argtypes = [i32, i64]
    lib.lava_select_topk_batch.restype = i32
    lib.lava_select_topk_batch.argtypes = [i32, i32, vp, i64, vp, sz, vp]
    lib.lava_select_batch_status.restype = i32
    lib.lava_select_batch_status.argtypes = [vp, i32, i64, vp]
    lib.lava_compact_batch.restype = i32
    lib.lava_compact_batch.argtypes = [dp, i32, vp, vp]
    lib.lava_cascade_step.restype = i32
    lib.lava_cascade_step.argtypes = [dp, i32, i64, vp, vp, vp, vp, i64, vp, vp, vp, sz, vp]
    lib.lava_decode_workspace_bytes.restype = sz
    lib.lava_decode_workspace_bytes.argtypes = [dp, i32, i64, i64]
    lib.lava_decode_attention.restype = i32
    lib.lava_decode_attention.argtypes = [dp, i32, vp, vp, vp, vp, vp, i64, vp, vp, i64, i64, vp, vp, vp, sz, vp]
    lib.lava_prof_kernel_count.restype = i32
    lib.lava_prof_kernel_name.restype = ctypes.c_char_p
    lib.lava_prof_kernel_name.argtypes = [i32]
    lib.lava_prof_enable.restype = i32
    lib.lava_prof_enable.argtypes = [i32]
    lib.lava_prof_reset.restype = i32
    lib.lava_prof_read.restype = i32
    lib.lava_prof_read.argtypes = [i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.lava_probe_stream.restype = i32
    lib.lava_probe_stream.argtypes = [vp, vp, i64, i32, i32, vp]
    return lib


lib = _load()


def status_string(status: int) -> str:
    return lib.lava_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != LAVA_OK:
        raise LavaError(status, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev(t: torch.Tensor, name: str, dtype=None) -> torch.Tensor:
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}")
    return t


def to_device(arr: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """Upload a stored array from the generator (float32, or uint16 bf16 bit patterns)."""
    if dtype in ("bf16", LAVA_BF16):
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to(device)


def to_host_bits(t: torch.Tensor) -> np.ndarray:
    """Download rows bit for bit (bf16 as uint16 patterns, f32 as float32)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


# ------------------------------------------------------------------------------ entry points
def set_tuning(sweep_shape="auto", sweep_workgroups=0, sweep_schedule="auto", decode_rows_per_unit=0,
               barrier_spin_limit=0, sweep_orphan_units=0) -> None:
    """lava_set_tuning; called without arguments it restores the library's own choices."""
    t = Tuning(SWEEP_SHAPES[sweep_shape], int(sweep_workgroups), SWEEP_SCHEDULES[sweep_schedule],
               int(decode_rows_per_unit), int(barrier_spin_limit), int(sweep_orphan_units))
    _check(lib.lava_set_tuning(ctypes.byref(t)), "lava_set_tuning")


def get_tuning() -> Tuning:
    t = Tuning()
    _check(lib.lava_get_tuning(ctypes.byref(t)), "lava_get_tuning")
    return t


def lava_window_scores_workspace_bytes(desc: LayerDesc, batch: int, total_tokens: int) -> int:
    return int(lib.lava_window_scores_workspace_bytes(ctypes.byref(desc), batch, total_tokens))


def lava_window_scores(desc: LayerDesc, seq_lens: Sequence[int], q_win: torch.Tensor, k: torch.Tensor,
                       v: torch.Tensor, lse: Optional[torch.Tensor] = None, scores=None, vbar=None,
                       layer_stat=None, workspace=None, stream=None, select_workspace=None, budget_plan=None):
    """Scores [sum_b H_kv * N_b] (per sequence [H_kv][N_b]), vbar [batch, H_kv], layer_stat [batch].
    With select_workspace the call is lava_window_scores_primed; with budget_plan (see make_budget_plan)
    it is lava_window_scores_planned, which also accepts select_workspace."""
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int64))
    batch, total = int(lens.shape[0]), int(lens.sum())
    dev = k.device
    _dev(q_win, "q_win", desc.torch_dtype), _dev(k, "k", desc.torch_dtype), _dev(v, "v", desc.torch_dtype)
    row = desc.n_kv_heads * desc.head_dim
    if k.numel() != total * row or v.numel() != total * row:
        raise ValueError("k / v hold a different number of tokens than seq_lens")
    if q_win.numel() != batch * desc.n_q_heads * desc.window * desc.head_dim:
        raise ValueError("q_win must be [batch, H, w, d_h]")
    if lse is not None:
        _dev(lse, "lse", torch.float32)
        if lse.numel() != batch * desc.n_q_heads * desc.window:
            raise ValueError("lse must be [batch, H, w]")
    if scores is None:
        scores = torch.empty(total * desc.n_kv_heads, dtype=torch.float32, device=dev)
    if vbar is None:
        vbar = torch.empty(batch, desc.n_kv_heads, dtype=torch.float32, device=dev)
    if layer_stat is None:
        layer_stat = torch.empty(batch, dtype=torch.float32, device=dev)
    if workspace is None:
        nbytes = lava_window_scores_workspace_bytes(desc, batch, total)
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    if budget_plan is not None:
        st = lib.lava_window_scores_planned(ctypes.byref(desc), batch, lens.ctypes.data_as(ctypes.c_void_p), _ptr(q_win),
                                            _ptr(k), _ptr(v), _ptr(lse), _ptr(scores), _ptr(vbar), _ptr(layer_stat),
                                            _ptr(workspace), workspace.numel(), _ptr(select_workspace),
                                            select_workspace.numel() if select_workspace is not None else 0,
                                            ctypes.byref(budget_plan), _stream(stream))
        _check(st, "lava_window_scores_planned")
        return scores, vbar, layer_stat
    if select_workspace is not None:
        st = lib.lava_window_scores_primed(ctypes.byref(desc), batch, lens.ctypes.data_as(ctypes.c_void_p), _ptr(q_win),
                                           _ptr(k), _ptr(v), _ptr(lse), _ptr(scores), _ptr(vbar), _ptr(layer_stat),
                                           _ptr(workspace), workspace.numel(), _ptr(select_workspace),
                                           select_workspace.numel(), _stream(stream))
        _check(st, "lava_window_scores_primed")
        return scores, vbar, layer_stat
    st = lib.lava_window_scores(ctypes.byref(desc), batch, lens.ctypes.data_as(ctypes.c_void_p), _ptr(q_win),
                                _ptr(k), _ptr(v), _ptr(lse), _ptr(scores), _ptr(vbar), _ptr(layer_stat),
                                _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, "lava_window_scores")
    return scores, vbar, layer_stat


def make_budget_plan(e: torch.Tensor, layer: int, total: torch.Tensor, lo: torch.Tensor, hi: torch.Tensor,
                     budgets: torch.Tensor) -> "BudgetPlan":
    """lava_budget_plan over device tensors e [batch, L] float32 (column `layer` is written by the scores
    call), total [batch], lo / hi / budgets [batch, L] int64.  The plan holds pointers only: keep the tensors."""
    batch, L = e.shape
    for name, t, dt in (("e", e, torch.float32), ("total", total, torch.int64), ("lo", lo, torch.int64),
                        ("hi", hi, torch.int64), ("budgets", budgets, torch.int64)):
        _dev(t, name, dt)
    if total.numel() != batch or lo.numel() != batch * L or hi.numel() != batch * L or budgets.numel() != batch * L:
        raise ValueError("budget plan tables must be [batch] / [batch, L]")
    return BudgetPlan(L, int(layer), e.data_ptr(), total.data_ptr(), lo.data_ptr(), hi.data_ptr(), budgets.data_ptr())


def lava_layer_budgets(e, total, lo, hi, budgets=None, stream=None):
    """e [batch, L] float32; total [batch], lo / hi [batch, L] int64.  All numpy (host path) or all
    device tensors (device path)."""
    on_device = isinstance(e, torch.Tensor) and e.is_cuda
    if on_device:
        batch, L = e.shape
        for name, t, dt in (("e", e, torch.float32), ("total", total, torch.int64), ("lo", lo, torch.int64),
                            ("hi", hi, torch.int64)):
            _dev(t, name, dt)
        if budgets is None:
            budgets = torch.empty(batch, L, dtype=torch.int64, device=e.device)
        st = lib.lava_layer_budgets(batch, L, _ptr(e), _ptr(total), _ptr(lo), _ptr(hi), _ptr(budgets), 1,
                                    _stream(stream))
        _check(st, "lava_layer_budgets")
        return budgets
    e = np.ascontiguousarray(np.asarray(e, dtype=np.float32))
    if e.ndim == 1:
        e = e[None, :]
    batch, L = e.shape
    total = np.ascontiguousarray(np.asarray(total, dtype=np.int64).reshape(batch))
    lo = np.ascontiguousarray(np.broadcast_to(np.asarray(lo, dtype=np.int64), (batch, L)))
    hi = np.ascontiguousarray(np.broadcast_to(np.asarray(hi, dtype=np.int64), (batch, L)))
    out = np.zeros((batch, L), dtype=np.int64)
    as_vp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    st = lib.lava_layer_budgets(batch, L, as_vp(e), as_vp(total), as_vp(lo), as_vp(hi), as_vp(out), 0, None)
    _check(st, "lava_layer_budgets")
    return out


def lava_select_workspace_bytes(total_entries: int) -> int:
    return int(lib.lava_select_workspace_bytes(total_entries))


def lava_select_topk(n_heads: int, scores: torch.Tensor, budget: int, seg_offsets: Optional[torch.Tensor] = None,
                     budget_dev: Optional[torch.Tensor] = None, total_entries: Optional[int] = None,
                     head_counts=None, head_offsets=None, kept_idx=None, kept_scores=None,
                     want_scores: bool = True, workspace=None, stream=None, primed: bool = False):
    """primed: `workspace` was prepared by lava_window_scores(select_workspace=workspace) for these scores."""
    _dev(scores, "scores", torch.float32)
    total = scores.numel() if total_entries is None else int(total_entries)
    dev = scores.device
    if seg_offsets is not None:
        _dev(seg_offsets, "seg_offsets", torch.int64)
    if budget_dev is not None:
        _dev(budget_dev, "budget_dev", torch.int64)
    if head_counts is None:
        head_counts = torch.empty(n_heads, dtype=torch.int32, device=dev)
    if head_offsets is None:
        head_offsets = torch.empty(n_heads + 1, dtype=torch.int64, device=dev)
    if kept_idx is None:
        kept_idx = torch.empty(max(int(budget), 1), dtype=torch.int32, device=dev)
    if kept_scores is None and want_scores:
        kept_scores = torch.empty(max(int(budget), 1), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(lava_select_workspace_bytes(total), 256), dtype=torch.uint8, device=dev)
    if primed:
        if seg_offsets is not None:
            raise ValueError("a prepared workspace serves equal segments only")
        st = lib.lava_select_topk_primed(n_heads, _ptr(scores), total, int(budget), _ptr(budget_dev),
                                         _ptr(head_counts), _ptr(head_offsets), _ptr(kept_idx), _ptr(kept_scores),
                                         _ptr(workspace), workspace.numel(), _stream(stream))
        _check(st, "lava_select_topk_primed")
        return head_counts, head_offsets, kept_idx, kept_scores
    st = lib.lava_select_topk(n_heads, _ptr(scores), _ptr(seg_offsets), total, int(budget), _ptr(budget_dev),
                              _ptr(head_counts), _ptr(head_offsets), _ptr(kept_idx), _ptr(kept_scores),
                              _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, "lava_select_topk")
    return head_counts, head_offsets, kept_idx, kept_scores


SELECT_STATIC_MAX_ENTRIES = 1 << 22


def lava_select_topk_static(n_heads: int, scores: torch.Tensor, budget: int, head_counts: torch.Tensor,
                            head_offsets: torch.Tensor, kept_idx: torch.Tensor,
                            kept_scores: Optional[torch.Tensor] = None, seg_offsets: Optional[torch.Tensor] = None,
                            budget_dev: Optional[torch.Tensor] = None, total_entries: Optional[int] = None,
                            stream=None) -> None:
    """lava_select_topk on the library's built-in scratch array.  Allocates nothing: every buffer is the caller's."""
    _dev(scores, "scores", torch.float32), _dev(head_counts, "head_counts", torch.int32)
    _dev(head_offsets, "head_offsets", torch.int64), _dev(kept_idx, "kept_idx", torch.int32)
    for name, t, dt in (("kept_scores", kept_scores, torch.float32), ("seg_offsets", seg_offsets, torch.int64),
                        ("budget_dev", budget_dev, torch.int64)):
        if t is not None:
            _dev(t, name, dt)
    total = scores.numel() if total_entries is None else int(total_entries)
    st = lib.lava_select_topk_static(n_heads, _ptr(scores), _ptr(seg_offsets), total, int(budget), _ptr(budget_dev),
                                     _ptr(head_counts), _ptr(head_offsets), _ptr(kept_idx), _ptr(kept_scores),
                                     _stream(stream))
    _check(st, "lava_select_topk_static")


def lava_select_status(workspace: torch.Tensor, total_entries: int, stream=None) -> int:
    """Synchronises; LAVA_OK, or LAVA_ERR_HIP if the selection's bounded barrier wait gave up."""
    return int(lib.lava_select_status(_ptr(workspace), int(total_entries), _stream(stream)))


class SelectProblem(ctypes.Structure):
    """Mirror of lava_select_problem."""
    _fields_ = [
        ("scores", ctypes.c_void_p), ("seg_offsets", ctypes.c_void_p), ("total_entries", ctypes.c_int64),
        ("budget", ctypes.c_int64), ("budget_dev", ctypes.c_void_p), ("head_counts", ctypes.c_void_p),
        ("head_offsets", ctypes.c_void_p), ("kept_idx", ctypes.c_void_p), ("kept_scores", ctypes.c_void_p),
        ("in_offset_dev", ctypes.c_void_p), ("out_offset_dev", ctypes.c_void_p), ("error_dev", ctypes.c_void_p),
        ("primed", ctypes.c_int32),
    ]


class CompactProblem(ctypes.Structure):
    """Mirror of lava_compact_problem."""
    _fields_ = [
        ("src_rows", ctypes.c_int64), ("src_offsets", ctypes.c_void_p), ("k_src", ctypes.c_void_p),
        ("v_src", ctypes.c_void_p), ("pos_src", ctypes.c_void_p), ("head_offsets", ctypes.c_void_p),
        ("kept_idx", ctypes.c_void_p), ("capacity", ctypes.c_int64), ("k_out", ctypes.c_void_p),
        ("v_out", ctypes.c_void_p), ("pos_out", ctypes.c_void_p),
        ("src_offset_dev", ctypes.c_void_p), ("out_offset_dev", ctypes.c_void_p),
    ]


def _addr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def select_problem(scores, budget, head_counts, head_offsets, kept_idx, kept_scores=None, seg_offsets=None,
                   budget_dev=None, total_entries=None, in_offset_dev=None, out_offset_dev=None,
                   error_dev=None, primed=False) -> SelectProblem:
    """One row of the table of lava_select_topk_batch from device tensors (the caller keeps them alive)."""
    _dev(scores, "scores", torch.float32), _dev(head_counts, "head_counts", torch.int32)
    _dev(head_offsets, "head_offsets", torch.int64), _dev(kept_idx, "kept_idx", torch.int32)
    for name, t, dt in (("kept_scores", kept_scores, torch.float32), ("seg_offsets", seg_offsets, torch.int64),
                        ("budget_dev", budget_dev, torch.int64), ("in_offset_dev", in_offset_dev, torch.int64),
                        ("out_offset_dev", out_offset_dev, torch.int64), ("error_dev", error_dev, torch.int32)):
        if t is not None:
            _dev(t, name, dt)
    total = scores.numel() if total_entries is None else int(total_entries)
    return SelectProblem(_addr(scores), _addr(seg_offsets), total, int(budget), _addr(budget_dev),
                         _addr(head_counts), _addr(head_offsets), _addr(kept_idx), _addr(kept_scores),
                         _addr(in_offset_dev), _addr(out_offset_dev), _addr(error_dev), 1 if primed else 0)


def compact_problem(desc: LayerDesc, src_rows, k_src, v_src, head_offsets, kept_idx, capacity, k_out, v_out,
                    src_offsets=None, pos_src=None, pos_out=None, src_offset_dev=None,
                    out_offset_dev=None) -> CompactProblem:
    """One row of the table of lava_compact_batch (dense source when src_offsets is None)."""
    for name, t in (("k_src", k_src), ("v_src", v_src), ("k_out", k_out), ("v_out", v_out)):
        _dev(t, name, desc.torch_dtype)
    _dev(head_offsets, "head_offsets", torch.int64), _dev(kept_idx, "kept_idx", torch.int32)
    for name, t, dt in (("src_offsets", src_offsets, torch.int64), ("pos_src", pos_src, torch.int32),
                        ("pos_out", pos_out, torch.int32), ("src_offset_dev", src_offset_dev, torch.int64),
                        ("out_offset_dev", out_offset_dev, torch.int64)):
        if t is not None:
            _dev(t, name, dt)
    return CompactProblem(int(src_rows), _addr(src_offsets), _addr(k_src), _addr(v_src), _addr(pos_src),
                          _addr(head_offsets), _addr(kept_idx), int(capacity), _addr(k_out), _addr(v_out),
                          _addr(pos_out), _addr(src_offset_dev), _addr(out_offset_dev))


def lava_select_batch_workspace_bytes(n_problems: int, max_total_entries: int) -> int:
    return int(lib.lava_select_batch_workspace_bytes(int(n_problems), int(max_total_entries)))


def lava_select_topk_batch(n_heads: int, problems, max_total_entries=None, workspace=None, device="cuda",
                           stream=None):
    """problems: sequence of SelectProblem, or a ready (SelectProblem * n) array that a caller reuses from
    step to step.  Returns the workspace (for lava_select_batch_status)."""
    table = problems if isinstance(problems, ctypes.Array) else (SelectProblem * len(problems))(*problems)
    widest = max((p.total_entries for p in problems), default=0) if max_total_entries is None else int(max_total_entries)
    if workspace is None:
        need = lava_select_batch_workspace_bytes(len(problems), widest)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    st = lib.lava_select_topk_batch(int(n_heads), len(problems), ctypes.cast(table, ctypes.c_void_p), widest,
                                    _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, "lava_select_topk_batch")
    return workspace


def lava_select_batch_status(workspace: torch.Tensor, n_problems: int, max_total_entries: int, stream=None) -> int:
    return int(lib.lava_select_batch_status(_ptr(workspace), int(n_problems), int(max_total_entries),
                                            _stream(stream)))


def lava_compact_batch(desc: LayerDesc, problems, stream=None) -> None:
    """problems: sequence of CompactProblem, or a ready (CompactProblem * n) array."""
    table = problems if isinstance(problems, ctypes.Array) else (CompactProblem * len(problems))(*problems)
    st = lib.lava_compact_batch(ctypes.byref(desc), len(problems), ctypes.cast(table, ctypes.c_void_p),
                                _stream(stream))
    _check(st, "lava_compact_batch")


def lava_compact_kv(desc: LayerDesc, n: int, k: torch.Tensor, v: torch.Tensor, head_offsets: torch.Tensor,
                    kept_idx: torch.Tensor, capacity: int, k_out=None, v_out=None, stream=None):
    _dev(k, "k", desc.torch_dtype), _dev(v, "v", desc.torch_dtype)
    _dev(head_offsets, "head_offsets", torch.int64), _dev(kept_idx, "kept_idx", torch.int32)
    if k_out is None:
        k_out = torch.empty(max(int(capacity), 1), desc.head_dim, dtype=desc.torch_dtype, device=k.device)
    if v_out is None:
        v_out = torch.empty(max(int(capacity), 1), desc.head_dim, dtype=desc.torch_dtype, device=k.device)
    st = lib.lava_compact_kv(ctypes.byref(desc), int(n), _ptr(k), _ptr(v), _ptr(head_offsets), _ptr(kept_idx),
                             int(capacity), _ptr(k_out), _ptr(v_out), _stream(stream))
    _check(st, "lava_compact_kv")
    return k_out, v_out


def lava_compact_packed(desc: LayerDesc, src_offsets: torch.Tensor, k_src: torch.Tensor, v_src: torch.Tensor,
                        head_offsets: torch.Tensor, kept_idx: torch.Tensor, capacity: int, pos_src=None,
                        k_out=None, v_out=None, pos_out=None, stream=None):
    """Gather from an already packed cache (re-eviction).  Returns (k_out, v_out, pos_out)."""
    _dev(k_src, "k_src", desc.torch_dtype), _dev(v_src, "v_src", desc.torch_dtype)
    _dev(src_offsets, "src_offsets", torch.int64), _dev(head_offsets, "head_offsets", torch.int64)
    _dev(kept_idx, "kept_idx", torch.int32)
    if pos_src is not None:
        _dev(pos_src, "pos_src", torch.int32)
    rows = max(int(capacity), 1)
    if k_out is None:
        k_out = torch.empty(rows, desc.head_dim, dtype=desc.torch_dtype, device=k_src.device)
    if v_out is None:
        v_out = torch.empty(rows, desc.head_dim, dtype=desc.torch_dtype, device=k_src.device)
    if pos_out is None:
        pos_out = torch.empty(rows, dtype=torch.int32, device=k_src.device)
    st = lib.lava_compact_packed(ctypes.byref(desc), _ptr(src_offsets), k_src.shape[0], _ptr(k_src), _ptr(v_src),
                                 _ptr(pos_src), _ptr(head_offsets), _ptr(kept_idx), int(capacity), _ptr(k_out),
                                 _ptr(v_out), _ptr(pos_out), _stream(stream))
    _check(st, "lava_compact_packed")
    return k_out, v_out, pos_out


class CascadeStateStruct(ctypes.Structure):
    """Mirror of lava_cascade_state."""
    _fields_ = [
        ("k", ctypes.c_void_p * 2), ("v", ctypes.c_void_p * 2), ("pos", ctypes.c_void_p * 2),
        ("scores", ctypes.c_void_p * 2), ("head_offsets", ctypes.c_void_p * 2), ("layer_start", ctypes.c_void_p * 2),
        ("head_counts", ctypes.c_void_p), ("kept_idx", ctypes.c_void_p), ("error", ctypes.c_void_p),
        ("capacity", ctypes.c_int64), ("max_layers", ctypes.c_int32), ("cur", ctypes.c_int32),
    ]


class CascadeState:
    """Device buffers of a stack of layers for lava_cascade_step (allocation and views only): two arenas of
    `capacity` rows in which the layers sit back to back, plus the per-layer offsets.  in_place: K and V
    share ONE arena (the step re-compacts the earlier layers inside it), which halves the state."""

    def __init__(self, desc: LayerDesc, max_layers: int, capacity: int, device="cuda", in_place: bool = False):
        self.desc, self.n_layers, self.capacity = desc, int(max_layers), int(capacity)
        self.in_place = bool(in_place)
        hk = desc.n_kv_heads
        self.k = [torch.empty(capacity, desc.head_dim, dtype=desc.torch_dtype, device=device)]
        self.v = [torch.empty(capacity, desc.head_dim, dtype=desc.torch_dtype, device=device)]
        self.k.append(self.k[0] if in_place else torch.empty_like(self.k[0]))
        self.v.append(self.v[0] if in_place else torch.empty_like(self.v[0]))
        self.pos = [torch.empty(capacity, dtype=torch.int32, device=device) for _ in range(2)]
        self.scores = [torch.empty(capacity, dtype=torch.float32, device=device) for _ in range(2)]
        self.head_offsets = [torch.zeros(max_layers, hk + 1, dtype=torch.int64, device=device) for _ in range(2)]
        self.layer_start = [torch.zeros(max_layers + 1, dtype=torch.int64, device=device) for _ in range(2)]
        self.head_counts = torch.zeros(max_layers, hk, dtype=torch.int32, device=device)
        self.kept_idx = torch.empty(capacity, dtype=torch.int32, device=device)
        self.error = torch.zeros(1, dtype=torch.int32, device=device)
        self.e = torch.zeros(max_layers, dtype=torch.float32, device=device)
        self.budgets = torch.zeros(max_layers, dtype=torch.int64, device=device)
        c = self.c = CascadeStateStruct()
        for i in range(2):
            c.k[i], c.v[i], c.pos[i] = self.k[i].data_ptr(), self.v[i].data_ptr(), self.pos[i].data_ptr()
            c.scores[i] = self.scores[i].data_ptr()
            c.head_offsets[i], c.layer_start[i] = self.head_offsets[i].data_ptr(), self.layer_start[i].data_ptr()
        c.head_counts, c.kept_idx = self.head_counts.data_ptr(), self.kept_idx.data_ptr()
        c.error = self.error.data_ptr()
        c.capacity, c.max_layers, c.cur = self.capacity, self.n_layers, 0

    @property
    def cur(self) -> int:
        return int(self.c.cur)

    def reset(self) -> None:
        self.c.cur = 0
        self.error.zero_()

    def bytes(self) -> int:
        """Device bytes the state holds."""
        ts = (self.k[:1] + self.v[:1] if self.in_place else self.k + self.v)
        ts = ts + self.pos + self.scores + self.head_offsets + self.layer_start
        ts += [self.head_counts, self.kept_idx, self.e, self.budgets]
        return sum(t.numel() * t.element_size() for t in ts)

    def decode_args(self, t: int) -> dict:
        """What lava_decode_attention needs to read layer t in place (nothing is read back)."""
        c = self.cur
        return dict(k_hat=self.k[c], v_hat=self.v[c], head_offsets=self.head_offsets[c][t: t + 1],
                    seq_base=self.layer_start[c][t: t + 1], rows_capacity=self.capacity)

    def current(self, t: int) -> dict:
        """Views of layer t's current state (reads the layer's extent back: synchronises)."""
        c = self.cur
        start, end = (int(x) for x in self.layer_start[c][t: t + 2].cpu())
        return dict(k_hat=self.k[c][start:end], v_hat=self.v[c][start:end], pos=self.pos[c][start:end],
                    scores=self.scores[c][start:end], head_offsets=self.head_offsets[c][t],
                    head_counts=self.head_counts[t], start=start)


def lava_cascade_workspace_bytes(desc: LayerDesc, n: int, n_layers: int, total_budget: int) -> int:
    return int(lib.lava_cascade_workspace_bytes(ctypes.byref(desc), int(n), int(n_layers), int(total_budget)))


def lava_cascade_step(desc: LayerDesc, layer: int, n: int, k_new: torch.Tensor, v_new: torch.Tensor,
                      scores_new: torch.Tensor, state: CascadeState, total_budget: int, workspace=None, stream=None):
    """Alg. 2, one outer iteration; state.e[: layer + 1] must hold the layers' statistics."""
    _dev(k_new, "k_new", desc.torch_dtype), _dev(v_new, "v_new", desc.torch_dtype)
    _dev(scores_new, "scores_new", torch.float32)
    if workspace is None:
        need = lava_cascade_workspace_bytes(desc, n, state.n_layers, total_budget)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=k_new.device)
    st = lib.lava_cascade_step(ctypes.byref(desc), int(layer), int(n), _ptr(k_new), _ptr(v_new), _ptr(scores_new),
                               _ptr(state.e), int(total_budget), ctypes.byref(state.c),
                               _ptr(state.budgets), _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, "lava_cascade_step")
    return workspace


def lava_decode_workspace_bytes(desc: LayerDesc, batch: int, rows_capacity: int, tail_len: int = 0) -> int:
    return int(lib.lava_decode_workspace_bytes(ctypes.byref(desc), int(batch), int(rows_capacity), int(tail_len)))


def lava_decode_attention(desc: LayerDesc, batch: int, q: torch.Tensor, k_hat, v_hat, head_offsets: torch.Tensor,
                          rows_capacity: int, seq_base=None, k_tail=None, v_tail=None, tail_len: int = 0,
                          tail_capacity: int = 0, out=None, lse=None, workspace=None, stream=None):
    """One new token per sequence attends to the packed cache (+ dense tail).  Returns (out, lse)."""
    _dev(q, "q", desc.torch_dtype), _dev(head_offsets, "head_offsets", torch.int64)
    for name, t in (("k_hat", k_hat), ("v_hat", v_hat), ("k_tail", k_tail), ("v_tail", v_tail)):
        if t is not None:
            _dev(t, name, desc.torch_dtype)
    if seq_base is not None:
        _dev(seq_base, "seq_base", torch.int64)
    if out is None:
        out = torch.empty(batch, desc.n_q_heads, desc.head_dim, dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty(batch, desc.n_q_heads, dtype=torch.float32, device=q.device)
    if workspace is None:
        need = lava_decode_workspace_bytes(desc, batch, rows_capacity, tail_len)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    st = lib.lava_decode_attention(ctypes.byref(desc), int(batch), _ptr(q), _ptr(k_hat), _ptr(v_hat),
                                   _ptr(head_offsets), _ptr(seq_base), int(rows_capacity), _ptr(k_tail),
                                   _ptr(v_tail), int(tail_len), int(tail_capacity), _ptr(out), _ptr(lse),
                                   _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, "lava_decode_attention")
    return out, lse


# ------------------------------------------------------------------------------ timing hook
def prof_enable(on: bool = True) -> None:
    lib.lava_prof_enable(1 if on else 0)


def prof_reset() -> None:
    lib.lava_prof_reset()


def prof_read() -> dict:
    """{kernel name: (total milliseconds, launches)} since the last reset."""
    out = {}
    for i in range(lib.lava_prof_kernel_count()):
        ms, cnt = ctypes.c_double(0.0), ctypes.c_int64(0)
        lib.lava_prof_read(i, ctypes.byref(ms), ctypes.byref(cnt))
        out[lib.lava_prof_kernel_name(i).decode()] = (ms.value, cnt.value)
    return out


def probe_stream(src: torch.Tensor, dst: torch.Tensor, nbytes: int, mode: int, blocks: int = 2048, stream=None):
    """mode 0: copy nbytes from src to dst; mode 1: read nbytes of src."""
    _check(lib.lava_probe_stream(_ptr(src), _ptr(dst), int(nbytes), int(mode), int(blocks), _stream(stream)),
           "lava_probe_stream")


def evict_layer(desc: LayerDesc, n: int, q_win, k, v, budget: int, lse=None, stream=None, primed: bool = True):
    """The calls of one layer in order for one sequence (fixed budget): scores, selection, compaction.
    primed: the scores call prepares the selection's workspace (lava_window_scores_primed +
    lava_select_topk_primed) instead of the plain pair; the results are the same."""
    ws = None
    if primed:
        ws = torch.empty(max(lava_select_workspace_bytes(desc.n_kv_heads * n), 256), dtype=torch.uint8, device=k.device)
    scores, vbar, stat = lava_window_scores(desc, [n], q_win, k, v, lse=lse, stream=stream, select_workspace=ws)
    counts, offs, idx, kept_s = lava_select_topk(desc.n_kv_heads, scores, budget, stream=stream, workspace=ws,
                                                 primed=primed)
    k_hat, v_hat = lava_compact_kv(desc, n, k, v, offs, idx, budget, stream=stream)
    return dict(scores=scores, vbar=vbar, layer_stat=stat, head_counts=counts, head_offsets=offs,
                kept_idx=idx, kept_scores=kept_s, k_hat=k_hat, v_hat=v_hat)
