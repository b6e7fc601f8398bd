"""ctypes binding of include/moe_hotpath.h and include/moe_sched.h -- argument
marshalling only.

Names mirror the C entry points.  Tensors are torch CUDA tensors owned by the
caller; bf16 data may be passed as ``torch.bfloat16`` or as raw ``int16`` /
``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

from .build import LIB

MOE_F32, MOE_BF16 = 0, 1
MOE_ROW_MAJOR, MOE_TILED = 0, 1
MOE_OPT_SYNC_COPIES, MOE_OPT_COPY_SPLIT, MOE_OPT_EXPORT_COUNTS = 0, 1, 2
STATUS = {0: "MOE_OK", -1: "MOE_ERR_INVALID_ARG", -2: "MOE_ERR_UNSUPPORTED",
          -3: "MOE_ERR_WORKSPACE", -4: "MOE_ERR_HIP", -5: "MOE_ERR_SLOT_EXHAUSTED"}


class MoEError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS.get(status, status)}: {msg}")
        self.status = status


class moe_shape(C.Structure):
    _fields_ = [("T", C.c_int32), ("H", C.c_int32), ("E", C.c_int32), ("k", C.c_int32),
                ("F", C.c_int32), ("S", C.c_int32), ("dtype", C.c_int32),
                ("weight_layout", C.c_int32)]


class moe_expert_ptrs(C.Structure):
    _fields_ = [("Wg", C.c_void_p), ("Wu", C.c_void_p), ("Wd", C.c_void_p)]


class moe_layer_desc(C.Structure):
    _fields_ = [("Wr", C.c_void_p), ("bias", C.c_void_p),
                ("host_dev", C.POINTER(moe_expert_ptrs)),
                ("host_pinned", C.POINTER(moe_expert_ptrs)),
                ("layer_id", C.c_uint64)]


class moe_layer_stats(C.Structure):
    _fields_ = [("n_active", C.c_int32), ("n_resident", C.c_int32), ("n_hit", C.c_int32),
                ("n_miss", C.c_int32), ("n_wasted", C.c_int32), ("n_prefetch_issued", C.c_int32),
                ("bytes_on_demand", C.c_int64), ("bytes_prefetch", C.c_int64)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_}


class moe_stream_totals(C.Structure):
    _fields_ = [("bytes", C.c_int64), ("n_copies", C.c_int64), ("copy_ms", C.c_double)]


class moe_phase_times(C.Structure):
    _fields_ = [("route_ms", C.c_double), ("permute_ms", C.c_double), ("gate_up_ms", C.c_double),
                ("down_ms", C.c_double), ("combine_ms", C.c_double), ("n_layers", C.c_int64),
                ("gate_up_only_ms", C.c_double), ("gate_up_only_layers", C.c_int64)]


SCHED_MAX = 128


class moe_presched_costs(C.Structure):
    _fields_ = [("t_io", C.c_double), ("t_g", C.c_double), ("t_attn", C.c_double),
                ("beta", C.c_double), ("C", C.c_double), ("alpha", C.c_double),
                ("r_hit", C.c_double), ("cpu_executor", C.c_int32)]


class moe_pending(C.Structure):
    _fields_ = [("expert", C.c_int32), ("tokens", C.c_int32)]


class moe_presched_plan(C.Structure):
    _fields_ = [("n_cur", C.c_int32), ("n_next", C.c_int32),
                ("cur_sorted", C.c_int32 * SCHED_MAX), ("next_sorted", C.c_int32 * SCHED_MAX),
                ("n_all", C.c_int32), ("all_layer", C.c_int32 * (2 * SCHED_MAX)),
                ("all_expert", C.c_int32 * (2 * SCHED_MAX)),
                ("all_in_queue", C.c_int32 * (2 * SCHED_MAX)),
                ("i_prime", C.c_int32), ("n_ondemand", C.c_int32),
                ("ondemand", C.c_int32 * SCHED_MAX),
                ("T_gap", C.c_double), ("f", C.c_double), ("f_abs", C.c_int32), ("xi", C.c_double),
                ("n_prefetch", C.c_int32), ("prefetch", C.c_int32 * SCHED_MAX)]


if not os.path.exists(LIB):
    raise ImportError(
        f"{LIB} is missing: build it first (python -m paper_2509_23638_amd.build, or "
        "__graft_entry__.build()).  There is no fallback path.")
_lib = C.CDLL(LIB)

_P = C.c_void_p
_SH = C.POINTER(moe_shape)
_lib.moe_version.restype = C.c_char_p
_lib.moe_last_error.restype = C.c_char_p
_lib.moe_ffn_kernel_name.restype = C.c_char_p
_lib.moe_ffn_kernel_name.argtypes = [_SH, C.c_int32, C.c_int32]
_lib.moe_layer_y_dtype.restype = C.c_int32
_lib.moe_layer_y_dtype.argtypes = [_SH]
_lib.moe_workspace_bytes.restype = C.c_size_t
_lib.moe_workspace_bytes.argtypes = [_SH]
_lib.moe_route.argtypes = [_SH, _P, _P, _P, _P, _P, _P, _P, _P]
_lib.moe_permute.argtypes = [_SH, _P, _P, _P, _P, _P, _P]
_lib.moe_grouped_ffn.argtypes = [_SH, _P, _P, _P, C.POINTER(moe_expert_ptrs),
                                 C.POINTER(C.c_uint64), _P, _P, _P]
_lib.moe_combine.argtypes = [_SH, _P, _P, _P, _P, _P, _P]
_lib.moe_create.argtypes = [_SH, C.c_int32, C.c_int32, C.POINTER(_P)]
_lib.moe_destroy.argtypes = [_P]
_lib.moe_layer_forward.argtypes = [_P, _SH, C.POINTER(moe_layer_desc), C.POINTER(C.c_uint64),
                                   C.POINTER(moe_layer_desc), C.POINTER(C.c_uint64),
                                   _P, _P, _P, _P, _P, C.POINTER(moe_layer_stats)]
_lib.moe_layer_forward_static.argtypes = [_SH, C.POINTER(moe_layer_desc), _P, _P, _P, _P]
_lib.moe_prefetch.argtypes = [_P, _SH, C.POINTER(moe_layer_desc), C.POINTER(C.c_uint64), _P,
                              C.POINTER(C.c_int32)]
_lib.moe_layer_counts.argtypes = [_P, C.POINTER(C.c_int32), C.c_int32]
_lib.moe_static_workspace_bytes.restype = C.c_size_t
_lib.moe_static_workspace_bytes.argtypes = []
_lib.moe_stream_totals_get.argtypes = [_P, C.POINTER(moe_stream_totals), C.c_int32]
_lib.moe_phase_timing.argtypes = [_P, C.c_int32]
_lib.moe_phase_times_get.argtypes = [_P, C.POINTER(moe_phase_times), C.c_int32]
_lib.moe_probe_copy.argtypes = [_P, _P, C.c_size_t, _P]
_lib.moe_probe_read.argtypes = [_P, C.c_size_t, _P, _P]
_lib.moe_probe_read_nt.argtypes = [_P, C.c_size_t, _P, _P]
_lib.moe_probe_stage.argtypes = [_P, C.c_size_t, _P, C.c_size_t, C.c_int32, C.c_int32, _P]
_lib.moe_set_option.argtypes = [_P, C.c_int32, C.c_int64]
_lib.moe_pack_weights.argtypes = [_P, _P, C.c_int32, C.c_int32, _P]
_lib.moe_rmsnorm.argtypes = [_SH, _P, _P, C.c_float, _P]
_lib.moe_workspace_views.argtypes = [_SH, _P] + [C.POINTER(_P)] * 7
_lib.moe_counter_add.argtypes = [_SH, _P, _P, _P]
_lib.moe_hot_table.argtypes = [_P, C.c_int32, C.c_int32, C.c_int64, _P]
_lib.moe_predict_counts.argtypes = [_SH, _P, _P, _P, _P, _P, _P]
_lib.moe_pending_experts.argtypes = [_P, C.c_int32, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64),
                                     C.POINTER(moe_pending), C.POINTER(C.c_int32)]
_lib.moe_prefetch_hottest.argtypes = [C.POINTER(moe_pending), C.c_int32, C.c_int32,
                                      C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
_lib.moe_presched.argtypes = [C.POINTER(moe_presched_costs), C.POINTER(moe_pending), C.c_int32,
                              C.POINTER(moe_pending), C.c_int32, C.POINTER(moe_presched_plan)]
for _n in ("moe_counter_add", "moe_hot_table", "moe_predict_counts", "moe_presched",
           "moe_pending_experts", "moe_prefetch_hottest", "moe_layer_forward_static",
           "moe_route", "moe_permute", "moe_grouped_ffn", "moe_combine", "moe_create",
           "moe_destroy", "moe_layer_forward", "moe_layer_forward_static", "moe_stream_totals_get",
           "moe_workspace_views", "moe_phase_timing", "moe_phase_times_get", "moe_probe_copy", "moe_probe_read",
           "moe_probe_read_nt", "moe_probe_stage", "moe_rmsnorm", "moe_set_option", "moe_pack_weights",
           "moe_prefetch", "moe_layer_counts"):
    getattr(_lib, _n).restype = C.c_int32

EXPORTS = ["moe_version", "moe_last_error", "moe_workspace_bytes", "moe_route", "moe_permute",
           "moe_grouped_ffn", "moe_combine", "moe_create", "moe_destroy", "moe_layer_forward",
           "moe_stream_totals_get", "moe_workspace_views", "moe_phase_timing",
           "moe_phase_times_get", "moe_probe_copy", "moe_probe_read", "moe_probe_read_nt",
           "moe_probe_stage", "moe_rmsnorm", "moe_set_option", "moe_pack_weights",
           "moe_counter_add", "moe_hot_table", "moe_predict_counts", "moe_presched",
           "moe_ffn_kernel_name", "moe_layer_forward_static", "moe_static_workspace_bytes",
           "moe_pending_experts", "moe_prefetch_hottest", "moe_prefetch", "moe_layer_counts",
           "moe_layer_y_dtype"]


def _check(st: int):
    if st != 0:
        raise MoEError(st, _lib.moe_last_error().decode())


def moe_layer_y_dtype(shape) -> torch.dtype:
    """Element type of the rows of Y that moe_layer_forward leaves in the workspace."""
    d = _lib.moe_layer_y_dtype(C.byref(shape))
    if d < 0:
        raise MoEError(-1, _lib.moe_last_error().decode())
    return torch.bfloat16 if d == MOE_BF16 else torch.float32


def moe_ffn_kernel_name(shape, phase: int, n_groups: int) -> str:
    return _lib.moe_ffn_kernel_name(C.byref(shape), phase, n_groups).decode()


def moe_version() -> str:
    return _lib.moe_version().decode()


def moe_last_error() -> str:
    return _lib.moe_last_error().decode()


# ------------------------------------------------------------ marshalling ---
def make_shape(T, H, E, k, F, S=0, dtype="bf16", layout="row_major") -> moe_shape:
    return moe_shape(T, H, E, k, F, S, MOE_F32 if dtype in ("f32", MOE_F32) else MOE_BF16,
                     MOE_TILED if layout in ("tiled", MOE_TILED) else MOE_ROW_MAJOR)


def with_T(shape: moe_shape, T: int) -> moe_shape:
    return moe_shape(T, shape.H, shape.E, shape.k, shape.F, shape.S, shape.dtype, shape.weight_layout)


def _ptr(t: Optional[torch.Tensor], what: str, dtypes=None, numel=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{what}: expected a CUDA tensor")
    if not t.is_contiguous():
        raise ValueError(f"{what}: tensor must be contiguous")
    if dtypes is not None and t.dtype not in dtypes:
        raise ValueError(f"{what}: dtype {t.dtype} not in {dtypes}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{what}: needs at least {numel} elements, has {t.numel()}")
    return t.data_ptr()


def _storage_dtypes(shape: moe_shape):
    return (torch.float32,) if shape.dtype == MOE_F32 else (torch.bfloat16, torch.int16, torch.uint16)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return stream or None


def _mask_words(mask, n: int):
    """bool sequence / int -> ctypes uint64 array (or None)."""
    if mask is None:
        return None
    words = (n + 63) // 64
    arr = (C.c_uint64 * words)()
    if isinstance(mask, int):
        for w in range(words):
            arr[w] = (mask >> (64 * w)) & 0xFFFFFFFFFFFFFFFF
    else:
        for e, on in enumerate(mask):
            if on:
                if e >= n:
                    raise ValueError("mask longer than the expert count")
                arr[e // 64] |= 1 << (e % 64)
    return arr


def moe_workspace_bytes(shape: moe_shape) -> int:
    n = _lib.moe_workspace_bytes(C.byref(shape))
    if n == 0:
        raise MoEError(-1, moe_last_error())
    return n


def alloc_workspace(shape: moe_shape, device="cuda") -> torch.Tensor:
    return torch.empty(moe_workspace_bytes(shape), dtype=torch.uint8, device=device)


def moe_route(shape, X, Wr, bias, topk_idx, topk_w, logits_out=None, workspace=None, stream=None):
    sd = _storage_dtypes(shape)
    A = shape.T * shape.k
    _check(_lib.moe_route(
        C.byref(shape), _ptr(X, "X", sd, shape.T * shape.H), _ptr(Wr, "Wr", sd, shape.E * shape.H),
        _ptr(bias, "bias", (torch.float32,), shape.E),
        _ptr(topk_idx, "topk_idx", (torch.int32,), A), _ptr(topk_w, "topk_w", (torch.float32,), A),
        _ptr(logits_out, "logits_out", (torch.float64,), shape.T * shape.E),
        _ptr(workspace, "workspace"), _stream(stream)))


def moe_permute(shape, topk_idx, count, offset, perm, inv_perm, stream=None):
    A = shape.T * shape.k
    i32 = (torch.int32,)
    _check(_lib.moe_permute(
        C.byref(shape), _ptr(topk_idx, "topk_idx", i32, A), _ptr(count, "count", i32, shape.E),
        _ptr(offset, "offset", i32, shape.E + 1), _ptr(perm, "perm", i32, A),
        _ptr(inv_perm, "inv_perm", i32, A), _stream(stream)))


def expert_table(shape, Wg, Wu, Wd, what="experts"):
    """ctypes array [E+S] of device (or pinned-host) pointers from stacked
    tensors [E+S, ...] or sequences of per-expert tensors (None = absent)."""
    n = shape.E + shape.S
    arr = (moe_expert_ptrs * n)()
    for e in range(n):
        for name, W in (("Wg", Wg), ("Wu", Wu), ("Wd", Wd)):
            t = W[e] if W is not None else None
            if t is not None:
                if not t.is_contiguous():
                    raise ValueError(f"{what}[{e}].{name} must be contiguous")
                if t.numel() != shape.H * shape.F:
                    raise ValueError(f"{what}[{e}].{name}: expected {shape.H * shape.F} elements")
                setattr(arr[e], name, t.data_ptr())
    return arr


def moe_grouped_ffn(shape, X, perm, offset, experts, expert_mask, Y, workspace, stream=None):
    sd = _storage_dtypes(shape)
    A = shape.T * shape.k
    rows = A + shape.S * shape.T
    _check(_lib.moe_grouped_ffn(
        C.byref(shape), _ptr(X, "X", sd, shape.T * shape.H), _ptr(perm, "perm", (torch.int32,), A),
        _ptr(offset, "offset", (torch.int32,), shape.E + 1), experts,
        _mask_words(expert_mask, shape.E + shape.S),
        _ptr(Y, "Y", (torch.float32,), rows * shape.H),
        _ptr(workspace, "workspace", (torch.uint8,), moe_workspace_bytes(shape)), _stream(stream)))


def moe_combine(shape, Y, topk_w, inv_perm, residual, out, stream=None):
    sd = _storage_dtypes(shape)
    A = shape.T * shape.k
    rows = A + shape.S * shape.T
    _check(_lib.moe_combine(
        C.byref(shape), _ptr(Y, "Y", (torch.float32,), rows * shape.H),
        _ptr(topk_w, "topk_w", (torch.float32,), A), _ptr(inv_perm, "inv_perm", (torch.int32,), A),
        _ptr(residual, "residual", sd, shape.T * shape.H), _ptr(out, "out", sd, shape.T * shape.H),
        _stream(stream)))


class Context:
    """moe_create / moe_destroy."""

    def __init__(self, max_shape: moe_shape, n_ondemand_slots=0, n_prefetch_slots_per_group=0):
        self._h = _P()
        _check(_lib.moe_create(C.byref(max_shape), n_ondemand_slots, n_prefetch_slots_per_group,
                               C.byref(self._h)))

    def close(self):
        if self._h:
            _check(_lib.moe_destroy(self._h))
            self._h = _P()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_sync_copies(self, enable: bool):
        _check(_lib.moe_set_option(self._h, MOE_OPT_SYNC_COPIES, 1 if enable else 0))

    def set_export_counts(self, enable: bool):
        _check(_lib.moe_set_option(self._h, MOE_OPT_EXPORT_COUNTS, 1 if enable else 0))

    def layer_counts(self, E: int):
        """Token counts per expert of the layer the last moe_layer_forward ran."""
        import numpy as np
        out = (C.c_int32 * E)()
        _check(_lib.moe_layer_counts(self._h, out, E))
        return np.frombuffer(out, dtype=np.int32).copy()

    def set_copy_split(self, n: int):
        _check(_lib.moe_set_option(self._h, MOE_OPT_COPY_SPLIT, n))

    def phase_timing(self, mode):
        """0/False off, 1/True all five phases, 2 only the gate/up kernel."""
        _check(_lib.moe_phase_timing(self._h, int(mode)))

    def phase_times(self, reset=False) -> dict:
        t = moe_phase_times()
        _check(_lib.moe_phase_times_get(self._h, C.byref(t), 1 if reset else 0))
        return {f: getattr(t, f) for f, _ in t._fields_}

    def stream_totals(self, reset=False) -> dict:
        t = moe_stream_totals()
        _check(_lib.moe_stream_totals_get(self._h, C.byref(t), 1 if reset else 0))
        return {"bytes": t.bytes, "n_copies": t.n_copies, "copy_ms": t.copy_ms}


@dataclass
class Layer:
    """Keeps a layer's tensors alive next to the descriptor built from them."""
    desc: moe_layer_desc
    keep: tuple


def make_layer_desc(shape, Wr, bias, dev=None, pinned=None, layer_id=0) -> Layer:
    """dev / pinned: (Wg, Wu, Wd) each a stacked tensor or a per-expert sequence
    with None for absent experts; pinned tensors must live in pinned host
    memory."""
    sd = _storage_dtypes(shape)
    d = moe_layer_desc()
    d.Wr = _ptr(Wr, "Wr", sd, shape.E * shape.H)
    d.bias = _ptr(bias, "bias", (torch.float32,), shape.E)
    dev_arr = expert_table(shape, *dev, what="dev") if dev is not None else None
    pin_arr = None
    if pinned is not None:
        for W in pinned:
            for t in W:
                if t is not None and not t.is_pinned():
                    raise ValueError("host expert copies must be in pinned memory")
        pin_arr = expert_table(shape, *pinned, what="pinned")
    if dev_arr is not None:
        d.host_dev = dev_arr
    if pin_arr is not None:
        d.host_pinned = pin_arr
    d.layer_id = layer_id
    return Layer(d, (Wr, bias, dev, pinned, dev_arr, pin_arr))


def moe_layer_forward(ctx: Context, shape, layer: Layer, X, out, workspace, resident_mask=None,
                      next_layer: Optional[Layer] = None, prefetch_next_mask=None,
                      residual=None, stream=None, want_stats=False):
    sd = _storage_dtypes(shape)
    stats = moe_layer_stats() if want_stats else None
    _check(_lib.moe_layer_forward(
        ctx._h, C.byref(shape), C.byref(layer.desc), _mask_words(resident_mask, shape.E),
        C.byref(next_layer.desc) if next_layer is not None else None,
        _mask_words(prefetch_next_mask, shape.E),
        _ptr(X, "X", sd, shape.T * shape.H), _ptr(residual, "residual", sd, shape.T * shape.H),
        _ptr(out, "out", sd, shape.T * shape.H),
        _ptr(workspace, "workspace", (torch.uint8,), moe_workspace_bytes(shape)),
        _stream(stream), C.byref(stats) if stats is not None else None))
    return stats.as_dict() if stats is not None else None


def moe_prefetch(ctx: Context, shape, next_layer: Layer, prefetch_mask, stream=None) -> int:
    """The prefetch step as a call of its own; returns the number of copies queued."""
    n = C.c_int32(0)
    _check(_lib.moe_prefetch(ctx._h, C.byref(shape), C.byref(next_layer.desc),
                             _mask_words(prefetch_mask, shape.E), _stream(stream), C.byref(n)))
    return n.value


def moe_static_workspace_bytes() -> int:
    return _lib.moe_static_workspace_bytes()


def moe_layer_forward_static(shape, layer: Layer, X, out, residual=None, stream=None):
    """moe_layer_forward for an all-resident layer, workspace inside the library."""
    sd = _storage_dtypes(shape)
    _check(_lib.moe_layer_forward_static(
        C.byref(shape), C.byref(layer.desc), _ptr(X, "X", sd, shape.T * shape.H),
        _ptr(residual, "residual", sd, shape.T * shape.H), _ptr(out, "out", sd, shape.T * shape.H),
        _stream(stream)))


def moe_pack_weights(src: torch.Tensor, dst: torch.Tensor, N: int, K: int, stream=None):
    """One [N,K] bf16 matrix, row-major -> tiled."""
    bf = (torch.bfloat16, torch.int16, torch.uint16)
    _check(_lib.moe_pack_weights(_ptr(src, "src", bf, N * K), _ptr(dst, "dst", bf, N * K), N, K,
                                 _stream(stream)))


def pack_experts(W: torch.Tensor) -> torch.Tensor:
    """[n, N, K] row-major expert matrices -> the same tensor shape holding each
    matrix in tiled form (a new tensor)."""
    out = torch.empty_like(W)
    n, N, K = W.shape
    for e in range(n):
        moe_pack_weights(W[e], out[e], N, K)
    return out


def moe_rmsnorm(shape, X, out, eps=1e-6, stream=None):
    sd = _storage_dtypes(shape)
    n = shape.T * shape.H
    _check(_lib.moe_rmsnorm(C.byref(shape), _ptr(X, "X", sd, n), _ptr(out, "out", sd, n),
                            C.c_float(eps), _stream(stream)))


def moe_probe_copy(dst: torch.Tensor, src: torch.Tensor, stream=None):
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < n:
        raise ValueError("dst smaller than src")
    _check(_lib.moe_probe_copy(_ptr(dst, "dst"), _ptr(src, "src"), n, _stream(stream)))


def moe_probe_read(src: torch.Tensor, sink: torch.Tensor, stream=None):
    n = src.numel() * src.element_size()
    _check(_lib.moe_probe_read(_ptr(src, "src"), n, _ptr(sink, "sink", None, 1), _stream(stream)))


def moe_probe_read_nt(src: torch.Tensor, sink: torch.Tensor, stream=None):
    n = src.numel() * src.element_size()
    _check(_lib.moe_probe_read_nt(_ptr(src, "src"), n, _ptr(sink, "sink", None, 1), _stream(stream)))


def moe_probe_stage(weights: torch.Tensor, tokens: torch.Tensor, token_fetches: int, stages: int, stream=None):
    _check(_lib.moe_probe_stage(_ptr(weights, "weights"), weights.numel() * weights.element_size(),
                                _ptr(tokens, "tokens"), tokens.numel() * tokens.element_size(),
                                int(token_fetches), int(stages), _stream(stream)))


def moe_workspace_views(shape, workspace: torch.Tensor) -> dict:
    """Typed tensor views of a workspace (same memory)."""
    ptrs = [_P() for _ in range(7)]
    _check(_lib.moe_workspace_views(C.byref(shape), workspace.data_ptr(), *[C.byref(p) for p in ptrs]))
    base = workspace.data_ptr()
    A = shape.T * shape.k
    rows = A + shape.S * shape.T
    spec = [("topk_idx", torch.int32, (shape.T, shape.k)), ("topk_w", torch.float32, (shape.T, shape.k)),
            ("count", torch.int32, (shape.E,)), ("offset", torch.int32, (shape.E + 1,)),
            ("perm", torch.int32, (A,)), ("inv_perm", torch.int32, (A,)),
            ("Y", moe_layer_y_dtype(shape), (rows, shape.H))]
    out = {}
    for p, (name, dt, shp) in zip(ptrs, spec):
        off = p.value - base
        n = 1
        for s in shp:
            n *= s
        nbytes = n * torch.empty((), dtype=dt).element_size()
        out[name] = workspace[off:off + nbytes].view(dt).view(shp)
    return out


# ------------------------------------------------------------ moe_sched.h --
def moe_counter_add(shape, count: torch.Tensor, total: torch.Tensor, stream=None):
    _check(_lib.moe_counter_add(C.byref(shape), _ptr(count, "count", (torch.int32,), shape.E),
                                _ptr(total, "total", (torch.int64,), shape.E), _stream(stream)))


def moe_hot_table(tokens, budget_experts: int):
    """tokens: int64 array-like [L, E] on the host -> bool numpy array [L, E]."""
    import numpy as np
    t = np.ascontiguousarray(np.asarray(tokens, dtype=np.int64))
    if t.ndim != 2:
        raise ValueError("tokens must be [L, E]")
    L, E = t.shape
    out = np.zeros((L, E), dtype=np.uint8)
    _check(_lib.moe_hot_table(t.ctypes.data, L, E, int(budget_experts), out.ctypes.data))
    return out.astype(bool)


def moe_predict_counts(shape, X, Wr_next, bias_next, pred_count, workspace, stream=None):
    sd = _storage_dtypes(shape)
    _check(_lib.moe_predict_counts(
        C.byref(shape), _ptr(X, "X", sd, shape.T * shape.H),
        _ptr(Wr_next, "Wr_next", sd, shape.E * shape.H),
        _ptr(bias_next, "bias_next", (torch.float32,), shape.E),
        _ptr(pred_count, "pred_count", (torch.int32,), shape.E),
        _ptr(workspace, "workspace"), _stream(stream)))


def moe_pending_experts(counts, resident=None, in_flight=None):
    """counts: E ints on the host; resident / in_flight: bool sequences or None.
    Returns [(expert, tokens)] by ascending expert id."""
    E = len(counts)
    arr = (C.c_int32 * E)(*[int(c) for c in counts])
    out = (moe_pending * E)()
    n = C.c_int32(0)
    _check(_lib.moe_pending_experts(arr, E, _mask_words(resident, E), _mask_words(in_flight, E),
                                    out, C.byref(n)))
    return [(out[i].expert, out[i].tokens) for i in range(n.value)]


def moe_prefetch_hottest(pending, n_prefetch: int):
    """pending: [(expert, tokens)] -> expert ids in issue order."""
    arr = (moe_pending * max(1, len(pending)))()
    for i, (e, m) in enumerate(pending):
        arr[i].expert, arr[i].tokens = int(e), int(m)
    out = (C.c_int32 * max(1, len(pending)))()
    n = C.c_int32(0)
    _check(_lib.moe_prefetch_hottest(arr, len(pending), int(n_prefetch), out, C.byref(n)))
    return [out[i] for i in range(n.value)]


def moe_presched(costs: moe_presched_costs, cur, nxt) -> moe_presched_plan:
    """cur / nxt: sequences of (expert id, pending tokens)."""
    def pack(lst):
        arr = (moe_pending * max(1, len(lst)))()
        for i, (e, m) in enumerate(lst):
            arr[i].expert, arr[i].tokens = int(e), int(m)
        return arr
    plan = moe_presched_plan()
    _check(_lib.moe_presched(C.byref(costs), pack(cur), len(cur), pack(nxt), len(nxt),
                             C.byref(plan)))
    return plan
