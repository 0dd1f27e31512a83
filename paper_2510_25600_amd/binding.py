"""ctypes binding of libpurekv.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/purekv.h).  PyTorch is used
for device memory and the current stream; no step of the method runs in Python or in PyTorch ops.
There is no CPU fallback: if the library is missing, import fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_size_t, c_uint32, c_void_p
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# PUREKV_LIB names another build of the same sources to load instead (the host-sanitizer build of the planner and
# the validation code, a tuning build); the default is the library built in-tree.
LIB_PATH = os.environ.get("PUREKV_LIB") or os.path.join(_HERE, "libpurekv.so")

PATTERN_DENSE, PATTERN_SPATIAL, PATTERN_TEMPORAL, PATTERN_ST = 0, 1, 2, 3
OP_PREFILL, OP_IMPORTANCE, OP_TOPK, OP_COMPACT, OP_DECODE = 0, 1, 2, 3, 4
OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP, ENOMEM = 0, -1, -2, -3, -4, -5
BLOCK, BK, WAVES = 32, 64, 8
KIND_FULL, KIND_CAUSAL, KIND_PREV, KIND_GENERAL = 0, 1, 2, 3


class Shape(ctypes.Structure):
    _fields_ = [
        ("n_frames", c_int32), ("patch_h", c_int32), ("patch_w", c_int32), ("n_text", c_int32),
        ("n_q_heads", c_int32), ("n_kv_heads", c_int32), ("head_dim", c_int32),
        ("pattern", c_uint32), ("softmax_scale", c_float),
        ("q_stride_head", c_int64), ("q_stride_tok", c_int64),
        ("kv_stride_head", c_int64), ("kv_stride_tok", c_int64),
        ("o_stride_head", c_int64), ("o_stride_tok", c_int64),
    ]


class PureKVError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {purekv_strerror(status)} (status {status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2510_25600_amd.build` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    P = c_void_p
    sig = {
        "purekv_plan_create": (c_int, [POINTER(Shape), POINTER(P), P]),
        "purekv_plan_create_host": (c_int, [POINTER(Shape), c_int32, POINTER(P)]),
        "purekv_plan_destroy": (c_int, [P]),
        "purekv_plan_create_heads": (c_int, [POINTER(Shape), P, POINTER(c_void_p), P]),
        "purekv_plan_create_heads_host": (c_int, [POINTER(Shape), P, c_int32, POINTER(c_void_p)]),
        "purekv_plan_create_window": (c_int, [POINTER(Shape), c_int32, POINTER(c_void_p), P]),
        "purekv_plan_create_window_host": (c_int, [POINTER(Shape), c_int32, c_int32, POINTER(c_void_p)]),
        "purekv_plan_counts": (c_int, [P, POINTER(c_int64)]),
        "purekv_plan_qtile_list": (c_int, [P, c_int32, POINTER(c_int32), c_int32]),
        "purekv_plan_item": (c_int, [P, c_int32, POINTER(c_int32)]),
        "purekv_plan_queue": (c_int, [P, c_int32, POINTER(c_int32), c_int32]),
        "purekv_plan_steps": (c_int, [P, c_int32, POINTER(c_int32), c_int32]),
        "purekv_spearman": (c_int, [P, P, c_int32, c_int32, P, P, P]),
        "purekv_workspace_bytes": (c_size_t, [P, c_int, c_int32, c_int32, c_int32]),
        "purekv_workspace_init": (c_int, [P, c_int, P, c_size_t, c_int32, c_int32, c_int32, P]),
        "purekv_stack_workspace_init": (c_int, [P, P, P, P, c_size_t, P]),
        "purekv_st_spattn_prefill": (c_int, [P, P, P, P, P, P, P, c_size_t, P]),
        "purekv_st_spattn_prefill_vnorm": (c_int, [P, P, P, P, P, P, P, P, c_size_t, P]),
        "purekv_topk_select_vnorm": (c_int, [P, P, P, c_int64, c_int32, c_int32, c_int32, P, P, P, c_size_t, P]),
        "purekv_lowlayer_importance": (c_int, [P, P, P, P, c_int32, P, P, c_size_t, P]),
        "purekv_topk_select": (c_int, [P, P, P, c_int64, c_int32, c_int32, c_int32, P, P, P, c_size_t, P]),
        "purekv_topk_select_static": (c_int, [P, P, P, c_int64, c_int32, c_int32, c_int32, P, P]),
        "purekv_kv_compact": (c_int, [P, P, P, c_int64, c_int32, P, c_int32, P, P, c_int32, P]),
        "purekv_kv_append": (c_int, [P, P, P, P, P, c_int32, c_int32, P]),
        "purekv_decode_attn": (c_int, [P, P, P, P, c_int32, c_int32, P, P, c_size_t, P]),
        "purekv_decode_step": (c_int, [P, P, P, P, P, P, c_int32, c_int32, P, P, c_size_t, P]),
        "purekv_stack_workspace_bytes": (c_size_t, [P, P, P]),
        "purekv_stack_layer": (c_int, [P, P, P, c_int32, P, P, P, P, P, P, P, c_size_t, P]),
        "purekv_stack_select_compact": (c_int, [P, P, P, P, P, P, c_int64, P, P, P, c_int32, P, c_size_t, P]),
        "purekv_budget": (c_int32, [c_int32, c_int32, c_double]),
        "purekv_plan_kept_tile_flops": (c_double, [P]),
        "purekv_plan_mask_flops": (c_double, [P]),
        "purekv_calib_mfma": (c_int, [P, c_int, c_int, c_int32, P, P, P]),
        "purekv_calib_mfma_flops": (c_double, [P, c_int32]),
        "purekv_calib_tile_step": (c_int, [P, c_int, c_int32, P, P, P, P]),
        "purekv_calib_tile_step_flops": (c_double, [P, c_int32]),
        "purekv_strerror": (c_char_p, [c_int]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = _load()
EXPORTS = (
    "purekv_plan_create", "purekv_plan_create_host", "purekv_plan_destroy", "purekv_plan_create_heads",
    "purekv_plan_create_heads_host", "purekv_plan_create_window", "purekv_plan_create_window_host", "purekv_plan_counts",
    "purekv_plan_qtile_list", "purekv_plan_item", "purekv_plan_queue", "purekv_plan_steps", "purekv_spearman", "purekv_workspace_bytes", "purekv_workspace_init",
    "purekv_stack_workspace_init", "purekv_st_spattn_prefill", "purekv_st_spattn_prefill_vnorm", "purekv_topk_select_vnorm",
    "purekv_lowlayer_importance", "purekv_topk_select", "purekv_topk_select_static", "purekv_kv_compact", "purekv_kv_append",
    "purekv_decode_attn", "purekv_decode_step", "purekv_stack_workspace_bytes", "purekv_stack_layer",
    "purekv_stack_select_compact", "purekv_budget", "purekv_plan_kept_tile_flops", "purekv_plan_mask_flops",
    "purekv_calib_mfma", "purekv_calib_mfma_flops", "purekv_calib_tile_step", "purekv_calib_tile_step_flops",
    "purekv_strerror",
)


def raw() -> ctypes.CDLL:
    """The ctypes handle, for tests that call the C ABI with hand-made (possibly invalid) arguments."""
    return _lib


def purekv_strerror(status: int) -> str:
    return _lib.purekv_strerror(status).decode()


def purekv_budget(n: int, w: int, ratio: float) -> int:
    return int(_lib.purekv_budget(n, w, ratio))


def _check(status: int, where: str) -> None:
    if status != OK:
        raise PureKVError(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dev_bf16(t: torch.Tensor, name: str) -> torch.Tensor:
    if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous bf16 device tensor")
    return t


def _strided_bf16(t: torch.Tensor, name: str, heads: int, n: int, d: int, strides: Tuple[int, int]) -> torch.Tensor:
    """A (heads, n, d) bf16 device view whose head and token strides are the plan's and whose channels are contiguous."""
    if not (t.is_cuda and t.dtype == torch.bfloat16):
        raise TypeError(f"{name} must be a bf16 device tensor")
    if tuple(t.shape[-3:]) != (heads, n, d) or t.stride(-1) != 1 or (t.stride(-3), t.stride(-2)) != tuple(strides):
        raise TypeError(f"{name}: shape {tuple(t.shape)} / strides {t.stride()} do not match the plan "
                        f"(({heads}, {n}, {d}), head stride {strides[0]}, token stride {strides[1]}, channel stride 1)")
    return t


class Plan:
    """Owns a purekv_plan_t.  `host_only` plans can be inspected without a GPU but not launched."""

    def __init__(self, n_frames: int, patch_h: int, patch_w: int, n_text: int, n_q_heads: int, n_kv_heads: int,
                 head_dim: int, pattern: int = PATTERN_ST, softmax_scale: float = 0.0, host_only: bool = False,
                 n_workgroups: int = 256, head_mask=None, q_strides: Tuple[int, int] = (0, 0),
                 kv_strides: Tuple[int, int] = (0, 0), o_strides: Tuple[int, int] = (0, 0), lse_window: int = 0):
        """head_mask: optional sequence of n_q_heads truth values: the plan covers those query heads only.
        lse_window: w > 0 makes a window plan (the prefill writes the log-sum-exp of the last w rows only).
        q_strides, kv_strides, o_strides: (head stride, token stride) in elements of Q, of K and V, of O;
        (0, 0) = packed [H, N, d]."""
        self.shape = Shape(n_frames, patch_h, patch_w, n_text, n_q_heads, n_kv_heads, head_dim, pattern,
                           softmax_scale, q_strides[0], q_strides[1], kv_strides[0], kv_strides[1],
                           o_strides[0], o_strides[1])
        self._h = c_void_p()
        self.lse_window = lse_window
        if lse_window and head_mask is not None:
            raise ValueError("a window plan covers every head")
        if lse_window:
            if host_only:
                _check(_lib.purekv_plan_create_window_host(byref(self.shape), lse_window, n_workgroups, byref(self._h)),
                       "purekv_plan_create_window_host")
            else:
                _check(_lib.purekv_plan_create_window(byref(self.shape), lse_window, byref(self._h), _stream()),
                       "purekv_plan_create_window")
        elif head_mask is not None:
            if len(head_mask) != n_q_heads:
                raise ValueError("head_mask needs one entry per query head")
            hm = (ctypes.c_uint8 * n_q_heads)(*[1 if x else 0 for x in head_mask])
            if host_only:
                _check(_lib.purekv_plan_create_heads_host(byref(self.shape), hm, n_workgroups, byref(self._h)),
                       "purekv_plan_create_heads_host")
            else:
                _check(_lib.purekv_plan_create_heads(byref(self.shape), hm, byref(self._h), _stream()),
                       "purekv_plan_create_heads")
        elif host_only:
            _check(_lib.purekv_plan_create_host(byref(self.shape), n_workgroups, byref(self._h)),
                   "purekv_plan_create_host")
        else:
            _check(_lib.purekv_plan_create(byref(self.shape), byref(self._h), _stream()), "purekv_plan_create")
        self.N = n_frames * patch_h * patch_w + n_text
        self.Hq, self.Hkv, self.d = n_q_heads, n_kv_heads, head_dim
        packed = (self.N * head_dim, head_dim)
        self.q_strides = tuple(q_strides) if any(q_strides) else packed
        self.kv_strides = tuple(kv_strides) if any(kv_strides) else packed
        self.o_strides = tuple(o_strides) if any(o_strides) else packed
        self._ws = {}

    @classmethod
    def for_workload(cls, wl, pattern: int = PATTERN_ST, host_only: bool = False, n_workgroups: int = 256,
                     **more) -> "Plan":
        return cls(wl.n_frames, wl.patch_h, wl.patch_w, wl.n_text, wl.n_q_heads, wl.n_kv_heads, wl.head_dim,
                   pattern, 0.0, host_only, n_workgroups, **more)

    def empty_out(self, device) -> torch.Tensor:
        """An output tensor laid out by the plan's O strides, as a (Hq, N, d) view."""
        sh, st = self.o_strides
        span = (self.Hq - 1) * sh + (self.N - 1) * st + self.d
        return torch.empty(span, dtype=torch.bfloat16, device=device).as_strided((self.Hq, self.N, self.d), (sh, st, 1))

    @property
    def handle(self) -> c_void_p:
        return self._h

    def close(self) -> None:
        if self._h:
            _lib.purekv_plan_destroy(self._h)
            self._h = c_void_p()
        self._ws = {}

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- inspection -------------------------------------------------------------------------------
    def counts(self) -> dict:
        c = (c_int64 * 16)()
        _check(_lib.purekv_plan_counts(self._h, c), "purekv_plan_counts")
        return dict(N=c[0], n_qtiles=c[1], n_items=c[2], n_tile_refs=c[3], n_blocks=c[4], n_split_qtiles=c[5],
                    n_workgroups=c[6], row_blocks=c[7], stacked_heads=c[8], n_head_groups=c[9],
                    n_full_blocks=c[10], n_causal_blocks=c[11], n_prev_blocks=c[12], n_general_blocks=c[13],
                    lse_window=c[14], lse_queue0=c[15])

    def qtile_list(self, qt: int) -> list:
        """[(key tile, need bits, kind bits)] of query tile `qt`: need bit 2*rb + kb, kind bits 4*rb + 2*kb."""
        n = _lib.purekv_plan_qtile_list(self._h, qt, None, 0)
        if n < 0:
            raise PureKVError(n, "purekv_plan_qtile_list")
        buf = (c_int32 * max(3 * n, 1))()
        _lib.purekv_plan_qtile_list(self._h, qt, buf, n)
        return [(buf[3 * i], buf[3 * i + 1] & 0xFFFFFFFF, buf[3 * i + 2] & 0xFFFFFFFF) for i in range(n)]

    def queue(self, wg: int) -> list:
        """[(work item, first query head of the group)] run by persistent workgroup `wg`, in order."""
        n = _lib.purekv_plan_queue(self._h, wg, None, 0)
        if n < 0:
            raise PureKVError(n, "purekv_plan_queue")
        buf = (c_int32 * max(2 * n, 1))()
        _lib.purekv_plan_queue(self._h, wg, buf, n)
        return [(buf[2 * i], buf[2 * i + 1]) for i in range(n)]

    def steps(self, wg: int) -> list:
        """Steps of persistent workgroup `wg`, in order: (kv_off, need | flags, kinds, k0) each."""
        n = _lib.purekv_plan_steps(self._h, wg, None, 0)
        if n < 0:
            raise PureKVError(n, "purekv_plan_steps")
        buf = (c_int32 * max(4 * n, 1))()
        _lib.purekv_plan_steps(self._h, wg, buf, n)
        return [(buf[4 * i] & 0xFFFFFFFF, buf[4 * i + 1] & 0xFFFFFFFF, buf[4 * i + 2] & 0xFFFFFFFF, buf[4 * i + 3])
                for i in range(n)]

    def item(self, it: int) -> Tuple[int, ...]:
        buf = (c_int32 * 6)()
        _check(_lib.purekv_plan_item(self._h, it, buf), "purekv_plan_item")
        return tuple(buf)

    def kept_tile_flops(self) -> float:
        return float(_lib.purekv_plan_kept_tile_flops(self._h))

    def mask_flops(self) -> float:
        return float(_lib.purekv_plan_mask_flops(self._h))

    def workspace_bytes(self, op: int, n_layers: int = 0, w: int = 0, cap: int = 0) -> int:
        return int(_lib.purekv_workspace_bytes(self._h, op, n_layers, w, cap))

    def _workspace(self, op: int, nbytes: int, device, n_layers: int = 0, w: int = 0, cap: int = 0) -> Optional[torch.Tensor]:
        """Device scratch owned by the Python wrapper (torch memory), reused across calls on the stream that first
        used it (a buffer used from another stream gets a workspace of its own: concurrent calls must not share one).
        A new buffer is handed to purekv_workspace_init once."""
        if nbytes == 0:
            return None
        key = (op, torch.cuda.current_stream().cuda_stream)
        t = self._ws.get(key)
        if t is None or t.numel() < nbytes or t.device != device:
            t = torch.empty(nbytes, dtype=torch.uint8, device=device)
            self._ws[key] = t
            if op >= 0:
                _check(_lib.purekv_workspace_init(self._h, op, t.data_ptr(), nbytes, n_layers, w, cap, _stream()),
                       "purekv_workspace_init")
        return t


def purekv_st_spattn_prefill(plan: Plan, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                             out: Optional[torch.Tensor] = None, want_lse: bool = False,
                             lse: Optional[torch.Tensor] = None, vnorm2: Optional[torch.Tensor] = None):
    """vnorm2: optional fp32 [Hkv, N] output: the call becomes purekv_st_spattn_prefill_vnorm and fills it."""
    _strided_bf16(q, "q", plan.Hq, plan.N, plan.d, plan.q_strides)
    _strided_bf16(k, "k", plan.Hkv, plan.N, plan.d, plan.kv_strides)
    _strided_bf16(v, "v", plan.Hkv, plan.N, plan.d, plan.kv_strides)
    if out is None:
        out = plan.empty_out(q.device)
    _strided_bf16(out, "out", plan.Hq, plan.N, plan.d, plan.o_strides)
    if want_lse and lse is None:
        lse = torch.empty((plan.Hq, plan.N), dtype=torch.float32, device=q.device)
    nb = plan.workspace_bytes(OP_PREFILL)
    ws = plan._workspace(OP_PREFILL, nb, q.device)
    if vnorm2 is not None:
        assert vnorm2.dtype == torch.float32 and vnorm2.is_contiguous() and vnorm2.shape == (plan.Hkv, plan.N)
        _check(_lib.purekv_st_spattn_prefill_vnorm(plan.handle, q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                                                   _ptr(lse), vnorm2.data_ptr(), _ptr(ws), nb, _stream()),
               "purekv_st_spattn_prefill_vnorm")
    else:
        _check(_lib.purekv_st_spattn_prefill(plan.handle, q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                                             _ptr(lse), _ptr(ws), nb, _stream()), "purekv_st_spattn_prefill")
    return (out, lse) if (want_lse or lse is not None) else out


def purekv_lowlayer_importance(plan: Plan, q: torch.Tensor, k: torch.Tensor, lse: torch.Tensor, w: int,
                               c_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    _strided_bf16(q, "q", plan.Hq, plan.N, plan.d, plan.q_strides)
    _strided_bf16(k, "k", plan.Hkv, plan.N, plan.d, plan.kv_strides)
    assert lse.dtype == torch.float32 and lse.is_contiguous() and lse.shape == (plan.Hq, plan.N)
    if c_out is None:
        c_out = torch.empty((plan.Hkv, max(plan.N - w, 0)), dtype=torch.float32, device=q.device)
    _check(_lib.purekv_lowlayer_importance(plan.handle, q.data_ptr(), k.data_ptr(), lse.data_ptr(), w,
                                           c_out.data_ptr(), None, 0, _stream()), "purekv_lowlayer_importance")
    return c_out


def purekv_topk_select(plan: Plan, c: torch.Tensor, v: Optional[torch.Tensor], w: int, h: int,
                       want_scores: bool = False, idx_out: Optional[torch.Tensor] = None):
    """v: None, [Hkv, N, d] or [L, Hkv, N, d] (layers share c).  Returns idx [L, Hkv, h+w] (L squeezed when v has no
    layer axis) and, if asked, the scores."""
    assert c.dtype == torch.float32 and c.is_contiguous() and c.is_cuda
    layered = v is not None and v.dim() == 4
    n_layers = v.shape[0] if layered else 1
    stride = v.stride(0) if layered else 0
    if v is not None:
        _strided_bf16(v, "v", plan.Hkv, plan.N, plan.d, plan.kv_strides)
    if idx_out is None:
        idx_out = torch.empty((n_layers, plan.Hkv, h + w), dtype=torch.int32, device=c.device)
    s_out = torch.empty((n_layers, plan.Hkv, plan.N - w), dtype=torch.float32, device=c.device) if want_scores else None
    nb = plan.workspace_bytes(OP_TOPK, n_layers, w) if (v is not None and s_out is None) else 0
    ws = plan._workspace(OP_TOPK, nb, c.device)
    _check(_lib.purekv_topk_select(plan.handle, c.data_ptr(), _ptr(v), stride, n_layers, w, h, idx_out.data_ptr(),
                                   _ptr(s_out), _ptr(ws), nb, _stream()), "purekv_topk_select")
    if not layered:
        idx_out = idx_out[0]
        s_out = None if s_out is None else s_out[0]
    return (idx_out, s_out) if want_scores else idx_out


def purekv_topk_select_vnorm(plan: Plan, c: torch.Tensor, vnorm2: torch.Tensor, w: int, h: int,
                             want_scores: bool = False, idx_out: Optional[torch.Tensor] = None):
    """vnorm2: fp32 [Hkv, N] or [L, Hkv, N] (layers share c), as purekv_st_spattn_prefill_vnorm emits it."""
    assert c.dtype == torch.float32 and c.is_contiguous() and c.is_cuda
    assert vnorm2.dtype == torch.float32 and vnorm2.is_cuda and vnorm2.shape[-2:] == (plan.Hkv, plan.N)
    assert vnorm2[0].is_contiguous() if vnorm2.dim() == 3 else vnorm2.is_contiguous()
    layered = vnorm2.dim() == 3
    n_layers = vnorm2.shape[0] if layered else 1
    stride = vnorm2.stride(0) if layered else 0
    if idx_out is None:
        idx_out = torch.empty((n_layers, plan.Hkv, h + w), dtype=torch.int32, device=c.device)
    s_out = torch.empty((n_layers, plan.Hkv, plan.N - w), dtype=torch.float32, device=c.device) if want_scores else None
    nb = plan.workspace_bytes(OP_TOPK, n_layers, w) if s_out is None else 0
    ws = plan._workspace(OP_TOPK, nb, c.device)
    _check(_lib.purekv_topk_select_vnorm(plan.handle, c.data_ptr(), vnorm2.data_ptr(), stride, n_layers, w, h,
                                         idx_out.data_ptr(), _ptr(s_out), _ptr(ws), nb, _stream()),
           "purekv_topk_select_vnorm")
    if not layered:
        idx_out = idx_out[0]
        s_out = None if s_out is None else s_out[0]
    return (idx_out, s_out) if want_scores else idx_out


def purekv_topk_select_static(plan: Plan, c: torch.Tensor, v: Optional[torch.Tensor], w: int, h: int,
                              idx_out: torch.Tensor) -> torch.Tensor:
    """purekv_topk_select on the library's static score buffer: no workspace, and nothing is allocated here either
    (idx_out [L, Hkv, h+w] int32, or [Hkv, h+w] when v has no layer axis, is the caller's)."""
    assert c.dtype == torch.float32 and c.is_contiguous() and c.is_cuda
    assert idx_out.dtype == torch.int32 and idx_out.is_contiguous() and idx_out.is_cuda
    layered = v is not None and v.dim() == 4
    n_layers = v.shape[0] if layered else 1
    stride = v.stride(0) if layered else 0
    if v is not None:
        _strided_bf16(v, "v", plan.Hkv, plan.N, plan.d, plan.kv_strides)
    assert idx_out.numel() == n_layers * plan.Hkv * (h + w)
    _check(_lib.purekv_topk_select_static(plan.handle, c.data_ptr(), _ptr(v), stride, n_layers, w, h,
                                          idx_out.data_ptr(), _stream()), "purekv_topk_select_static")
    return idx_out


def purekv_spearman(s_hat: torch.Tensor, s: torch.Tensor):
    """s_hat, s: fp32 [..., n_keys] device tensors of one shape.  Returns (sum of squared rank differences, int64
    [...] -- exact, below 2^63 for n_keys <= 131072 -- and rho, fp64 [...])."""
    assert s_hat.shape == s.shape and s.dtype == torch.float32 and s_hat.dtype == torch.float32
    assert s.is_cuda and s_hat.is_cuda and s.is_contiguous() and s_hat.is_contiguous()
    n = s.shape[-1]
    rows = s.numel() // n if n else 0
    d2 = torch.empty(s.shape[:-1], dtype=torch.int64, device=s.device)
    rho = torch.empty(s.shape[:-1], dtype=torch.float64, device=s.device)
    _check(_lib.purekv_spearman(s_hat.data_ptr(), s.data_ptr(), rows, n, d2.data_ptr(), rho.data_ptr(), _stream()),
           "purekv_spearman")
    return d2, rho


def purekv_kv_compact(plan: Plan, k: torch.Tensor, v: torch.Tensor, idx: torch.Tensor, cap: Optional[int] = None,
                      kc: Optional[torch.Tensor] = None, vc: Optional[torch.Tensor] = None):
    """k, v: [Hkv, N, d] or [L, Hkv, N, d]; idx: [Hkv, n_keep] or [L, Hkv, n_keep] int32."""
    _strided_bf16(k, "k", plan.Hkv, plan.N, plan.d, plan.kv_strides)
    _strided_bf16(v, "v", plan.Hkv, plan.N, plan.d, plan.kv_strides)
    assert idx.dtype == torch.int32 and idx.is_contiguous() and idx.is_cuda
    layered = k.dim() == 4
    n_layers = k.shape[0] if layered else 1
    stride = k.stride(0) if layered else 0
    assert (not layered) or v.stride(0) == stride
    n_keep = idx.shape[-1]
    cap = n_keep if cap is None else cap
    shape = (n_layers, plan.Hkv, cap, plan.d) if layered else (plan.Hkv, cap, plan.d)
    if kc is None:
        kc = torch.empty(shape, dtype=torch.bfloat16, device=k.device)
    if vc is None:
        vc = torch.empty(shape, dtype=torch.bfloat16, device=k.device)
    _check(_lib.purekv_kv_compact(plan.handle, k.data_ptr(), v.data_ptr(), stride, n_layers, idx.data_ptr(), n_keep,
                                  kc.data_ptr(), vc.data_ptr(), cap, _stream()), "purekv_kv_compact")
    return kc, vc


def purekv_kv_append(plan: Plan, k_new: torch.Tensor, v_new: torch.Tensor, kc: torch.Tensor, vc: torch.Tensor,
                     n_cached: int) -> int:
    _dev_bf16(k_new, "k_new"), _dev_bf16(v_new, "v_new"), _dev_bf16(kc, "kc"), _dev_bf16(vc, "vc")
    cap = kc.shape[-2]
    _check(_lib.purekv_kv_append(plan.handle, k_new.data_ptr(), v_new.data_ptr(), kc.data_ptr(), vc.data_ptr(),
                                 n_cached, cap, _stream()), "purekv_kv_append")
    return n_cached + 1


def purekv_decode_attn(plan: Plan, q_new: torch.Tensor, kc: torch.Tensor, vc: torch.Tensor, n_cached: int,
                       out: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev_bf16(q_new, "q_new"), _dev_bf16(kc, "kc"), _dev_bf16(vc, "vc")
    cap = kc.shape[-2]
    if out is None:
        out = torch.empty_like(q_new)
    nb = plan.workspace_bytes(OP_DECODE, cap=cap)
    ws = plan._workspace(OP_DECODE, nb, q_new.device, cap=cap)
    _check(_lib.purekv_decode_attn(plan.handle, q_new.data_ptr(), kc.data_ptr(), vc.data_ptr(), n_cached, cap,
                                   out.data_ptr(), _ptr(ws), nb, _stream()), "purekv_decode_attn")
    return out


def purekv_decode_step(plan: Plan, q_new: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor, kc: torch.Tensor,
                       vc: torch.Tensor, n_cached: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Appends k_new, v_new as row n_cached of kc, vc and attends q_new over rows 0 .. n_cached, in one launch."""
    for t, name in ((q_new, "q_new"), (k_new, "k_new"), (v_new, "v_new"), (kc, "kc"), (vc, "vc")):
        _dev_bf16(t, name)
    cap = kc.shape[-2]
    if out is None:
        out = torch.empty_like(q_new)
    nb = plan.workspace_bytes(OP_DECODE, cap=cap)
    ws = plan._workspace(OP_DECODE, nb, q_new.device, cap=cap)
    _check(_lib.purekv_decode_step(plan.handle, q_new.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), kc.data_ptr(),
                                   vc.data_ptr(), n_cached, cap, out.data_ptr(), _ptr(ws), nb, _stream()),
           "purekv_decode_step")
    return out


class Stack(ctypes.Structure):
    """purekv_stack_t: which layer runs which attention and whose C drives whose selection."""
    _fields_ = [("n_layers", c_int32), ("clie_layer", c_int32), ("st_layer", c_int32), ("w", c_int32), ("h", c_int32)]


def _stack_ws(dense: Plan, st: Optional[Plan], stack: Stack, device) -> tuple:
    sth = st.handle if st is not None else None
    nb = int(_lib.purekv_stack_workspace_bytes(dense.handle, sth, byref(stack)))
    if nb == 0:
        return 0, None
    key = (-1, torch.cuda.current_stream().cuda_stream, int(st._h.value or 0) if st is not None else 0,
           stack.n_layers, stack.clie_layer, stack.st_layer, stack.w)
    t = dense._ws.get(key)
    if t is None or t.numel() < nb or t.device != device:
        t = torch.empty(nb, dtype=torch.uint8, device=device)
        dense._ws[key] = t
        _check(_lib.purekv_stack_workspace_init(dense.handle, sth, byref(stack), t.data_ptr(), nb, _stream()),
               "purekv_stack_workspace_init")
    return nb, t


def purekv_stack_layer(dense: Plan, st: Optional[Plan], stack: Stack, layer: int, q: torch.Tensor, k: torch.Tensor,
                       v: torch.Tensor, out: torch.Tensor, lse: Optional[torch.Tensor], c_all: Optional[torch.Tensor]):
    """One layer of the stack's prefill (plus importance on the layers that emit C)."""
    _strided_bf16(q, "q", dense.Hq, dense.N, dense.d, dense.q_strides)
    _strided_bf16(k, "k", dense.Hkv, dense.N, dense.d, dense.kv_strides)
    _strided_bf16(v, "v", dense.Hkv, dense.N, dense.d, dense.kv_strides)
    _strided_bf16(out, "out", dense.Hq, dense.N, dense.d, dense.o_strides)
    nb, ws = _stack_ws(dense, st, stack, q.device)
    _check(_lib.purekv_stack_layer(dense.handle, st.handle if st is not None else None, byref(stack), layer,
                                   q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), _ptr(lse), _ptr(c_all),
                                   _ptr(ws), nb, _stream()), "purekv_stack_layer")
    return out


def purekv_stack_select_compact(dense: Plan, st: Optional[Plan], stack: Stack, c_all: torch.Tensor, k_all: torch.Tensor,
                                v_all: torch.Tensor, idx_all: torch.Tensor, kc_all: torch.Tensor, vc_all: torch.Tensor):
    """Selection and compaction of all layers of the stack; k_all, v_all [L, Hkv, N, d], kc_all, vc_all [L, Hkv, cap, d]."""
    _strided_bf16(k_all, "k_all", dense.Hkv, dense.N, dense.d, dense.kv_strides)
    _strided_bf16(v_all, "v_all", dense.Hkv, dense.N, dense.d, dense.kv_strides)
    _dev_bf16(kc_all, "kc_all"), _dev_bf16(vc_all, "vc_all")
    assert k_all.dim() == 4 and v_all.stride(0) == k_all.stride(0)
    nb, ws = _stack_ws(dense, st, stack, k_all.device)
    _check(_lib.purekv_stack_select_compact(dense.handle, st.handle if st is not None else None, byref(stack), _ptr(c_all), k_all.data_ptr(), v_all.data_ptr(),
                                            k_all.stride(0), idx_all.data_ptr(), kc_all.data_ptr(), vc_all.data_ptr(),
                                            kc_all.shape[-2], _ptr(ws), nb, _stream()), "purekv_stack_select_compact")
    return idx_all, kc_all, vc_all


def purekv_calib_mfma(plan: Plan, mix: int, random_operands: bool, iters: int,
                      sink: Optional[torch.Tensor] = None, ticks: Optional[torch.Tensor] = None):
    """Launches the board-calibration loop once on the current stream (asynchronous).  Returns (flops of the launch,
    ticks): ticks is an int64 device tensor [2], shader cycles and 100 MHz ticks of wavefront 0, valid once the
    stream has been synchronised.  Time the call with events around it."""
    dev = torch.device("cuda", torch.cuda.current_device())
    if sink is None:
        sink = torch.empty(512 * plan.counts()["n_workgroups"], dtype=torch.float32, device=dev)
    if ticks is None:
        ticks = torch.zeros(2, dtype=torch.int64, device=dev)
    _check(_lib.purekv_calib_mfma(plan.handle, mix, int(bool(random_operands)), iters, sink.data_ptr(),
                                  ticks.data_ptr(), _stream()), "purekv_calib_mfma")
    return float(_lib.purekv_calib_mfma_flops(plan.handle, iters)), ticks


def purekv_calib_tile_step(plan: Plan, rows_per_wavefront: int, iters: int, src: torch.Tensor,
                           sink: Optional[torch.Tensor] = None, ticks: Optional[torch.Tensor] = None):
    """Launches the tile-step skeleton once on the current stream (asynchronous).  `src`: bf16 device tensor of at
    least 4 MiB of finite values.  Returns (flops of the launch, ticks) like purekv_calib_mfma."""
    _dev_bf16(src, "src")
    if src.numel() * 2 < (4 << 20):
        raise ValueError("src must hold at least 4 MiB")
    dev = src.device
    if sink is None:
        sink = torch.empty(512 * plan.counts()["n_workgroups"], dtype=torch.float32, device=dev)
    if ticks is None:
        ticks = torch.zeros(2, dtype=torch.int64, device=dev)
    _check(_lib.purekv_calib_tile_step(plan.handle, rows_per_wavefront, iters, src.data_ptr(), sink.data_ptr(),
                                       ticks.data_ptr(), _stream()), "purekv_calib_tile_step")
    return float(_lib.purekv_calib_tile_step_flops(plan.handle, iters)), ticks
