"""Python binding of libsdl.so, the MI355X-native Streaming DiLoCo fragment outer step.

Argument marshalling only: every function has the name and the meaning of the C entry
point declared in include/sdl.h, takes torch tensors (device memory) where the C call
takes device pointers, and raises SdlError on a non-zero status.  All arithmetic runs
in the HIP kernels of the library; there is no Python or CPU fallback, and importing
this module fails loudly if the library has not been built
(``python paper_2501_18512_amd/build.py``).
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

FMT_FP32, FMT_BF16, FMT_E4M3, FMT_E3M0 = 0, 1, 2, 3
FMT_E3M0_B64, FMT_E3M0_B128, FMT_E3M0_SPAN, FMT_E3M0_RN = 4, 5, 6, 7
FORMATS = {"fp32": FMT_FP32, "bf16": FMT_BF16, "e4m3": FMT_E4M3, "e3m0": FMT_E3M0,
           "e3m0_b64": FMT_E3M0_B64, "e3m0_b128": FMT_E3M0_B128, "e3m0_span": FMT_E3M0_SPAN,
           "e3m0_rn": FMT_E3M0_RN}
PATTERN_STRIDED, PATTERN_SEQUENTIAL = 0, 1
UNIT_PRE, UNIT_POST = -1, -2
MAX_WORKERS = 16
BLOCK = 32

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsdl.so")


class SdlError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {_lib.sdl_status_string(status).decode()} (status {status})")


class _Span(ctypes.Structure):
    _fields_ = [("offset", ctypes.c_uint64), ("numel", ctypes.c_uint64), ("unit", ctypes.c_int32)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2501_18512_amd/build.py` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, u32, u64, f32 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float
    pp = ctypes.POINTER(ctypes.c_void_p)
    lib.sdl_fragment_plan.argtypes = [ctypes.POINTER(u64), ctypes.POINTER(ctypes.c_int32), u32, u32, u32,
                                      ctypes.c_int, u32, u32, ctypes.POINTER(u32), ctypes.POINTER(vp)]
    lib.sdl_fragment_plan_ex.argtypes = [ctypes.POINTER(u64), ctypes.POINTER(ctypes.c_int32), u32, u32, u32,
                                         ctypes.c_int, u32, u32, ctypes.POINTER(u32), u32, ctypes.POINTER(vp)]
    lib.sdl_plan_destroy.argtypes = [vp]
    lib.sdl_plan_destroy.restype = None
    lib.sdl_plan_num_fragments.argtypes = [vp]
    lib.sdl_plan_num_fragments.restype = u32
    lib.sdl_plan_total_numel.argtypes = [vp]
    lib.sdl_plan_total_numel.restype = u64
    lib.sdl_plan_block_fragment.argtypes = [vp, u32]
    for name in ("sdl_plan_fragment_spans", "sdl_plan_fragment_runs"):
        getattr(lib, name).argtypes = [vp, u32, ctypes.POINTER(ctypes.POINTER(_Span)), ctypes.POINTER(u32)]
    lib.sdl_plan_offset.argtypes = [vp, u32, ctypes.POINTER(u32)]
    lib.sdl_plan_events.argtypes = [vp, u64, ctypes.POINTER(u32), ctypes.POINTER(u32),
                                    ctypes.POINTER(u32), ctypes.POINTER(u32)]
    lib.sdl_exchange_bytes.argtypes = [ctypes.c_int, u64, ctypes.POINTER(ctypes.c_size_t),
                                       ctypes.POINTER(ctypes.c_size_t)]
    lib.sdl_exchange_bytes.restype = ctypes.c_size_t
    lib.sdl_quantize_outer_grad.argtypes = [vp, pp, u32, u64, ctypes.c_int, pp, pp, vp]
    lib.sdl_dequant_reduce_nesterov.argtypes = [vp, vp, pp, pp, u32, u64, ctypes.c_int, f32, f32, vp]
    lib.sdl_merge_overlap.argtypes = [vp, pp, u32, u64, f32, vp]
    lib.sdl_fragment_outer_step.argtypes = [vp, vp, pp, pp, u32, u64, ctypes.c_int, f32, f32, f32,
                                            pp, pp, vp]
    lib.sdl_fragment_outer_step_plan.argtypes = [vp, u32, vp, vp, pp, pp, u32, ctypes.c_int, f32, f32,
                                                 f32, vp]
    lib.sdl_plan_message_bytes.argtypes = [vp, u32, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t),
                                           ctypes.POINTER(ctypes.c_size_t)]
    lib.sdl_quantize_outer_grad_plan.argtypes = [vp, u32, vp, pp, u32, ctypes.c_int, pp, pp, vp]
    lib.sdl_dequant_reduce_nesterov_plan.argtypes = [vp, u32, vp, vp, pp, pp, u32, ctypes.c_int, f32, f32, vp]
    lib.sdl_merge_overlap_plan.argtypes = [vp, u32, vp, pp, u32, f32, vp]
    lib.sdl_engine_create.argtypes = [vp, u32, u32, ctypes.POINTER(u32), ctypes.c_int, f32, f32, f32,
                                      ctypes.POINTER(vp)]
    lib.sdl_engine_destroy.argtypes = [vp]
    lib.sdl_engine_destroy.restype = None
    lib.sdl_engine_bind.argtypes = [vp, vp, vp, pp, pp, pp]
    lib.sdl_engine_step.argtypes = [vp, u64, vp, ctypes.POINTER(u32), ctypes.POINTER(u32)]
    lib.sdl_receive_outer_step.argtypes = [vp, vp, pp, pp, pp, u32, u64, ctypes.c_int, f32, f32, f32, vp]
    lib.sdl_receive_outer_step_plan.argtypes = [vp, u32, vp, vp, pp, pp, pp, u32, ctypes.c_int, f32, f32, f32, vp]
    lib.sdl_receive_outer_step_staged.argtypes = lib.sdl_receive_outer_step_plan.argtypes
    lib.sdl_plan_staged_numel.argtypes = [vp, u32]
    lib.sdl_plan_staged_numel.restype = u64
    lib.sdl_fragment_outer_step_staged.argtypes = lib.sdl_fragment_outer_step_plan.argtypes
    lib.sdl_fragment_outer_step_plan_ex.argtypes = [vp, u32, vp, vp, pp, pp, u32, ctypes.c_int, f32, f32, f32, pp, pp, vp]
    lib.sdl_fragment_outer_step_staged_ex.argtypes = lib.sdl_fragment_outer_step_plan_ex.argtypes
    lib.sdl_fragment_outer_step_plan_static.argtypes = lib.sdl_fragment_outer_step_plan.argtypes
    lib.sdl_quantize_outer_grad_staged.argtypes = lib.sdl_quantize_outer_grad_plan.argtypes
    lib.sdl_dequant_reduce_nesterov_staged.argtypes = lib.sdl_dequant_reduce_nesterov_plan.argtypes
    lib.sdl_merge_overlap_staged.argtypes = lib.sdl_merge_overlap_plan.argtypes
    lib.sdl_offload_create.argtypes = [vp, u32, ctypes.POINTER(vp)]
    lib.sdl_offload_destroy.argtypes = [vp]
    lib.sdl_offload_destroy.restype = None
    lib.sdl_offload_slot_numel.argtypes = [vp]
    lib.sdl_offload_slot_numel.restype = u64
    lib.sdl_offload_num_slots.argtypes = [vp]
    lib.sdl_offload_num_slots.restype = u32
    lib.sdl_offload_bind.argtypes = [vp, vp, vp, pp, pp]
    lib.sdl_offload_resident.argtypes = [vp, u32]
    lib.sdl_offload_prefetch.argtypes = [vp, u32, vp]
    lib.sdl_offload_acquire.argtypes = [vp, u32, vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp)]
    lib.sdl_offload_release.argtypes = [vp, u32, vp, vp]
    lib.sdl_offload_flush.argtypes = [vp, vp, vp]
    lib.sdl_engine_bind_offload.argtypes = [vp, vp, pp, pp, pp, vp, u32]
    lib.sdl_copy_bytes.argtypes = [vp, vp, u64, vp]
    lib.sdl_memory_probe.argtypes = [ctypes.c_int, vp, vp, u64, vp]
    lib.sdl_flat_layout.argtypes = [u64, u32, ctypes.c_int, ctypes.POINTER(u64), ctypes.POINTER(u64)]
    lib.sdl_engine_track_cosine.argtypes = [vp, pp, vp, vp, ctypes.c_size_t]
    lib.sdl_evaluation_params.argtypes = [ctypes.c_int, vp, pp, u32, u64, vp, vp]
    lib.sdl_cosine_workspace_bytes.argtypes = [u32, u32]
    lib.sdl_cosine_workspace_bytes.restype = ctypes.c_size_t
    lib.sdl_outer_grad_cosine.argtypes = [vp, pp, u32, u64, vp, vp, ctypes.c_size_t, vp]
    lib.sdl_outer_grad_cosine_plan.argtypes = [vp, u32, vp, pp, u32, vp, vp, vp, ctypes.c_size_t, vp]
    lib.sdl_cosine_combine.argtypes = [vp, u64, u32, u32, vp, vp]
    lib.sdl_status_string.argtypes = [ctypes.c_int]
    lib.sdl_status_string.restype = ctypes.c_char_p
    return lib


_lib = _load()


def _check(status: int, where: str):
    if status != 0:
        raise SdlError(status, where)


def _ptr(t) -> int:
    """Device address of a tensor (or a raw integer address, passed through)."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _ptr_array(ts: Optional[Sequence]):
    if ts is None:
        return None
    return (ctypes.c_void_p * len(ts))(*[_ptr(t) for t in ts])


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _require_device(*tensors):
    for t in tensors:
        if isinstance(t, torch.Tensor):
            if not t.is_cuda:
                raise ValueError("sdl calls take device tensors; there is no CPU path")
            if not t.is_contiguous():
                raise ValueError("sdl calls take contiguous tensors")


# ------------------------------------------------------------------------------ plan

class Plan:
    """Owner of an sdl_plan_t handle."""

    def __init__(self, handle: int):
        self._h = ctypes.c_void_p(handle)

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.sdl_plan_destroy(self._h)
            self._h = None

    @property
    def num_fragments(self) -> int:
        return _lib.sdl_plan_num_fragments(self._h)

    @property
    def total_numel(self) -> int:
        return _lib.sdl_plan_total_numel(self._h)


PLAN_PRE_OWN_FRAGMENT = 1
PLAN_ALIGN_GROUPS = 2
PLAN_GROUP_ALIGN = 64


def sdl_fragment_plan_ex(unit_numel: Sequence[int], unit_block: Sequence[int], n_blocks: int, P: int,
                         pattern: int = PATTERN_STRIDED, H: int = 100, tau: int = 0,
                         t_p: Optional[Sequence[int]] = None, flags: int = 0) -> Plan:
    n = len(unit_numel)
    assert len(unit_block) == n
    numel = (ctypes.c_uint64 * n)(*unit_numel)
    block = (ctypes.c_int32 * n)(*unit_block)
    offs = None if t_p is None else (ctypes.c_uint32 * len(t_p))(*t_p)
    n_frag = P + (1 if flags & PLAN_PRE_OWN_FRAGMENT else 0)
    if t_p is not None and len(t_p) != n_frag:
        raise SdlError(-1, "sdl_fragment_plan_ex")
    out = ctypes.c_void_p()
    _check(_lib.sdl_fragment_plan_ex(numel, block, n, n_blocks, P, pattern, H, tau, offs, flags,
                                     ctypes.byref(out)), "sdl_fragment_plan_ex")
    return Plan(out.value)


def sdl_fragment_plan(unit_numel: Sequence[int], unit_block: Sequence[int], n_blocks: int, P: int,
                      pattern: int = PATTERN_STRIDED, H: int = 100, tau: int = 0,
                      t_p: Optional[Sequence[int]] = None) -> Plan:
    n = len(unit_numel)
    assert len(unit_block) == n
    numel = (ctypes.c_uint64 * n)(*unit_numel)
    block = (ctypes.c_int32 * n)(*unit_block)
    offs = None if t_p is None else (ctypes.c_uint32 * len(t_p))(*t_p)
    if t_p is not None and len(t_p) != P:
        raise SdlError(-1, "sdl_fragment_plan")
    out = ctypes.c_void_p()
    _check(_lib.sdl_fragment_plan(numel, block, n, n_blocks, P, pattern, H, tau, offs,
                                  ctypes.byref(out)), "sdl_fragment_plan")
    return Plan(out.value)


def _span_list(fn, plan: Plan, p: int) -> List[Tuple[int, int, int]]:
    arr = ctypes.POINTER(_Span)()
    n = ctypes.c_uint32()
    _check(fn(plan._h, p, ctypes.byref(arr), ctypes.byref(n)), fn.__name__)
    return [(arr[i].offset, arr[i].numel, arr[i].unit) for i in range(n.value)]


def sdl_plan_fragment_spans(plan: Plan, p: int):
    return _span_list(_lib.sdl_plan_fragment_spans, plan, p)


def sdl_plan_fragment_runs(plan: Plan, p: int):
    return _span_list(_lib.sdl_plan_fragment_runs, plan, p)


def sdl_plan_block_fragment(plan: Plan, block: int) -> int:
    rc = _lib.sdl_plan_block_fragment(plan._h, block)
    if rc < 0:
        raise SdlError(rc, "sdl_plan_block_fragment")
    return rc


def sdl_plan_offset(plan: Plan, p: int) -> int:
    out = ctypes.c_uint32()
    _check(_lib.sdl_plan_offset(plan._h, p, ctypes.byref(out)), "sdl_plan_offset")
    return out.value


def sdl_plan_events(plan: Plan, t: int) -> Tuple[List[int], List[int]]:
    P = plan.num_fragments
    send, recv = (ctypes.c_uint32 * P)(), (ctypes.c_uint32 * P)()
    ns, nr = ctypes.c_uint32(), ctypes.c_uint32()
    _check(_lib.sdl_plan_events(plan._h, t, send, ctypes.byref(ns), recv, ctypes.byref(nr)),
           "sdl_plan_events")
    return list(send[:ns.value]), list(recv[:nr.value])


def sdl_exchange_bytes(fmt: int, numel: int) -> Tuple[int, int]:
    c, s = ctypes.c_size_t(), ctypes.c_size_t()
    _lib.sdl_exchange_bytes(fmt, numel, ctypes.byref(c), ctypes.byref(s))
    return c.value, s.value


# ------------------------------------------------------------------------ device calls

def sdl_quantize_outer_grad(g, w_send, n: int, fmt: int, codes, scales=None, stream=None):
    _require_device(g, *w_send, *codes, *(scales or []))
    _check(_lib.sdl_quantize_outer_grad(_ptr(g), _ptr_array(w_send), len(w_send), n, fmt,
                                        _ptr_array(codes), _ptr_array(scales), _stream(stream)),
           "sdl_quantize_outer_grad")


def sdl_dequant_reduce_nesterov(g, mom, codes, scales, n: int, fmt: int, lr: float, mu: float,
                                stream=None):
    _require_device(g, mom, *codes, *(scales or []))
    _check(_lib.sdl_dequant_reduce_nesterov(_ptr(g), _ptr(mom), _ptr_array(codes), _ptr_array(scales),
                                            len(codes), n, fmt, lr, mu, _stream(stream)),
           "sdl_dequant_reduce_nesterov")


def sdl_merge_overlap(g_new, w_now, n: int, alpha: float, stream=None):
    _require_device(g_new, *w_now)
    _check(_lib.sdl_merge_overlap(_ptr(g_new), _ptr_array(w_now), len(w_now), n, alpha,
                                  _stream(stream)), "sdl_merge_overlap")


def sdl_receive_outer_step(g, mom, codes, scales, w_now, n: int, fmt: int, lr: float, mu: float, alpha: float,
                           stream=None):
    _require_device(g, mom, *codes, *(scales or []), *w_now)
    if len(codes) != len(w_now):
        raise SdlError(-1, "sdl_receive_outer_step")
    _check(_lib.sdl_receive_outer_step(_ptr(g), _ptr(mom), _ptr_array(codes), _ptr_array(scales),
                                       _ptr_array(w_now), len(w_now), n, fmt, lr, mu, alpha, _stream(stream)),
           "sdl_receive_outer_step")


def sdl_receive_outer_step_plan(plan: "Plan", p: int, g_base, mom_base, codes, scales, w_now_base, fmt: int,
                                lr: float, mu: float, alpha: float, stream=None):
    _require_device(g_base, mom_base, *codes, *(scales or []), *w_now_base)
    _check(_lib.sdl_receive_outer_step_plan(plan._h, p, _ptr(g_base), _ptr(mom_base), _ptr_array(codes),
                                            _ptr_array(scales), _ptr_array(w_now_base), len(w_now_base), fmt, lr,
                                            mu, alpha, _stream(stream)), "sdl_receive_outer_step_plan")


def sdl_fragment_outer_step(g, mom, w_send, w_now, n: int, fmt: int, lr: float, mu: float,
                            alpha: float, codes=None, scales=None, stream=None):
    _require_device(g, mom, *w_send, *w_now, *(codes or []), *(scales or []))
    if len(w_send) != len(w_now):
        raise SdlError(-1, "sdl_fragment_outer_step")
    _check(_lib.sdl_fragment_outer_step(_ptr(g), _ptr(mom), _ptr_array(w_send), _ptr_array(w_now),
                                        len(w_send), n, fmt, lr, mu, alpha, _ptr_array(codes),
                                        _ptr_array(scales), _stream(stream)),
           "sdl_fragment_outer_step")


def sdl_fragment_outer_step_plan(plan: Plan, p: int, g_base, mom_base, w_send_base, w_now_base,
                                 fmt: int, lr: float, mu: float, alpha: float, stream=None):
    _require_device(g_base, mom_base, *w_send_base, *w_now_base)
    if len(w_send_base) != len(w_now_base):
        raise SdlError(-1, "sdl_fragment_outer_step_plan")
    _check(_lib.sdl_fragment_outer_step_plan(plan._h, p, _ptr(g_base), _ptr(mom_base),
                                             _ptr_array(w_send_base), _ptr_array(w_now_base),
                                             len(w_send_base), fmt, lr, mu, alpha, _stream(stream)),
           "sdl_fragment_outer_step_plan")


STATIC_MAX_SPANS = 1024


def sdl_fragment_outer_step_plan_static(plan: Plan, p: int, g_base, mom_base, w_send_base, w_now_base,
                                        fmt: int, lr: float, mu: float, alpha: float, stream=None):
    _require_device(g_base, mom_base, *w_send_base, *w_now_base)
    if len(w_send_base) != len(w_now_base):
        raise SdlError(-1, "sdl_fragment_outer_step_plan_static")
    _check(_lib.sdl_fragment_outer_step_plan_static(plan._h, p, _ptr(g_base), _ptr(mom_base),
                                                    _ptr_array(w_send_base), _ptr_array(w_now_base),
                                                    len(w_send_base), fmt, lr, mu, alpha, _stream(stream)),
           "sdl_fragment_outer_step_plan_static")


def sdl_fragment_outer_step_plan_ex(plan: Plan, p: int, g_base, mom_base, w_send_base, w_now_base,
                                    fmt: int, lr: float, mu: float, alpha: float, codes=None, scales=None,
                                    stream=None):
    _require_device(g_base, mom_base, *w_send_base, *w_now_base, *(codes or []), *(scales or []))
    if len(w_send_base) != len(w_now_base):
        raise SdlError(-1, "sdl_fragment_outer_step_plan_ex")
    _check(_lib.sdl_fragment_outer_step_plan_ex(plan._h, p, _ptr(g_base), _ptr(mom_base),
                                                _ptr_array(w_send_base), _ptr_array(w_now_base),
                                                len(w_send_base), fmt, lr, mu, alpha, _ptr_array(codes),
                                                _ptr_array(scales), _stream(stream)),
           "sdl_fragment_outer_step_plan_ex")


def sdl_fragment_outer_step_staged_ex(plan: Plan, p: int, g_frag, mom_frag, w_send_base, w_now_base,
                                      fmt: int, lr: float, mu: float, alpha: float, codes=None, scales=None,
                                      stream=None):
    _require_device(g_frag, mom_frag, *w_send_base, *w_now_base, *(codes or []), *(scales or []))
    _check(_lib.sdl_fragment_outer_step_staged_ex(plan._h, p, _ptr(g_frag), _ptr(mom_frag),
                                                  _ptr_array(w_send_base), _ptr_array(w_now_base),
                                                  len(w_send_base), fmt, lr, mu, alpha, _ptr_array(codes),
                                                  _ptr_array(scales), _stream(stream)),
           "sdl_fragment_outer_step_staged_ex")


def sdl_plan_message_bytes(plan: Plan, p: int, fmt: int) -> Tuple[int, int]:
    c, s = ctypes.c_size_t(), ctypes.c_size_t()
    _check(_lib.sdl_plan_message_bytes(plan._h, p, fmt, ctypes.byref(c), ctypes.byref(s)),
           "sdl_plan_message_bytes")
    return c.value, s.value


def sdl_quantize_outer_grad_plan(plan: Plan, p: int, g_base, w_send_base, fmt: int, codes, scales=None,
                                 stream=None):
    _require_device(g_base, *w_send_base, *codes, *(scales or []))
    _check(_lib.sdl_quantize_outer_grad_plan(plan._h, p, _ptr(g_base), _ptr_array(w_send_base),
                                             len(w_send_base), fmt, _ptr_array(codes), _ptr_array(scales),
                                             _stream(stream)), "sdl_quantize_outer_grad_plan")


def sdl_dequant_reduce_nesterov_plan(plan: Plan, p: int, g_base, mom_base, codes, scales, fmt: int, lr: float,
                                     mu: float, stream=None):
    _require_device(g_base, mom_base, *codes, *(scales or []))
    _check(_lib.sdl_dequant_reduce_nesterov_plan(plan._h, p, _ptr(g_base), _ptr(mom_base), _ptr_array(codes),
                                                 _ptr_array(scales), len(codes), fmt, lr, mu, _stream(stream)),
           "sdl_dequant_reduce_nesterov_plan")


def sdl_merge_overlap_plan(plan: Plan, p: int, g_new_base, w_now_base, alpha: float, stream=None):
    _require_device(g_new_base, *w_now_base)
    _check(_lib.sdl_merge_overlap_plan(plan._h, p, _ptr(g_new_base), _ptr_array(w_now_base), len(w_now_base),
                                       alpha, _stream(stream)), "sdl_merge_overlap_plan")


class Engine:
    """Owner of an sdl_engine_t handle (keeps the plan and the bound tensors alive)."""

    def __init__(self, handle: int, plan: Plan):
        self._h = ctypes.c_void_p(handle)
        self._plan = plan
        self._keep = None

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.sdl_engine_destroy(self._h)
            self._h = None


def sdl_engine_create(plan: Plan, H: int, tau_m: Sequence[int], fmt: int, lr: float, mu: float,
                      alpha: float) -> Engine:
    taus = (ctypes.c_uint32 * len(tau_m))(*tau_m)
    out = ctypes.c_void_p()
    _check(_lib.sdl_engine_create(plan._h, H, len(tau_m), taus, fmt, lr, mu, alpha, ctypes.byref(out)),
           "sdl_engine_create")
    return Engine(out.value, plan)


def sdl_engine_bind(engine: Engine, g_base, mom_base, w_base, codes=None, scales=None):
    """codes / scales: flat lists of P*M tensors, entry p*M + m."""
    _require_device(g_base, mom_base, *w_base, *(codes or []), *(scales or []))
    _check(_lib.sdl_engine_bind(engine._h, _ptr(g_base), _ptr(mom_base), _ptr_array(w_base), _ptr_array(codes),
                                _ptr_array(scales)), "sdl_engine_bind")
    engine._keep = (g_base, mom_base, list(w_base), codes, scales)


def sdl_engine_step(engine: Engine, t: int, stream=None) -> Tuple[int, int]:
    ns, nr = ctypes.c_uint32(), ctypes.c_uint32()
    _check(_lib.sdl_engine_step(engine._h, t, _stream(stream), ctypes.byref(ns), ctypes.byref(nr)),
           "sdl_engine_step")
    return ns.value, nr.value


# ------------------------------------------------------------- outer state in host memory

def sdl_plan_staged_numel(plan: Plan, p: int) -> int:
    return _lib.sdl_plan_staged_numel(plan._h, p)


def sdl_fragment_outer_step_staged(plan: Plan, p: int, g_frag, mom_frag, w_send_base, w_now_base, fmt: int,
                                   lr: float, mu: float, alpha: float, stream=None):
    _require_device(g_frag, mom_frag, *w_send_base, *w_now_base)
    _check(_lib.sdl_fragment_outer_step_staged(plan._h, p, _ptr(g_frag), _ptr(mom_frag), _ptr_array(w_send_base),
                                               _ptr_array(w_now_base), len(w_send_base), fmt, lr, mu, alpha,
                                               _stream(stream)), "sdl_fragment_outer_step_staged")


class Offload:
    """Owner of an sdl_offload_t handle (keeps the plan and the bound tensors alive)."""

    def __init__(self, handle: int, plan: Plan):
        self._h = ctypes.c_void_p(handle)
        self._plan = plan
        self._keep = None

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.sdl_offload_destroy(self._h)
            self._h = None

    @property
    def slot_numel(self) -> int:
        return _lib.sdl_offload_slot_numel(self._h)


def sdl_offload_create(plan: Plan, n_slots: int) -> Offload:
    out = ctypes.c_void_p()
    _check(_lib.sdl_offload_create(plan._h, n_slots, ctypes.byref(out)), "sdl_offload_create")
    return Offload(out.value, plan)


def sdl_offload_bind(pool: Offload, g_host, mom_host, slot_g, slot_mom):
    """g_host / mom_host: host tensors (pinned for asynchronous copies); slot_*: device tensors."""
    for t in (g_host, mom_host):
        if isinstance(t, torch.Tensor) and (t.is_cuda or not t.is_contiguous()):
            raise ValueError("the offloaded outer state lives in contiguous host tensors")
    _require_device(*slot_g, *slot_mom)
    _check(_lib.sdl_offload_bind(pool._h, _ptr(g_host), _ptr(mom_host), _ptr_array(slot_g), _ptr_array(slot_mom)),
           "sdl_offload_bind")
    pool._keep = (g_host, mom_host, list(slot_g), list(slot_mom))


def sdl_offload_resident(pool: Offload, p: int) -> bool:
    rc = _lib.sdl_offload_resident(pool._h, p)
    if rc < 0:
        raise SdlError(rc, "sdl_offload_resident")
    return bool(rc)


def sdl_offload_prefetch(pool: Offload, p: int, copy_stream):
    _check(_lib.sdl_offload_prefetch(pool._h, p, _stream(copy_stream)), "sdl_offload_prefetch")


def sdl_offload_acquire(pool: Offload, p: int, copy_stream, stream=None) -> Tuple[int, int]:
    """Returns the device addresses (g_frag, mom_frag) of the slot that holds fragment p."""
    g, m = ctypes.c_void_p(), ctypes.c_void_p()
    _check(_lib.sdl_offload_acquire(pool._h, p, _stream(stream), _stream(copy_stream), ctypes.byref(g),
                                    ctypes.byref(m)), "sdl_offload_acquire")
    return g.value, m.value


def sdl_offload_release(pool: Offload, p: int, copy_stream, stream=None):
    _check(_lib.sdl_offload_release(pool._h, p, _stream(stream), _stream(copy_stream)), "sdl_offload_release")


def sdl_offload_flush(pool: Offload, copy_stream, stream=None):
    _check(_lib.sdl_offload_flush(pool._h, _stream(stream), _stream(copy_stream)), "sdl_offload_flush")


def sdl_engine_bind_offload(engine: Engine, pool: Offload, w_base, codes=None, scales=None, copy_stream=None,
                            lookahead: int = 1):
    _require_device(*w_base, *(codes or []), *(scales or []))
    _check(_lib.sdl_engine_bind_offload(engine._h, pool._h, _ptr_array(w_base), _ptr_array(codes),
                                        _ptr_array(scales), _stream(copy_stream), lookahead),
           "sdl_engine_bind_offload")
    engine._keep = (pool, list(w_base), codes, scales, copy_stream)


PROBE_COPY, PROBE_COPY_NT, PROBE_READ_NT, PROBE_FILL_NT = 0, 1, 2, 3


def sdl_memory_probe(kind: int, dst, src, nbytes: int, stream=None):
    _require_device(dst, src)
    _check(_lib.sdl_memory_probe(kind, _ptr(dst), _ptr(src), nbytes, _stream(stream)), "sdl_memory_probe")


def sdl_copy_bytes(dst, src, nbytes: int, stream=None):
    _require_device(dst, src)
    _check(_lib.sdl_copy_bytes(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "sdl_copy_bytes")


EVAL_FIRST_REPLICA, EVAL_REPLICA_MEAN, EVAL_OUTER = 0, 1, 2


def sdl_evaluation_params(which: int, g, w, n: int, out_bf16, stream=None):
    _require_device(g, *(w or []), out_bf16)
    _check(_lib.sdl_evaluation_params(which, _ptr(g), _ptr_array(w), len(w) if w else 0, n, _ptr(out_bf16),
                                      _stream(stream)), "sdl_evaluation_params")


def sdl_cosine_workspace_bytes(M: int, n_sets: int) -> int:
    return _lib.sdl_cosine_workspace_bytes(M, n_sets)


def cosine_result_doubles(M: int) -> int:
    """SDL_COSINE_RESULT_DOUBLES: Gram matrix, cosine matrix, mean over pairs."""
    return 2 * M * M + 1


def alloc_cosine(M: int, n_sets: int = 1, device="cuda"):
    """Device buffers for the cosine calls: (results [n_sets, 2*M*M+1] fp64, workspace uint8)."""
    results = torch.empty((n_sets, cosine_result_doubles(M)), dtype=torch.float64, device=device)
    workspace = torch.empty(max(sdl_cosine_workspace_bytes(M, n_sets), 8), dtype=torch.uint8, device=device)
    return results, workspace


def split_cosine_result(result, M: int):
    """(G [M, M], cos [M, M], mean) views of one result row."""
    mm = M * M
    return result[:mm].view(M, M), result[mm:2 * mm].view(M, M), result[2 * mm]


def sdl_outer_grad_cosine(g, w, n: int, result, workspace, stream=None):
    _require_device(g, *w, result, workspace)
    _check(_lib.sdl_outer_grad_cosine(_ptr(g), _ptr_array(w), len(w), n, _ptr(result), _ptr(workspace),
                                      workspace.numel(), _stream(stream)), "sdl_outer_grad_cosine")


def sdl_outer_grad_cosine_plan(plan: "Plan", p: int, g_base, w_base, span_results, fragment_result, workspace,
                               stream=None):
    _require_device(g_base, *w_base, span_results, fragment_result, workspace)
    _check(_lib.sdl_outer_grad_cosine_plan(plan._h, p, _ptr(g_base), _ptr_array(w_base), len(w_base),
                                           _ptr(span_results), _ptr(fragment_result), _ptr(workspace),
                                           workspace.numel(), _stream(stream)), "sdl_outer_grad_cosine_plan")


def sdl_cosine_combine(results, n_sets: int, M: int, result, stream=None, stride_doubles: Optional[int] = None):
    _require_device(results, result)
    stride = cosine_result_doubles(M) if stride_doubles is None else stride_doubles
    _check(_lib.sdl_cosine_combine(_ptr(results), stride, n_sets, M, _ptr(result), _stream(stream)),
           "sdl_cosine_combine")


def sdl_engine_track_cosine(engine: "Engine", span_results, fragment_results, workspace):
    """span_results: None or a list of P tensors (or None entries); fragment_results: [P, 2*M*M+1] fp64."""
    _require_device(fragment_results, workspace, *[t for t in (span_results or []) if t is not None])
    _check(_lib.sdl_engine_track_cosine(engine._h, _ptr_array(span_results), _ptr(fragment_results), _ptr(workspace),
                                        workspace.numel() if workspace is not None else 0),
           "sdl_engine_track_cosine")
    engine._keep_cosine = (span_results, fragment_results, workspace)


def sdl_flat_layout(total_numel: int, M: int, separate_w_now: bool) -> Tuple[List[int], int]:
    """Byte offsets of g, mom, w_send[0..M) (, w_now[0..M)) inside one allocation, and its size."""
    n = 2 + (2 if separate_w_now else 1) * M
    offs = (ctypes.c_uint64 * n)()
    size = ctypes.c_uint64()
    _check(_lib.sdl_flat_layout(total_numel, M, int(separate_w_now), offs, ctypes.byref(size)), "sdl_flat_layout")
    return list(offs), size.value


def alloc_flat_model(total_numel: int, M: int, separate_w_now: bool, device="cuda"):
    """The flat model arrays carved from one device allocation as sdl_flat_layout says (allocation only, the
    contents are uninitialised).  Returns (g, mom, w_send, w_now, pool); w_now is w_send itself when there is
    no overlap delay.  Keep `pool` alive as long as the views."""
    offs, size = sdl_flat_layout(total_numel, M, separate_w_now)
    align = 1 << 21
    pool = torch.empty(size + align, dtype=torch.uint8, device=device)
    base = (-pool.data_ptr()) % align

    def view(k, dtype, width):
        return pool[base + offs[k]: base + offs[k] + total_numel * width].view(dtype)

    g, mom = view(0, torch.float32, 4), view(1, torch.float32, 4)
    w_send = [view(2 + m, torch.bfloat16, 2) for m in range(M)]
    w_now = [view(2 + M + m, torch.bfloat16, 2) for m in range(M)] if separate_w_now else w_send
    return g, mom, w_send, w_now, pool


def alloc_exchange(fmt: int, n: int, M: int, device="cuda"):
    """Device buffers for M messages of n elements: (codes, scales) lists of uint8 tensors."""
    cb, sb = sdl_exchange_bytes(fmt, n)
    codes = [torch.empty(max(cb, 16), dtype=torch.uint8, device=device) for _ in range(M)]
    scales = [torch.empty(max(sb, 16), dtype=torch.uint8, device=device) for _ in range(M)]
    return codes, scales
