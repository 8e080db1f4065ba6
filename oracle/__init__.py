"""CPU oracle of the Streaming DiLoCo fragment outer step (TEST INFRASTRUCTURE ONLY).

Thin numpy/ctypes front end of ``sdl_ref.c`` (arithmetic of the outer step) and ``plan.py``
(fragment map and schedule); ``engine.py`` walks Algorithm 2 over many steps with them;
``cosine.py`` and ``evalparams.py`` are the appendix's diagnostics, in numpy.  Nothing in the GPU package may import this
package; only the tests, the smoke check and the CPU-baseline leg of the
benchmark do.  The C file is compiled with gcc, ``-O2 -ffp-contract=off`` so
that every fp32 operation rounds once, as written.

Arrays are numpy: fp32 as ``float32``, bf16 replicas as ``uint16`` bit
patterns, codes and scale bytes as ``uint8``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import cosine, evalparams  # noqa: F401
from .plan import (PATTERN_SEQUENTIAL, PATTERN_STRIDED, UNIT_POST, UNIT_PRE,  # noqa: F401
                   RefPlan, fragment_plan)

FMT_FP32, FMT_BF16, FMT_E4M3, FMT_E3M0 = 0, 1, 2, 3
FMT_E3M0_B64, FMT_E3M0_B128, FMT_E3M0_SPAN = 4, 5, 6
FMT_E3M0_RN = 7            # 32-element blocks, block maximum rounded to nearest (scale one binade higher)
BLOCK = 32
MAX_BLOCK = 128

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sdl_ref.c")
_SO = os.path.join(_HERE, "libsdl_ref.so")
# The mutation test of the pins points this at a deliberately broken build of sdl_ref.c.
_OVERRIDE = os.environ.get("SDL_ORACLE_LIB")
_lib = None


def compile_source(src: str, out: str) -> None:
    cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", out, src, "-lm"]
    subprocess.run(cmd, check=True)


def build(force: bool = False) -> str:
    """Compile sdl_ref.c into libsdl_ref.so next to it (gcc, plain C)."""
    if _OVERRIDE:
        return _OVERRIDE
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        compile_source(_SRC, _SO)
    return _SO


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        pp = ctypes.POINTER(ctypes.c_void_p)
        lib.sdl_ref_exchange_bytes.restype = ctypes.c_size_t
        lib.sdl_ref_exchange_bytes.argtypes = [ctypes.c_int, ctypes.c_uint64,
                                               ctypes.POINTER(ctypes.c_size_t),
                                               ctypes.POINTER(ctypes.c_size_t)]
        lib.sdl_ref_quantize_outer_grad.argtypes = [ctypes.c_void_p, pp, ctypes.c_uint32,
                                                    ctypes.c_uint64, ctypes.c_int, pp, pp]
        lib.sdl_ref_dequant_reduce_nesterov.argtypes = [ctypes.c_void_p, ctypes.c_void_p, pp, pp,
                                                        ctypes.c_uint32, ctypes.c_uint64,
                                                        ctypes.c_int, ctypes.c_float,
                                                        ctypes.c_float]
        lib.sdl_ref_merge_overlap.argtypes = [ctypes.c_void_p, pp, ctypes.c_uint32,
                                              ctypes.c_uint64, ctypes.c_float]
        lib.sdl_ref_fragment_outer_step.argtypes = [ctypes.c_void_p, ctypes.c_void_p, pp, pp,
                                                    ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int,
                                                    ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                                    pp, pp]
        lib.sdl_ref_encode_block.argtypes = [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_int,
                                             ctypes.c_void_p]
        lib.sdl_ref_decode_code.restype = ctypes.c_float
        lib.sdl_ref_decode_code.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_int]
        _lib = lib
    return _lib


def _check(a: np.ndarray, dtype, n=None):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, (a.dtype, dtype)
    if n is not None:
        assert a.size >= n, (a.size, n)
    return a


def _ptrs(arrs):
    return (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def exchange_bytes(fmt: int, n: int):
    """(code_bytes, scale_bytes) of one replica's message for n elements."""
    c, s = ctypes.c_size_t(), ctypes.c_size_t()
    _load().sdl_ref_exchange_bytes(fmt, n, ctypes.byref(c), ctypes.byref(s))
    return c.value, s.value


def alloc_exchange(fmt: int, n: int, M: int):
    cb, sb = exchange_bytes(fmt, n)
    return ([np.zeros(max(cb, 1), np.uint8) for _ in range(M)],
            [np.zeros(max(sb, 1), np.uint8) for _ in range(M)])


def quantize_outer_grad(g, w_send, fmt, codes=None, scales=None):
    """Encode g - w_send[m] for every replica; returns (codes, scales) lists of uint8 arrays."""
    n, M = g.size, len(w_send)
    _check(g, np.float32)
    for w in w_send:
        _check(w, np.uint16, n)
    if codes is None:
        codes, scales = alloc_exchange(fmt, n, M)
    rc = _load().sdl_ref_quantize_outer_grad(g.ctypes.data, _ptrs(w_send), M, n, fmt,
                                             _ptrs(codes), _ptrs(scales))
    assert rc == 0, rc
    cb, sb = exchange_bytes(fmt, n)
    return [c[:cb] for c in codes], [s[:sb] for s in scales]


def dequant_reduce_nesterov(g, mom, codes, scales, fmt, lr, mu, n=None):
    """In-place update of g and mom from the M messages."""
    n = g.size if n is None else n
    _check(g, np.float32, n), _check(mom, np.float32, n)
    rc = _load().sdl_ref_dequant_reduce_nesterov(g.ctypes.data, mom.ctypes.data, _ptrs(codes),
                                                 _ptrs(scales), len(codes), n, fmt, lr, mu)
    assert rc == 0, rc


def merge_overlap(g_new, w_now, alpha):
    """In-place alpha-merge of g_new into every replica of w_now."""
    n = g_new.size
    _check(g_new, np.float32)
    for w in w_now:
        _check(w, np.uint16, n)
    rc = _load().sdl_ref_merge_overlap(g_new.ctypes.data, _ptrs(w_now), len(w_now), n, alpha)
    assert rc == 0, rc


def fragment_outer_step(g, mom, w_send, w_now, fmt, lr, mu, alpha, want_codes=False):
    """Whole outer step of one span, in place; optionally returns (codes, scales)."""
    n, M = g.size, len(w_send)
    _check(g, np.float32), _check(mom, np.float32, n)
    for w in list(w_send) + list(w_now):
        _check(w, np.uint16, n)
    codes = scales = None
    cp = sp = None
    if want_codes:
        codes, scales = alloc_exchange(fmt, n, M)
        cp, sp = _ptrs(codes), _ptrs(scales)
    rc = _load().sdl_ref_fragment_outer_step(g.ctypes.data, mom.ctypes.data, _ptrs(w_send),
                                             _ptrs(w_now), M, n, fmt, lr, mu, alpha, cp, sp)
    assert rc == 0, rc
    if want_codes:
        cb, sb = exchange_bytes(fmt, n)
        return [c[:cb] for c in codes], [s[:sb] for s in scales]
    return None


def fragment_outer_step_chunked(g, mom, w_send, w_now, fmt, lr, mu, alpha, threads: int):
    """The same step, with the span cut into block-aligned ranges that are handed to
    `threads` host threads.  Every element's arithmetic is unchanged (the step is
    independent per 32-element block); only the benchmark's CPU baseline uses this."""
    n = g.size
    # cutting is only valid where no scale is shared across the cut: never for the whole-span
    # scale, and at multiples of the largest scale block (128) otherwise
    if threads <= 1 or n < MAX_BLOCK * threads or fmt == FMT_E3M0_SPAN:
        fragment_outer_step(g, mom, w_send, w_now, fmt, lr, mu, alpha)
        return 1
    per = -(-n // threads)
    per = -(-per // MAX_BLOCK) * MAX_BLOCK
    ranges = [(lo, min(lo + per, n)) for lo in range(0, n, per)]
    aliased = all(a is b for a, b in zip(w_send, w_now))

    def run(r):
        lo, hi = r
        ws = [w[lo:hi] for w in w_send]
        wn = ws if aliased else [w[lo:hi] for w in w_now]
        fragment_outer_step(g[lo:hi], mom[lo:hi], ws, wn, fmt, lr, mu, alpha)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(run, ranges))
    return len(ranges)


def encode_block(delta: np.ndarray, fmt: int):
    """Encode <= 32 fp32 values as one block: (unpacked codes uint8[len], scale byte)."""
    _check(delta, np.float32)
    out = np.zeros(delta.size, np.uint8)
    sb = _load().sdl_ref_encode_block(delta.ctypes.data, delta.size, fmt, out.ctypes.data)
    assert sb >= 0, sb
    return out, sb


def decode_code(code: int, sb: int, fmt: int) -> float:
    return float(_load().sdl_ref_decode_code(code, sb, fmt))


def unpack_e3m0(codes: np.ndarray, n: int) -> np.ndarray:
    """Packed nibbles -> one code per element (pure re-indexing, for test read-outs)."""
    lo, hi = codes & 15, codes >> 4
    return np.stack([lo, hi], axis=1).reshape(-1)[:n]


from .engine import RefEngine  # noqa: E402,F401
