"""Whole-fragment parity at the large configurations: every element of a fragment is compared with
the oracle, streamed through pinned host memory a batch of spans at a time.

The device keeps a copy of the fragment's inputs; after the GPU calls have run, each batch of spans
is copied to the host once, the oracle advances it (all host threads, block-aligned pieces; whole
spans for the whole-span scale, which cannot be cut), and the outputs of every GPU variant that
started from those inputs are compared with the oracle's: g', mom' and every replica in full, and
every code and scale byte where the variant wrote its messages.
"""
from __future__ import annotations

import os
import time
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import oracle
import paper_2501_18512_amd as sdl
from gpu_util import RTOL, ATOL, _bf16_key

THREADS = max(1, min(16, os.cpu_count() or 1))
PIECE = 1 << 20                 # elements per oracle call (a multiple of the largest scale block)
BATCH_ELEMS = 48 << 20          # spans are grouped into batches of about this many elements


@dataclass
class Variant:
    """Outputs of one GPU path that started from the kept inputs: flat model arrays, and, if the path
    wrote messages, per replica the fragment's code / scale arrays in the plan-level layout."""
    name: str
    g: Optional[torch.Tensor]               # g, mom = None: only the messages are compared
    mom: Optional[torch.Tensor]
    w_now: Optional[Sequence[torch.Tensor]]
    codes: Optional[Sequence[torch.Tensor]] = None
    scales: Optional[Sequence[torch.Tensor]] = None
    stats: Dict[str, int] = field(default_factory=dict)


class _Pinned:
    """Pinned host buffers that are reused from batch to batch (pinning memory is slow)."""

    def __init__(self):
        self._buf: Dict[str, torch.Tensor] = {}

    def get(self, key: str, dtype, n: int) -> torch.Tensor:
        t = self._buf.get(key)
        if t is None or t.numel() < n or t.dtype != dtype:
            t = torch.empty(max(n, 1), dtype=dtype, pin_memory=True)
            self._buf[key] = t
        return t[:n]


def _bits16(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).numpy().view(np.uint16)


def _check_f32(got: np.ndarray, want: np.ndarray, what: str) -> int:
    """Tolerance check with a bitwise fast path; returns the number of elements that are not bit-identical."""
    if np.array_equal(got.view(np.uint32), want.view(np.uint32)):
        return 0
    nan_g, nan_w = np.isnan(got), np.isnan(want)
    assert np.array_equal(nan_g, nan_w), f"{what}: NaN positions differ"
    ok = np.isclose(got, want, rtol=RTOL, atol=ATOL, equal_nan=True)
    if not ok.all():
        i = int(np.argmin(ok))
        raise AssertionError(f"{what}: {int((~ok).sum())} of {ok.size} out of tolerance, first at {i}: "
                             f"got {got[i]!r} want {want[i]!r}")
    return int((got.view(np.uint32) != want.view(np.uint32)).sum())


def _check_bf16(got: np.ndarray, want: np.ndarray, what: str) -> int:
    if np.array_equal(got, want):
        return 0
    nan_g, nan_w = (got & 0x7fff) > 0x7f80, (want & 0x7fff) > 0x7f80
    assert np.array_equal(nan_g, nan_w), f"{what}: NaN positions differ"
    d = np.abs(_bf16_key(got) - _bf16_key(want))
    d[nan_g] = 0
    if d.max(initial=0) > 1:
        i = int(np.argmax(d))
        raise AssertionError(f"{what}: {int((d > 1).sum())} elements differ by more than one bf16 ulp, first at {i}: "
                             f"got {got[i]:#06x} want {want[i]:#06x}")
    return int((d != 0).sum())


def _check_bytes(got: np.ndarray, want: np.ndarray, what: str):
    if not np.array_equal(got, want):
        bad = np.nonzero(got != want)[0]
        i = int(bad[0])
        raise AssertionError(f"{what}: {bad.size} of {got.size} bytes differ, first at {i}: "
                             f"got {got[i]:#04x} want {want[i]:#04x}")


def message_positions(plan, p: int, fmt: int) -> Dict[int, int]:
    """Flat offset of every span of fragment p -> element position of the span in the fragment's
    message arrays (the plan-level layout: pieces back to back, each padded to 512 elements; the pieces
    are the joined runs, or the spans themselves for the whole-span scale)."""
    spans = sdl.sdl_plan_fragment_spans(plan, p)
    pieces = spans if fmt == sdl.FMT_E3M0_SPAN else sdl.sdl_plan_fragment_runs(plan, p)
    start, pos = [], 0
    for off, n, _ in pieces:
        start.append((off, n, pos))
        if n:
            pos += (n + 511) // 512 * 512
    out = {}
    for off, n, _ in spans:
        for po, pn, pp in start:
            if po <= off and off + n <= po + pn and pn:
                out[off] = pp + (off - po)
                break
    return out


def stream_check(plan, p: int, fmt: int, lr: float, mu: float, alpha: float, *, g0, mom0, w_send, w_now0,
                 variants: List[Variant], what: str, progress=None, stage: str = "fused") -> Dict[str, int]:
    """Compare every element of fragment p.

    g0, mom0, w_send, w_now0: flat device arrays that hold the fragment's INPUTS (w_now0 may be the same
    list as w_send when there is no overlap delay).  variants: the outputs of the GPU paths.
    stage: "fused" = the whole outer step; "quantize" = messages only; "reduce" = g', mom' only (no merge).
    Returns counts of compared elements / bytes."""
    M = len(w_send)
    aliased = all(a.data_ptr() == b.data_ptr() for a, b in zip(w_send, w_now0))
    spans = [(off, n, i) for i, (off, n, _) in enumerate(sdl.sdl_plan_fragment_spans(plan, p)) if n]
    want_codes = any(v.codes is not None for v in variants)
    pos = message_positions(plan, p, fmt) if want_codes else {}
    span_scaled = fmt == sdl.FMT_E3M0_SPAN
    pin = _Pinned()
    counts = {"elements": 0, "code_bytes": 0, "scale_bytes": 0, "g_not_bit_identical": 0,
              "mom_not_bit_identical": 0, "w_not_bit_identical": 0}
    # batches of whole spans
    batches, cur, cur_n = [], [], 0
    for s in spans:
        if cur and cur_n + s[1] > BATCH_ELEMS:
            batches.append(cur)
            cur, cur_n = [], 0
        cur.append(s)
        cur_n += s[1]
    if cur:
        batches.append(cur)
    t_start = time.time()
    with ThreadPoolExecutor(max_workers=THREADS) as pool:
        for bi, batch in enumerate(batches):
            nb = sum(n for _, n, _ in batch)
            hg = pin.get("g", torch.float32, nb)
            hmom = pin.get("mom", torch.float32, nb)
            hs = [pin.get(f"ws{m}", torch.bfloat16, nb) for m in range(M)]
            hn = hs if aliased else [pin.get(f"wn{m}", torch.bfloat16, nb) for m in range(M)]
            lo = 0
            where = []                       # (flat offset, n, start in the batch, span index)
            for off, n, si in batch:
                hg[lo:lo + n].copy_(g0[off:off + n])
                hmom[lo:lo + n].copy_(mom0[off:off + n])
                for m in range(M):
                    hs[m][lo:lo + n].copy_(w_send[m][off:off + n])
                    if not aliased:
                        hn[m][lo:lo + n].copy_(w_now0[m][off:off + n])
                where.append((off, n, lo, si))
                lo += n
            torch.cuda.synchronize()
            ng, nmom = hg.numpy(), hmom.numpy()
            ns = [_bits16(t) for t in hs]
            nn = ns if aliased else [_bits16(t) for t in hn]
            # the oracle, in place, on pieces that share no scale
            items = []
            for off, n, lo_b, si in where:
                step = n if span_scaled else PIECE
                for a in range(0, n, step):
                    items.append((lo_b + a, min(step, n - a), off, a))
            exp_codes = {}

            def run(item):
                b0, k, off, a = item
                sl = slice(b0, b0 + k)
                ws = [w[sl] for w in ns]
                wn = ws if aliased else [w[sl] for w in nn]
                if stage == "quantize":
                    return item, oracle.quantize_outer_grad(ng[sl], ws, fmt)
                if stage == "reduce":
                    rc, rs = oracle.quantize_outer_grad(ng[sl], ws, fmt)
                    oracle.dequant_reduce_nesterov(ng[sl], nmom[sl], rc, rs, fmt, lr, mu)
                    return item, (rc, rs)
                return item, oracle.fragment_outer_step(ng[sl], nmom[sl], ws, wn, fmt, lr, mu, alpha,
                                                        want_codes=want_codes)

            for item, msg in pool.map(run, items):
                if want_codes:
                    exp_codes[(item[2], item[3])] = msg
            # the GPU variants against it
            for v in variants:
                tag = f"{what} [{v.name}]"
                if stage != "quantize" and v.mom is not None:
                    og = pin.get("out_g", torch.float32, nb)
                    om = pin.get("out_mom", torch.float32, nb)
                    for off, n, lo_b, _ in where:
                        og[lo_b:lo_b + n].copy_(v.g[off:off + n])
                        om[lo_b:lo_b + n].copy_(v.mom[off:off + n])
                    torch.cuda.synchronize()
                    for off, n, lo_b, _ in where:
                        sl = slice(lo_b, lo_b + n)
                        counts["g_not_bit_identical"] += _check_f32(og.numpy()[sl], ng[sl], f"{tag} g span@{off}")
                        counts["mom_not_bit_identical"] += _check_f32(om.numpy()[sl], nmom[sl], f"{tag} mom span@{off}")
                if stage == "fused" and v.w_now is not None:
                    for m in range(M):
                        ow = pin.get("out_w", torch.bfloat16, nb)
                        for off, n, lo_b, _ in where:
                            ow[lo_b:lo_b + n].copy_(v.w_now[m][off:off + n])
                        torch.cuda.synchronize()
                        got = _bits16(ow)
                        for off, n, lo_b, _ in where:
                            sl = slice(lo_b, lo_b + n)
                            counts["w_not_bit_identical"] += _check_bf16(got[sl], nn[m][sl], f"{tag} w_now[{m}] span@{off}")
                if v.codes is not None:
                    for off, n, lo_b, si in where:
                        mp = pos[off]
                        step = n if span_scaled else PIECE
                        for a in range(0, n, step):
                            k = min(step, n - a)
                            rc, rs = exp_codes[(off, a)]
                            c0 = sdl.sdl_exchange_bytes(fmt, mp + a)[0]
                            for m in range(M):
                                got = v.codes[m][c0:c0 + rc[m].size].cpu().numpy()
                                _check_bytes(got, rc[m], f"{tag} codes[{m}] span@{off}+{a}")
                                counts["code_bytes"] += rc[m].size
                                if span_scaled:
                                    got_s = v.scales[m][4 * si:4 * si + 4].cpu().numpy()
                                    _check_bytes(got_s, rs[m], f"{tag} scale word[{m}] span@{off}")
                                    counts["scale_bytes"] += 4
                                elif rs[m].size and v.scales is not None:
                                    s0 = sdl.sdl_exchange_bytes(fmt, mp + a)[1]
                                    got_s = v.scales[m][s0:s0 + rs[m].size].cpu().numpy()
                                    _check_bytes(got_s, rs[m], f"{tag} scales[{m}] span@{off}+{a}")
                                    counts["scale_bytes"] += rs[m].size
            counts["elements"] += nb
            if progress is not None and (bi + 1 == len(batches) or (bi + 1) % max(1, len(batches) // 6) == 0):
                progress(f"{what}: batch {bi + 1}/{len(batches)}, {counts['elements']} elements compared, "
                         f"{time.time() - t_start:.0f} s")
    return counts
