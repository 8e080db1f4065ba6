"""Oracle of the parameters handed to evaluation (TEST INFRASTRUCTURE ONLY).

Appendix, paragraph "Which parameters to evaluate": three candidates --
the first replica theta_1, the average of all replicas (1/M) sum_m theta_m, or the globally
shared outer parameters theta.  Written out in the model's storage type (bf16):

    FIRST_REPLICA   out = w[0]
    REPLICA_MEAN    acc = 0; for m = 0..M-1: acc += float(w[m])   (fp32, this order)
                    out = bf16(acc / float(M))                    (round to nearest even)
    OUTER           out = bf16(g)

Reading where the paper is silent: the average is taken in fp32 in replica order, as the
outer step's own mean is (Section 2.4 fixes fp32 for the accumulation there).
"""
from __future__ import annotations

import numpy as np

FIRST_REPLICA, REPLICA_MEAN, OUTER = 0, 1, 2


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest, ties to even; NaN stays NaN (quiet)."""
    assert x.dtype == np.float32
    bits = x.view(np.uint32).astype(np.uint64)
    rounded = (bits + 0x7fff + ((bits >> 16) & 1)) >> 16
    nan = np.isnan(x)
    out = rounded.astype(np.uint16)
    out[nan] = ((bits[nan] >> 16) | 0x40).astype(np.uint16)
    return out


def evaluation_params(which: int, g: np.ndarray, w_bits) -> np.ndarray:
    """bf16 bit patterns of the parameters to evaluate."""
    if which == FIRST_REPLICA:
        return w_bits[0].copy()
    if which == OUTER:
        return bf16_round(g)
    assert which == REPLICA_MEAN
    acc = np.zeros(w_bits[0].shape, np.float32)
    for w in w_bits:
        acc = acc + (w.astype(np.uint32) << 16).view(np.float32)       # one fp32 addition per replica
    return bf16_round(acc / np.float32(len(w_bits)))
