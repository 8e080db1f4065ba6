"""GPU parity of sdl_evaluation_params (Appendix, "Which parameters to evaluate") against the
oracle: bit-exact bf16 outputs (both sides do the same single-rounded fp32 operations and the
same round-to-nearest-even to bf16)."""
import numpy as np
import pytest
import torch

import paper_2501_18512_amd as sdl
import workloads
from gpu_util import host_bits, host_f32
from oracle import evalparams as ref

pytestmark = pytest.mark.gpu
DEV = "cuda"
SIZES = [1, 7, 8, 511, 512, 513, 4096 + 33, 3 * 512 * 41 + 5]


def _inputs(n, M, seed=0):
    g, _, w, _ = workloads.make_span(n, M, tau=0, delta="student_t3", unit=n % 83, base_seed=seed, device=DEV)
    return g, w


@pytest.mark.parametrize("which", [sdl.EVAL_FIRST_REPLICA, sdl.EVAL_REPLICA_MEAN, sdl.EVAL_OUTER])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 8, 16])
def test_matches_oracle_bit_for_bit(which, M):
    for n in SIZES:
        print(f"evaluation params which={which} M={M} n={n}", flush=True)
        g, w = _inputs(n, M)
        out = torch.full((n + 8,), -1.0, dtype=torch.bfloat16, device=DEV)
        sdl.sdl_evaluation_params(which, g, w, n, out)
        torch.cuda.synchronize()
        want = ref.evaluation_params(which, host_f32(g), [host_bits(x) for x in w])
        assert np.array_equal(host_bits(out[:n]), want), f"which={which} M={M} n={n}"
        assert torch.all(out[n:] == -1.0), "wrote past the end"


@pytest.mark.parametrize("which", [sdl.EVAL_FIRST_REPLICA, sdl.EVAL_REPLICA_MEAN, sdl.EVAL_OUTER])
def test_unaligned_arrays_and_optional_pointers(which):
    n, M = 5003, 3
    g0, w0 = _inputs(n + 8, M)
    g = g0[1:1 + n]
    w = [x[o:o + n] for x, o in zip(w0, (3, 0, 5))]
    buf = torch.zeros(n + 9, dtype=torch.bfloat16, device=DEV)
    out = buf[1:1 + n]
    sdl.sdl_evaluation_params(which, None if which != sdl.EVAL_OUTER else g,
                              None if which == sdl.EVAL_OUTER else w, n, out)
    torch.cuda.synchronize()
    want = ref.evaluation_params(which, host_f32(g), [host_bits(x) for x in w])
    assert np.array_equal(host_bits(out), want)
    assert buf[0] == 0 and torch.all(buf[1 + n:] == 0)


def test_mean_may_overwrite_the_first_replica():
    n, M = 100_000 + 17, 4
    g, w = _inputs(n, M)
    want = ref.evaluation_params(ref.REPLICA_MEAN, host_f32(g), [host_bits(x) for x in w])
    sdl.sdl_evaluation_params(sdl.EVAL_REPLICA_MEAN, None, w, n, w[0])
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(w[0]), want)


def test_special_values():
    bits = np.array([0x7f800000, 0xff800000, 0x7fc00000, 0x7f7f8000, 0x3f808000, 0x3f818000, 0x80000000, 0x00011704,
                     0x7f800001, 0xff80ffff], np.uint32)       # the last two: NaN with payload only in the low half
    g = torch.from_numpy(bits.view(np.float32)).to(DEV)
    n = bits.size
    out = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    sdl.sdl_evaluation_params(sdl.EVAL_OUTER, g, None, n, out)
    torch.cuda.synchronize()
    got, want = host_bits(out), ref.evaluation_params(ref.OUTER, host_f32(g), [])
    nan = np.isnan(bits.view(np.float32))
    assert nan.sum() == 3
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7f80) == 0x7f80) and np.all((got[nan] & 0x7f) != 0)      # NaN stays NaN


def test_argument_errors():
    g, w = _inputs(64, 2)
    out = torch.zeros(64, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(sdl.SdlError):
        sdl.sdl_evaluation_params(7, g, w, 64, out)
    with pytest.raises(sdl.SdlError):
        sdl.sdl_evaluation_params(sdl.EVAL_REPLICA_MEAN, g, None, 64, out)
    with pytest.raises(sdl.SdlError):
        sdl.sdl_evaluation_params(sdl.EVAL_OUTER, None, w, 64, out)
    with pytest.raises(sdl.SdlError):
        sdl.sdl_evaluation_params(sdl.EVAL_REPLICA_MEAN, g, w, 64, None)
    sdl.sdl_evaluation_params(sdl.EVAL_REPLICA_MEAN, None, w, 0, None)       # nothing to do
