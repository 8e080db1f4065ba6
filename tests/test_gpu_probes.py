"""The memory yardsticks and the layout helper do what their descriptions say (they are not part of the
method, but bench.py's roofline is judged against them)."""
import pytest
import torch

import paper_2501_18512_amd as sdl

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("nbytes", [16, 4096, 256 * 16 * 3 + 16, 1 << 24])
def test_memory_probes(nbytes):
    gen = torch.Generator(DEV).manual_seed(nbytes)
    src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV, generator=gen)
    guard = 4096
    for kind in (sdl.PROBE_COPY, sdl.PROBE_COPY_NT):
        buf = torch.full((nbytes + 2 * guard,), 0x5a, dtype=torch.uint8, device=DEV)
        sdl.sdl_memory_probe(kind, buf[guard:guard + nbytes], src, nbytes)
        torch.cuda.synchronize()
        assert torch.equal(buf[guard:guard + nbytes], src)
        assert bool((buf[:guard] == 0x5a).all()) and bool((buf[guard + nbytes:] == 0x5a).all())
    # the read-only pass writes nothing (random bytes do not spell the one value it would react to)
    buf = torch.full((nbytes + 2 * guard,), 0x5a, dtype=torch.uint8, device=DEV)
    sdl.sdl_memory_probe(sdl.PROBE_READ_NT, buf[guard:guard + nbytes], src, nbytes)
    torch.cuda.synchronize()
    assert bool((buf == 0x5a).all())
    # the write-only pass writes all of dst and nothing else: 16-byte records (index, 0, 0, 0)
    sdl.sdl_memory_probe(sdl.PROBE_FILL_NT, buf[guard:guard + nbytes], None, nbytes)
    torch.cuda.synchronize()
    words = buf[guard:guard + nbytes].view(torch.int32).view(-1, 4)
    assert torch.equal(words[:, 0], torch.arange(nbytes // 16, dtype=torch.int32, device=DEV))
    assert bool((words[:, 1:] == 0).all())
    assert bool((buf[:guard] == 0x5a).all()) and bool((buf[guard + nbytes:] == 0x5a).all())


def test_memory_probe_argument_errors():
    a = torch.zeros(64, dtype=torch.uint8, device=DEV)
    b = torch.zeros(64, dtype=torch.uint8, device=DEV)
    for bad in (lambda: sdl.sdl_memory_probe(7, a, b, 32),                 # unknown kind
                lambda: sdl.sdl_memory_probe(sdl.PROBE_COPY, a, b, 24),    # not a multiple of 16
                lambda: sdl.sdl_memory_probe(sdl.PROBE_COPY, a[8:], b, 16),   # unaligned
                lambda: sdl.sdl_memory_probe(sdl.PROBE_COPY_NT, a, None, 16)):
        with pytest.raises(sdl.SdlError):
            bad()
    sdl.sdl_memory_probe(sdl.PROBE_COPY, a, b, 0)                           # nothing to do


def test_flat_model_arrays_are_disjoint_views_of_one_allocation():
    total, M = 100_000 + 13, 3
    g, mom, w_send, w_now, pool = sdl.alloc_flat_model(total, M, True, device=DEV)
    arrays = [g, mom, *w_send, *w_now]
    assert g.dtype == torch.float32 and w_send[0].dtype == torch.bfloat16 and len(w_now) == M
    lo, hi = pool.data_ptr(), pool.data_ptr() + pool.numel()
    spans = sorted((t.data_ptr(), t.data_ptr() + t.numel() * t.element_size()) for t in arrays)
    assert all(lo <= a and b <= hi for a, b in spans)
    assert all(spans[i][1] <= spans[i + 1][0] for i in range(len(spans) - 1))
    assert all(t.numel() == total for t in arrays)
    assert [t.data_ptr() % (1 << 21) for t in arrays] == [k * 32768 for k in range(len(arrays))]
    g2, mom2, ws2, wn2, _ = sdl.alloc_flat_model(total, M, False, device=DEV)
    assert wn2 is ws2
