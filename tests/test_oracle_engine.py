"""Pins of the oracle's walk of Algorithm 2 (oracle/engine.py) against what the paper fixes:
the reduction to DiLoCo (Algorithm 1) for one fragment without overlap, the meaning of the overlap
delay tau and of the mixing factor alpha (Section 2.3), per-worker delays (Section 3.3.2), and the
independence of fragments (Section 2.2)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from oracle import FMT_BF16, FMT_E3M0, FMT_FP32, PATTERN_STRIDED, RefEngine, fragment_plan


def _bits(x):
    return workloads.bf16_bits(torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16))


def _f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _model(L=4, per=96):
    return [per] * L, list(range(L)), L


def _state(total, M, seed=0):
    rng = np.random.default_rng(seed)
    g = (rng.standard_normal(total) * 0.02).astype(np.float32)
    w = [_bits(g + rng.standard_normal(total).astype(np.float32) * 1e-3) for _ in range(M)]
    return g, np.zeros(total, np.float32), w


def _inner(w, rng, scale=3e-4):
    for m in range(len(w)):
        w[m][:] = _bits(_f32(w[m]) + rng.standard_normal(w[m].size).astype(np.float32) * scale)


def test_one_fragment_without_overlap_is_diloco():
    """P = 1, tau = 0, alpha = 0, no quantisation: Algorithm 1.  Every H steps the replicas' mean
    outer gradient goes through SGD with Nesterov momentum and every replica restarts from the
    result -- recomputed here with torch.optim.SGD on float tensors."""
    numel, block, L = _model()
    H, M, lr, mu = 5, 3, 0.7, 0.9
    plan = fragment_plan(numel, block, L, 1, PATTERN_STRIDED, H, 0)
    g, mom, w = _state(plan.total, M, seed=1)
    eng = RefEngine(plan, [0] * M, FMT_FP32, lr, mu, 0.0, g, mom, w)
    theta = torch.tensor(g.copy(), requires_grad=True)
    opt = torch.optim.SGD([theta], lr=lr, momentum=mu, nesterov=True)
    mine = [_f32(x).copy() for x in w]
    rng, rng2 = np.random.default_rng(7), np.random.default_rng(7)
    for t in range(1, 3 * H + 1):
        _inner(w, rng)
        for m in range(M):        # the same inner noise on the independent copy
            mine[m] = _f32(_bits(mine[m] + rng2.standard_normal(mine[m].size).astype(np.float32) * 3e-4))
        sent, received = eng.step(t)
        if t % H == 0:
            assert (sent, received) == (1, 1)
            acc = np.zeros(plan.total, np.float32)
            for m in range(M):
                acc = acc + (theta.detach().numpy() - mine[m])
            theta.grad = torch.tensor(acc / np.float32(M))
            opt.step()
            new = _f32(_bits(theta.detach().numpy()))
            mine = [new.copy() for _ in range(M)]
            np.testing.assert_allclose(g, theta.detach().numpy(), rtol=1e-6, atol=1e-7)
            for m in range(M):
                assert np.array_equal(_f32(w[m]), new)
        else:
            assert (sent, received) == (0, 0)


def test_outer_gradient_is_taken_at_the_send_step():
    """Section 2.3: the outer gradient sent at t is computed from the replicas at t; what they do
    during the tau overlapped steps must not change the new outer parameters."""
    numel, block, L = _model()
    H, tau, M = 6, 3, 2
    plan = fragment_plan(numel, block, L, 2, PATTERN_STRIDED, H, tau)
    results = []
    for later_noise in (1e-4, 5e-2):
        g, mom, w = _state(plan.total, M, seed=2)
        eng = RefEngine(plan, [tau] * M, FMT_E3M0, 0.7, 0.9, 0.5, g, mom, w)
        rng = np.random.default_rng(3)
        for t in range(1, H + tau + 1):
            _inner(w, rng, scale=3e-4 if t <= H else later_noise)
            eng.step(t)
        results.append((g.copy(), mom.copy()))
    sl = slice(*[(s[0], s[0] + s[1]) for s in plan.spans[0]][0])
    assert np.array_equal(results[0][0][sl], results[1][0][sl]) and np.array_equal(results[0][1][sl], results[1][1][sl])


@pytest.mark.parametrize("alpha", [0.0, 1.0, 0.5])
def test_alpha_semantics_under_overlap(alpha):
    """alpha = 0 discards the tau overlapped inner steps, alpha = 1 never lets the outer step reach
    the replicas, alpha = 0.5 averages the two (Section 2.3)."""
    numel, block, L = _model(L=2)
    H, tau, M = 4, 2, 2
    plan = fragment_plan(numel, block, L, 1, PATTERN_STRIDED, H, tau)
    g, mom, w = _state(plan.total, M, seed=4)
    shadow = [x.copy() for x in w]                    # replicas that only ever see inner steps
    eng = RefEngine(plan, [tau] * M, FMT_BF16, 0.7, 0.9, alpha, g, mom, w)
    rng, rng2 = np.random.default_rng(5), np.random.default_rng(5)
    for t in range(1, H + tau + 1):
        _inner(w, rng)
        _inner(shadow, rng2)
        before = [_f32(x).copy() for x in w]
        sent, received = eng.step(t)
        if t == H:
            assert (sent, received) == (1, 0)
            assert all(np.array_equal(_f32(a), b) for a, b in zip(w, before))      # sending changes nothing
        if t == H + tau:
            assert received == 1
            for m in range(M):
                if alpha == 1.0:
                    assert np.array_equal(w[m], shadow[m])
                elif alpha == 0.0:
                    assert np.array_equal(w[m], _bits(g))
                else:
                    want = _bits(np.float32(0.5) * before[m] + np.float32(0.5) * g)
                    assert np.array_equal(w[m], want)


def test_slack_between_workers():
    """Section 3.3.2: the workers receive the same outer update at different steps; until its own
    delay has passed a worker's replica is untouched by the synchronisation."""
    numel, block, L = _model(L=2)
    H, M, taus = 5, 3, (1, 3, 2)
    plan = fragment_plan(numel, block, L, 1, PATTERN_STRIDED, H, min(taus))
    g, mom, w = _state(plan.total, M, seed=6)
    eng = RefEngine(plan, taus, FMT_E3M0, 0.7, 0.9, 0.0, g, mom, w)          # alpha = 0: a merge is visible as w == bf16(g)
    g_after = None
    for t in range(1, H + max(taus) + 1):
        before = [x.copy() for x in w]
        sent, received = eng.step(t)                  # no inner noise: only the outer step moves anything
        if t == H + min(taus):
            assert received == 1
            g_after = g.copy()
        if t > H + min(taus):
            assert received == 0 and np.array_equal(g, g_after)             # the mean and Nesterov ran once
        for m in range(M):
            if t == H + taus[m]:
                assert np.array_equal(w[m], _bits(g_after))
            else:
                assert np.array_equal(w[m], before[m])


def test_fragments_are_synchronised_separately():
    """Section 2.2: a fragment's synchronisation touches that fragment only, at its own steps."""
    numel, block, L = _model(L=6)
    H, P, M = 9, 3, 2
    plan = fragment_plan(numel, block, L, P, PATTERN_STRIDED, H, 0)
    g, mom, w = _state(plan.total, M, seed=8)
    eng = RefEngine(plan, [0] * M, FMT_E3M0, 0.7, 0.9, 0.5, g, mom, w)
    mask = np.zeros((P, plan.total), bool)
    for p in range(P):
        for off, n, _ in plan.spans[p]:
            mask[p, off:off + n] = True
    assert np.array_equal(mask.sum(0), np.ones(plan.total))
    for t in range(1, 2 * H + 1):
        before_g = g.copy()
        before_w = [x.copy() for x in w]
        eng.step(t)
        due = plan.sends(t)
        untouched = ~np.any(mask[due], axis=0) if due else np.ones(plan.total, bool)
        assert np.array_equal(g[untouched], before_g[untouched])
        assert all(np.array_equal(a[untouched], b[untouched]) for a, b in zip(w, before_w))
        for p in due:
            assert not np.array_equal(g[mask[p]], before_g[mask[p]])
    assert [p for t in range(1, 2 * H + 1) for p in plan.sends(t)] == [0, 1, 2, 0]       # offsets 0, 3, 6
