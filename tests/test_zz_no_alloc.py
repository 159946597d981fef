"""GPU test of gs_grad_sqnorm_noalloc, the norm for callers that cannot allocate: its partials
live in the library's fixed device array instead of a caller workspace.  It must give what
gs_grad_sqnorm gives (bit for bit with the minimum workspace: same kernels and shapes), and what
the oracle gives, on two calls in a row -- the second with a smaller input, so stale partials of
the first call sit in the array beyond what the second one writes."""
import pytest
import torch

from gpu_util import DEV, DeviceCase, O, gs

pytestmark = pytest.mark.gpu


def _both(case, begin, end, accumulate=False, start=0.0):
    sq_a = torch.full((1,), start, dtype=torch.float64, device=DEV)
    sq_b = torch.full((1,), start, dtype=torch.float64, device=DEV)
    gs.gs_grad_sqnorm(case.grads, begin, end, sq_a, case.ws, accumulate=accumulate)
    before = torch.cuda.memory_allocated()
    gs.gs_grad_sqnorm_noalloc(case.grads, begin, end, sq_b, accumulate=accumulate)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return float(sq_a.item()), float(sq_b.item())


def test_noalloc_norm_equals_workspace_norm_on_two_calls_in_a_row():
    big = DeviceCase(9 * 8192 * 40 + 1237, 16, seed=11, sigma=5e-4)      # ~2.9 M elements: 360 norm workgroups
    small = DeviceCase(8192 * 3 + 77, 4, seed=12)                        # 4 workgroups: most old partials stay behind
    for case in (big, small):
        want = O.grad_sqnorm(case.h_g)
        a, b = _both(case, 0, case.n)
        assert b == a, (a, b)
        assert abs(b - want) <= 1e-5 * want and abs(b - want) <= 1e-10 * want, (b, want)   # 1e-5 is the bar
    # ranges, accumulation and the empty range behave like the existing entry point
    for begin, end in ((13, 100_003), (0, 1), (7, 7), (2048 * 7 + 1, big.n - 3)):
        a, b = _both(big, begin, end)
        assert b == a and abs(b - O.grad_sqnorm(big.h_g, begin, end)) <= 1e-10 * max(a, 1e-300)
    a, b = _both(small, 5, small.n, accumulate=True, start=3.5)
    assert b == a and b > 3.5
    a, b = _both(small, 9, 9, accumulate=True, start=3.5)
    assert a == 3.5 and b == 3.5


def test_noalloc_norm_on_a_side_stream_and_too_large_is_refused():
    case = DeviceCase(1_000_003, 8, seed=13)
    want = O.grad_sqnorm(case.h_g)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    sq = torch.zeros(1, dtype=torch.float64, device=DEV)
    with torch.cuda.stream(s):
        gs.gs_grad_sqnorm_noalloc(case.grads, 0, case.n, sq, stream=s)
    s.synchronize()
    assert abs(float(sq.item()) - want) <= 1e-10 * want
    # a range beyond the stated maximum is refused before anything is enqueued (raw addresses:
    # the check needs no tensors of that size)
    sq.fill_(-1.0)
    st = gs.gs_grad_sqnorm_noalloc([case.grads[0].data_ptr()], 0, gs.GS_NOALLOC_MAX_ELEMS + 1, sq, check=False)
    assert st == gs.GS_ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert float(sq.item()) == -1.0


def test_noalloc_norm_and_step_replay_from_a_hip_graph():
    """What the entry point is for: under stream capture nothing may allocate.  After one call outside
    capture (which looks up the array's address), the no-allocation norm and the step are captured
    once and replayed three times with eager work between the replays; every replay has to equal
    the eager run with the workspace entry point, bit for bit."""
    from test_gpu_parity import HP, compare_states
    n = 2048 * 150 + 9
    case = DeviceCase(n, 8, seed=172)
    p, m, v, w = case.clone_states()
    sq_g = torch.zeros(1, dtype=torch.float64, device=DEV)
    gs.gs_grad_sqnorm_noalloc(case.grads, 0, n, sq_g)                # first call on the device: outside capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        gs.gs_grad_sqnorm_noalloc(case.grads, 0, n, sq_g)
        gs.gs_accum_adamw(p, m, v, w, case.grads, 0, n, HP, sq_g)
    torch.cuda.synchronize()
    eager = case.clone_states()
    first = None
    for it in range(3):
        g.replay()
        torch.cuda.synchronize()
        gs.gs_grad_sqnorm(case.grads, 0, n, case.sq, case.ws)        # eager work between replays, workspace variant
        gs.gs_accum_adamw(*eager, case.grads, 0, n, HP, case.sq)
        torch.cuda.synchronize()
        assert float(sq_g.item()) == float(case.sq.item())
        for a, b in zip((p, m, v, w), eager):
            assert torch.equal(a, b), f"replay {it}"
        if it == 0:
            first = [t.clone() for t in (p, m, v, w)]
    c = O.clip_coef(O.grad_sqnorm(case.h_g), HP.max_grad_norm)
    compare_states(first, case.oracle_step(HP, c), "no-alloc graph, first replay")
