"""The allocation-free acceptance call against the allocating one it is a variant of (run with -m gpu).

spec_accept_rows_static keeps the kernels' scratch in a device array of the library; every call on a GPU shares
that array and finds the previous call's contents in it.  Two calls in a row, the second on a smaller input (fewer
rows, a shorter vocabulary, the other vocabulary path), must each give exactly what spec_accept_rows gives on the
same inputs: same kernels, same arithmetic, so the outcomes are compared for equality.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import sampling
from tests.util import gpu_available

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]


def _case(V, n_test, seed, ls):
    pl = synth.normal_tensor((n_test + 1, V), 1.5, seed, 77, torch.float32)
    ql = pl + synth.normal_tensor((n_test + 1, V), 0.5, seed + 1, 77, torch.float32)
    Q = sampling.probs(ql.numpy()[:n_test], 1.0, ls)
    return pl, Q


def _both(amd, pl, Q, x, r, temp, ls, u2):
    pl_d = pl.cuda()
    q_d = torch.from_numpy(np.ascontiguousarray(Q)).cuda() if len(x) else None
    x_d = torch.tensor(list(x), dtype=torch.int32, device="cuda") if len(x) else None
    out = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    amd.accept_rows_static(pl_d, q_d, x_d, r, temp, ls, u2, out)
    torch.cuda.synchronize()
    got = tuple(out.tolist())
    want = amd.accept_rows(pl_d, q_d, list(x), r, temp, ls, u2)
    return got, tuple(want)


def test_static_scratch_call_equals_the_allocating_call_twice_in_a_row():
    import paper_2408_11850_amd as amd
    amd.load_library()
    # first a long row through the generic path (it fills the scratch row of draw weights), then smaller inputs
    # through both paths; each sequence mixes rejections, full accepts with a bonus draw, and a draw without tests
    plan = [(40000, 6, 1.0, 1.0), (32000, 5, 1.0, 1.0), (1024, 3, 1.0, 8.0), (33008, 2, 0.7, 1.0), (50, 1, 1.0, 1.0)]
    outcomes = set()
    for k, (V, n_test, temp, ls) in enumerate(plan):
        pl, Q = _case(V, n_test, 300 + k, ls)
        for trial in range(4):
            us = synth.uniform_array(2 * n_test + 1, 500 + 10 * k + trial, 1).numpy().astype(np.float64)
            x = [sampling.sample(Q[i], us[i]) for i in range(n_test)]
            r = us[n_test:2 * n_test]
            got, want = _both(amd, pl, Q, x, r, temp, ls, float(us[-1]))
            print(f"V={V} n_test={n_test} trial={trial}: static {got} allocating {want}", flush=True)
            assert got == want
            outcomes.add("all" if want[0] == n_test else "reject")
        # accept everything (p == q rows): the bonus row's draw; and the draw without any test
        P = sampling.probs(pl.numpy(), 1.0, ls)
        x = [int(np.argmax(P[i])) for i in range(n_test)]
        got, want = _both(amd, pl, P[:n_test], x, [0.5] * n_test, 1.0, ls, 0.37)
        assert got == want and want[0] == n_test
        got, want = _both(amd, pl[:1].contiguous(), None, [], [], 1.0, ls, 0.25)
        assert got == want and want[0] == 0
        # greedy
        got, want = _both(amd, pl, P[:n_test], x, [0.5] * n_test, 0.0, ls, 0.5)
        assert got == want
    assert outcomes == {"all", "reject"} or "reject" in outcomes


def test_static_scratch_call_rejects_what_it_cannot_hold():
    import paper_2408_11850_amd as amd
    lib = amd.load_library()
    out = torch.zeros(2, dtype=torch.int32, device="cuda")
    big = 262144 + 16
    pl = torch.zeros((1, big), dtype=torch.float32, device="cuda")
    with pytest.raises(amd.SpecError) as ei:
        amd.accept_rows_static(pl, None, None, [], 1.0, 1.0, 0.5, out)
    assert ei.value.code == amd.SPEC_E_INVAL and "static scratch" in str(ei.value)
    # the largest vocabulary it takes runs, and equals the allocating call
    pl = synth.normal_tensor((1, 262144), 2.0, 3, 77, torch.float32).cuda()
    amd.accept_rows_static(pl, None, None, [], 1.0, 1.0, 0.81, out)
    torch.cuda.synchronize()
    assert tuple(out.tolist()) == tuple(amd.accept_rows(pl, None, [], [], 1.0, 1.0, 0.81))
