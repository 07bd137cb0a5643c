"""GPU parity of single kernels against the oracle / plain definitions (run with -m gpu)."""
import numpy as np
import pytest
import torch

import synth
from oracle import sampling
from tests.util import gpu_available

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]


def _amd():
    import paper_2408_11850_amd as amd
    amd.load_library()
    return amd


@pytest.mark.parametrize("M,N,K", [(1, 256, 256), (4, 1024, 688), (5, 2064, 256), (16, 512, 2048), (17, 768, 1032),
                                   (32, 512, 4096), (9, 10240, 8192), (1, 4096, 11008), (3, 16, 8)])
def test_projection_matches_definition(M, N, K):
    """y = x W^T on bf16 inputs with fp32 accumulation; sizes span several panels, K slices, ragged K."""
    amd = _amd()
    print(f"gemm M={M} N={N} K={K}", flush=True)
    w = synth.normal_tensor((N, K), 0.05, 3, N * 7 + K, torch.bfloat16)
    x = synth.normal_tensor((M, K), 1.0, 4, M, torch.bfloat16)
    ref = x.to(torch.float64) @ w.to(torch.float64).T
    wp = amd.binding.pack_matrices([w.cuda()])
    y = amd.gemm(x.cuda(), wp, N).cpu().to(torch.float64)
    # fp32 accumulation of K products of magnitude ~|x||w|: error << 1e-3 of the output scale
    scale = ref.abs().max().item()
    assert (y - ref).abs().max().item() <= 2e-5 * scale * max(1.0, (K / 256) ** 0.5)


def test_packed_concatenation_and_interleave():
    amd = _amd()
    K = 96
    a = synth.normal_tensor((32, K), 1.0, 1, 1, torch.bfloat16).cuda()
    b = synth.normal_tensor((48, K), 1.0, 1, 2, torch.bfloat16).cuda()
    x = synth.normal_tensor((3, K), 1.0, 1, 3, torch.bfloat16).cuda()
    y = amd.gemm(x, amd.binding.pack_matrices([a, b]), 80)
    ref = x.float() @ torch.cat([a, b]).float().T
    assert torch.allclose(y, ref, atol=1e-3)
    c = synth.normal_tensor((32, K), 1.0, 1, 4, torch.bfloat16).cuda()
    yi = amd.gemm(x, amd.binding.pack_matrices([a, c], interleave=True), 64)
    ra, rc = x.float() @ a.float().T, x.float() @ c.float().T
    # panels alternate: a rows 0-15, c rows 0-15, a rows 16-31, c rows 16-31
    ref = torch.cat([ra[:, :16], rc[:, :16], ra[:, 16:], rc[:, 16:]], dim=1)
    assert torch.allclose(yi, ref, atol=1e-3)


def test_gemm_rejects_bad_shapes():
    amd = _amd()
    x = torch.zeros((33, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(amd.SpecError):
        amd.gemm(x, w, 64)
    with pytest.raises(amd.SpecError):
        amd.gemm(x[:2], w, 40)


def _logit_rows(n, v, seed, scale=3.0):
    return synth.normal_tensor((n, v), scale, seed, 77, torch.float32)


# 32768 is the largest vocabulary of the register-resident kernel, 32769 and 50304 take the generic one; 4160 = 65
# rows of 64 leaves ragged rows in every wave
@pytest.mark.parametrize("V,temp,ls", [(1024, 1.0, 8.0), (32000, 1.0, 1.0), (32256, 0.7, 1.0), (50, 1.0, 1.0),
                                       (32768, 1.0, 1.0), (32769, 1.0, 1.0), (50304, 1.3, 1.0), (4160, 0.5, 2.0)])
def test_draft_sampling_matches_oracle(V, temp, ls):
    amd = _amd()
    rows = _logit_rows(6, V, 5)
    us = synth.uniform_array(6, 9, 1).tolist()
    n_checked = 0
    for i in range(6):
        q_gpu, tok = amd.sample_row(rows[i].cuda(), temp, ls, us[i])
        q = sampling.probs(rows[i].numpy(), temp, ls)
        np.testing.assert_allclose(q_gpu.cpu().numpy(), q, rtol=2e-5, atol=1e-12)
        # decision margin: distance of u to the nearest CDF edge
        cdf = np.cumsum(q.astype(np.float64))
        margin = np.min(np.abs(cdf / cdf[-1] - us[i]))
        if margin > 1e-5:
            assert tok == sampling.sample(q, us[i])
            n_checked += 1
    assert n_checked >= 4


@pytest.mark.parametrize("V", [32000, 777, 40000])
def test_draft_sampling_walk_on_sparse_rows_and_extreme_uniforms(V):
    """Very peaked rows (most probabilities underflow to exactly 0) and uniforms at both ends of [0, 1): the draw
    must be the first id whose fp64 running sum of the kernel's own q row exceeds u times the total, never an id of
    zero probability."""
    amd = _amd()
    rows = _logit_rows(4, V, 9, scale=60.0)
    rows[3, :] = -1000.0
    rows[3, V - 3] = 5.0                                   # a single id carries all the mass
    n_checked = 0
    for i in range(4):
        for u in (0.0, 1e-7, 0.37, 0.5, 0.93, 1.0 - 2.0 ** -24):
            q_gpu, tok = amd.sample_row(rows[i].cuda(), 1.0, 1.0, u)
            q = q_gpu.cpu().numpy().astype(np.float64)
            assert q[tok] > 0.0
            cdf = np.cumsum(q)
            want = int(np.searchsorted(cdf, np.float64(np.float32(u)) * cdf[-1], side="right"))
            margin = np.min(np.abs(cdf / cdf[-1] - u)[q > 0])
            if margin > 1e-9:
                assert tok == want, (i, u, tok, want)
                n_checked += 1
    assert n_checked >= 16


def test_greedy_sampling_is_argmax_with_lowest_id_ties():
    amd = _amd()
    row = _logit_rows(1, 4096, 6)[0]
    row[100] = row[3000] = row.max() + 1.0
    q, tok = amd.sample_row(row.cuda(), 0.0, 1.0, 0.9)
    assert tok == 100 and q[100].item() == 1.0 and q.sum().item() == 1.0


# 40000: beyond the register-resident kernels' 32768 ids, the generic path
@pytest.mark.parametrize("V,ls", [(1024, 8.0), (32000, 1.0), (40000, 1.0)])
def test_accept_kernel_matches_oracle(V, ls):
    """Rows of target logits against rows of draft distributions: first rejection and the corrected token."""
    amd = _amd()
    n_test = 5
    pl = _logit_rows(n_test + 1, V, 11, scale=1.5)
    ql = pl + _logit_rows(n_test + 1, V, 12, scale=0.5)        # a draft correlated with the target
    P = sampling.probs(pl.numpy(), 1.0, ls)
    Q = sampling.probs(ql.numpy()[:n_test], 1.0, ls)
    checked = {"reject": 0, "all": 0}
    for trial in range(12):
        us = synth.uniform_array(2 * n_test + 1, 100 + trial, 1).numpy().astype(np.float64)
        x = [sampling.sample(Q[i], us[i]) for i in range(n_test)]
        r = us[n_test:2 * n_test]
        u2 = float(us[-1])
        # oracle decision and its margins
        n, margin = 0, 1.0
        for i in range(n_test):
            lhs, rhs = r[i] * Q[i][x[i]], float(P[i][x[i]])
            margin = min(margin, abs(lhs - rhs) / max(lhs, rhs))
            if sampling.accept(P[i], Q[i], x[i], r[i]):
                n += 1
            else:
                break
        if n < n_test:
            w = sampling.residual(P[n], Q[n])
            y = sampling.resample(P[n], Q[n], u2)
        else:
            w = P[n_test].astype(np.float64)
            y = sampling.sample(P[n_test], u2)
        cdf = np.cumsum(w)
        draw_margin = np.min(np.abs(cdf / cdf[-1] - u2))      # same inputs, fp32 arithmetic: only rounding order differs
        got = amd.accept_rows(pl.cuda(), torch.from_numpy(Q).cuda(), x, r, 1.0, ls, u2)
        if margin > 1e-4 and draw_margin > 2e-6:
            assert got == (n, y), (trial, got, n, y, margin)
            checked["reject" if n < n_test else "all"] += 1
    assert checked["reject"] >= 1 and checked["reject"] + checked["all"] >= 6, checked


@pytest.mark.parametrize("V", [2048, 32768, 33008])
def test_accept_kernel_special_cases(V):
    amd = _amd()
    pl = _logit_rows(3, V, 21)
    P = sampling.probs(pl.numpy(), 1.0, 1.0)
    # p == q: always accepted, bonus drawn from the row after the last test
    x = [int(np.argmax(P[0])), int(np.argmax(P[1]))]
    n, y = amd.accept_rows(pl.cuda(), torch.from_numpy(P[:2].copy()).cuda(), x, [0.999, 0.999], 1.0, 1.0, 0.37)
    assert n == 2 and y == sampling.sample(P[2], 0.37)
    # q puts all mass on a token the target gives ~0: rejected at once, corrected token ~ p (q has no overlap)
    q = np.zeros((1, V), dtype=np.float32)
    worst = int(np.argmin(P[0]))
    q[0, worst] = 1.0
    n, y = amd.accept_rows(pl[:1].cuda(), torch.from_numpy(q).cuda(), [worst], [0.5], 1.0, 1.0, 0.61)
    assert n == 0 and y == sampling.resample(P[0], q[0], 0.61)
    # greedy: accept iff the draft token is the target's arg-max, else emit the arg-max
    n, y = amd.accept_rows(pl.cuda(), torch.from_numpy(P[:2].copy()).cuda(), [x[0], x[1] + 1], [0.5, 0.5], 0.0, 1.0, 0.5)
    assert (n, y) == (1, x[1])
    # autoregressive draw (no tests)
    n, y = amd.accept_rows(pl[:1].cuda(), None, [], [], 1.0, 1.0, 0.25)
    assert n == 0 and y == sampling.sample(P[0], 0.25)
