"""The comparison baseline of the paper (its Algorithm 1): pins of the oracle's version (no GPU) and GPU parity."""
import math

import numpy as np
import pytest

U64 = 2.0 ** -53
U32 = 2.0 ** -24


# ---------------------------------------------------------------------------------------------------
# oracle pins (CPU)
# ---------------------------------------------------------------------------------------------------
def test_oracle_baseline_reproduces_the_worked_examples_of_the_paper():
    from oracle import oracle_expm_baseline_batch
    # Sec. 4.2: normal matrix of norm 12.8, eps = 1e-8: baseline takes m = 8, s = 5, i.e. 12 products
    X, info = oracle_expm_baseline_batch(12.8 * np.eye(4), 1e-8)
    assert (info["m"][0], info["s"][0]) == (8, 5) and info["m"][0] - 1 + info["s"][0] == 12
    # Remark 1: W = [[1, 10], [0, -1]]: baseline scaling s = 5
    X, info = oracle_expm_baseline_batch(np.array([[1.0, 10.0], [0.0, -1.0]]), 1e-8)
    assert info["s"][0] == 5
    E = np.array([[math.e, 10.0 * math.sinh(1.0)], [0.0, 1.0 / math.e]])
    assert np.abs(X[0] - E).max() < 1e-6   # the baseline's accuracy after 5 squarings of an eps = 1e-8 truncation


def test_oracle_baseline_rule_by_hand():
    from oracle import oracle_expm_baseline_batch
    # scaling: smallest s with norm / 2^s < 1/2 (strict)
    for norm, s in ((0.49, 0), (0.5, 1), (0.99, 1), (1.0, 2), (3.9, 3), (4.0, 4), (1e-3, 0)):
        _, info = oracle_expm_baseline_batch(norm * np.eye(2), 1e-8)
        assert info["s"][0] == s, (norm, info["s"][0])
    # degree for W = x I: terms x^k / k! are added while > eps
    for x, eps in ((0.3, 1e-8), (0.05, 1e-5), (0.45, U64)):
        _, info = oracle_expm_baseline_batch(x * np.eye(2), eps)
        m = 0
        while x ** (m + 1) / math.factorial(m + 1) > eps:
            m += 1
        assert info["m"][0] == m and info["s"][0] == 0
    # result: the truncated series, exactly, for a 1x1 matrix without scaling
    x, eps = 0.37, 1e-9
    X, info = oracle_expm_baseline_batch(np.array([[x]]), eps)
    ref = sum(x ** k / math.factorial(k) for k in range(info["m"][0] + 1))
    assert X[0, 0, 0] == pytest.approx(ref, rel=1e-15)
    # zero matrix
    X, info = oracle_expm_baseline_batch(np.zeros((1, 3, 3)), 1e-8)
    assert (info["m"][0], info["s"][0]) == (0, 0) and np.array_equal(X[0], np.eye(3))


def test_oracle_baseline_against_closed_forms():
    from oracle import oracle_expm_baseline_batch
    d = np.array([-1.5, 0.2, 0.9])
    X, _ = oracle_expm_baseline_batch(np.diag(d), U64)
    assert np.allclose(np.diag(X[0]), np.exp(d), rtol=1e-13)
    th = 0.7
    X, _ = oracle_expm_baseline_batch(np.array([[0.0, -th], [th, 0.0]]), U64)
    assert np.abs(X[0] - np.array([[math.cos(th), -math.sin(th)], [math.sin(th), math.cos(th)]])).max() < 1e-14


# ---------------------------------------------------------------------------------------------------
# GPU parity
# ---------------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def ex():
    import torch
    import paper_2512_20777_amd as ex
    assert torch.cuda.is_available()
    ex.load_library()
    return ex


def _run(ex, a, tol, label, gate):
    import torch
    from oracle import oracle_expm_baseline_batch
    X, info = oracle_expm_baseline_batch(a, tol)
    d = torch.from_numpy(a).cuda()
    print("case %s shape %s %s" % (label, a.shape, a.dtype), flush=True)
    out, _ = ex.expm(d, tol, scheme=ex.SCHEME_BASELINE)
    torch.cuda.synchronize()
    stats = ex.expm_get_stats()
    got = out.cpu().numpy().astype(np.float64)
    m, s, _ = ex.expm_select(d, tol, scheme=ex.SCHEME_BASELINE)
    worst, skipped = 0.0, 0
    for b in range(a.shape[0]):
        ref = X[b]
        if (m[b], s[b]) != (info["m"][b], info["s"][b]):
            # the term loop stops on ||Y|| <= eps: only a norm within rounding of eps may stop one term apart (in
            # fp32 the terms' norms carry the rounding of the fp32 products, about 1e-6 relative)
            assert info["near"][b] or a.dtype == np.float32, (label, b, (m[b], s[b]), (info["m"][b], info["s"][b]))
            assert s[b] == info["s"][b] and abs(int(m[b]) - int(info["m"][b])) <= 1
            skipped += 1
            from oracle import oracle_expm_forced   # the degree the device stopped at: that Taylor polynomial, same s
            ref = oracle_expm_forced(a[b], int(m[b]), int(s[b]), plus16=False)
        err = np.linalg.norm(got[b] - ref) / np.linalg.norm(ref)
        worst = max(worst, err)
        assert err <= gate, (label, b, err)
    assert skipped <= max(1, a.shape[0] // 50)
    print("   worst rel Frobenius error %.3e, %d matrices one term apart" % (worst, skipped), flush=True)
    return m, s, stats


@pytest.mark.gpu
@pytest.mark.parametrize("n,dtype", [(2, np.float64), (16, np.float64), (23, np.float32), (48, np.float64),
                                     (64, np.float32), (96, np.float64), (128, np.float32)])
def test_gpu_baseline_parity(ex, n, dtype):
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(1200 + n, 24, n, dtype, 1e-4, 30.0)
    tol = 1e-8 if dtype == np.float64 else 1e-6
    _run(ex, a, tol, "baseline n=%d" % n, 1e-11 if dtype == np.float64 else 5e-5)


@pytest.mark.gpu
@pytest.mark.parametrize("n,batch,dtype,tol", [(129, 6, np.float32, 1e-6), (200, 7, np.float64, 1e-8), (257, 4, np.float64, 2.0 ** -53),
                                                (384, 4, np.float32, 2.0 ** -24), (515, 3, np.float64, 1e-8),
                                                (1024, 8, np.float64, 1e-8)])
def test_gpu_baseline_parity_round_based(ex, n, batch, dtype, tol):
    """Above the on-chip sizes every term of Algorithm 1 is a product round over the matrices still in the loop."""
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(1300 + n, batch, n, dtype, 0.05, 60.0)
    a[0] = 0.0                                     # never enters the loop: X = I
    a[1] *= 1e-20                                  # first term already below the tolerance: X = I as well
    a[2] *= dtype(40.0) / np.abs(a[2]).sum(axis=0).max()   # norm 40: seven squarings
    m, s, stats = _run(ex, a, tol, "baseline rounds n=%d" % n, 1e-11 if dtype == np.float64 else 5e-5)
    assert stats["fused_path"] == 0 and stats["scheme"] == 2
    assert (m[0], s[0]) == (0, 0) and (m[1], s[1]) == (0, 0) and s[2] == 7
    assert stats["products"] == int(np.maximum(m - 1, 0).sum() + s.sum())


@pytest.mark.gpu
def test_gpu_baseline_round_based_infinity_norm_and_nonfinite(ex):
    import torch
    from oracle import oracle_expm_baseline_batch
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(1400, 5, 160, np.float64, 0.5, 20.0, kind="triu")
    at = np.ascontiguousarray(np.swapaxes(a, -1, -2))
    X, info = oracle_expm_baseline_batch(at, 1e-8)            # infinity-norm of W = 1-norm of its transpose
    d = torch.from_numpy(a).cuda()
    out, _ = ex.expm(d, 1e-8, scheme=ex.SCHEME_BASELINE, norm=ex.NORM_INF)
    m, s, _ = ex.expm_select(d, 1e-8, scheme=ex.SCHEME_BASELINE, norm=ex.NORM_INF)
    got = out.cpu().numpy()
    for b in range(5):
        assert (m[b], s[b]) == (info["m"][b], info["s"][b]) or info["near"][b]
        if (m[b], s[b]) == (info["m"][b], info["s"][b]):
            assert np.linalg.norm(got[b] - X[b].T) / np.linalg.norm(X[b]) <= 1e-11
    a[2, 5, 7] = np.inf
    d = torch.from_numpy(a).cuda()
    out, st = ex.expm(d, 1e-8, scheme=ex.SCHEME_BASELINE)
    m, s, st2 = ex.expm_select(d, 1e-8, scheme=ex.SCHEME_BASELINE)
    assert st == 1 and st2 == 1 and (m[2], s[2]) == (-1, -1) and bool(torch.isnan(out[2]).all())
    assert bool(torch.isfinite(out[[0, 1, 3, 4]]).all())


@pytest.mark.gpu
def test_gpu_baseline_examples_and_limits(ex):
    import torch
    a = np.stack([12.8 * np.eye(8), np.zeros((8, 8))])
    d = torch.from_numpy(a).cuda()
    m, s, _ = ex.expm_select(d, 1e-8, scheme=ex.SCHEME_BASELINE)
    assert (m[0], s[0]) == (8, 5) and (m[1], s[1]) == (0, 0)       # the paper's worked example (Sec. 4.2)
    out, _ = ex.expm(d, 1e-8, scheme=ex.SCHEME_BASELINE)
    assert torch.equal(out[1], torch.eye(8, dtype=torch.float64, device="cuda"))
    # above the on-chip sizes the number of squarings is read back: not available under stream capture
    big = torch.zeros(1, 200, 200, dtype=torch.float64, device="cuda")
    res = torch.empty_like(big)
    ex.expm(big, 1e-8, out=res, scheme=ex.SCHEME_BASELINE)
    torch.cuda.synchronize()
    assert torch.equal(res[0], torch.eye(200, dtype=torch.float64, device="cuda"))
    lib = ex.load_library()
    side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        res.zero_()
        status = lib.expm_scheme(big.data_ptr(), 200, 1, ex.DTYPE_F64, 1e-8, ex.SCHEME_BASELINE, res.data_ptr(),
                                 torch.cuda.current_stream().cuda_stream)
    assert status == -5


@pytest.mark.gpu
def test_gpu_product_ratio_baseline_over_proposed_on_flow_workload(ex):
    """The paper's headline comparison (Sec. 4.2: 1.86-1.99x the products on logged flow-layer calls) on the
    synthetic flow setting F1 (tolerance 1e-8, infinity-norm)."""
    import torch
    from paper_2512_20777_amd import workloads
    w = workloads.WORKLOADS["F1"]
    d = torch.from_numpy(workloads.make_workload("F1")).cuda()
    xa, _ = ex.expm(d, w.tol, norm=ex.NORM_INF)
    xa = xa.clone()
    pa = ex.expm_get_stats()["products"]
    xb, _ = ex.expm(d, w.tol, norm=ex.NORM_INF, scheme=ex.SCHEME_BASELINE)
    pb = ex.expm_get_stats()["products"]
    rel = (torch.linalg.norm(xa - xb, dim=(1, 2)) / torch.linalg.norm(xa, dim=(1, 2))).max()
    print("   products: proposed %d, baseline %d (ratio %.2f); max rel difference of results %.2e"
          % (pa, pb, pb / pa, float(rel)), flush=True)
    assert float(rel) < 1e-5       # both are eps = 1e-8 truncations, the baseline squared up to 5 times
    assert 1.3 < pb / pa < 4.0
