"""GPU parity of the Paterson-Stockmeyer scheme (Algorithm 3 + Horner in W^j) against the CPU oracle.

Same gates as the main scheme: (m, s) identical unless a norm lies within 1e-6 relative of a switch point
(then one of the corner choices); relative Frobenius error <= 1e-11 (fp64) / 5e-5 (fp32).
"""
import itertools

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

U64 = 2.0 ** -53
U32 = 2.0 ** -24
GATE = {np.dtype(np.float64): 1e-11, np.dtype(np.float32): 5e-5}


@pytest.fixture(scope="module")
def ex():
    import torch
    import paper_2512_20777_amd as ex
    assert torch.cuda.is_available()
    ex.load_library()
    return ex


def _corners(norms, tol):
    from oracle import oracle_select_ps_from_norms
    out = set()
    for f in itertools.product((1 - 1e-6, 1 + 1e-6), repeat=4):
        out.add(oracle_select_ps_from_norms(*(norms[i] * f[i] for i in range(4)), tol))
    return out


def _run(ex, a, tol=None, label=""):
    import torch
    from oracle import oracle_expm_ps_batch
    tol = (U32 if a.dtype == np.float32 else U64) if tol is None else tol
    X, info = oracle_expm_ps_batch(a, tol)
    d = torch.from_numpy(a).cuda()
    print("case %s shape %s %s" % (label, a.shape, a.dtype), flush=True)
    out, status = ex.expm(d, tol, scheme=ex.SCHEME_PS)
    torch.cuda.synchronize()
    stats = ex.expm_get_stats()
    got = out.cpu().numpy().astype(np.float64)
    m, s, _ = ex.expm_select(d, tol, scheme=ex.SCHEME_PS)
    worst = 0.0
    for b in range(a.shape[0]):
        ref = X[b]
        if (m[b], s[b]) != (info["m"][b], info["s"][b]):
            assert info["near"][b], "%s matrix %d: GPU (%d,%d) oracle (%d,%d)" % (label, b, m[b], s[b], info["m"][b], info["s"][b])
            assert (int(m[b]), int(s[b])) in _corners(info["norms"][b], tol)
            from oracle import oracle_expm_forced   # the neighbouring choice: the Taylor polynomial of that order
            ref = oracle_expm_forced(a[b], int(m[b]), int(s[b]), plus16=False)
        err = np.linalg.norm(got[b] - ref) / np.linalg.norm(ref)
        worst = max(worst, err)
        assert err <= GATE[a.dtype], "%s matrix %d (m=%d s=%d): %.3e" % (label, b, m[b], s[b], err)
    print("   worst rel Frobenius error %.3e, status %d" % (worst, status), flush=True)
    return got, m, s, info, stats


@pytest.mark.parametrize("n", [1, 7, 16, 33, 64, 96])
def test_ps_fused_fp64(ex, n):
    from paper_2512_20777_amd import workloads
    _, m, s, _, stats = _run(ex, workloads.random_stack(500 + n, 29, n, np.float64, 1e-4, 60.0), label="ps fused64 n=%d" % n)
    assert stats["fused_path"] == 1 and stats["scheme"] == 1


@pytest.mark.parametrize("n", [4, 16, 47, 80, 128])
def test_ps_fused_fp32(ex, n):
    from paper_2512_20777_amd import workloads
    _run(ex, workloads.random_stack(600 + n, 33, n, np.float32, 1e-4, 60.0, kind="skew" if n % 2 else "dense"),
         label="ps fused32 n=%d" % n)


@pytest.mark.parametrize("n,batch,dtype", [(97, 4, np.float64), (200, 3, np.float64), (257, 2, np.float64),
                                           (129, 4, np.float32), (250, 3, np.float32), (515, 2, np.float32)])
def test_ps_rounds(ex, n, batch, dtype):
    from paper_2512_20777_amd import workloads
    _, m, s, _, stats = _run(ex, workloads.random_stack(700 + n, batch, n, dtype, 0.05, 80.0), label="ps rounds n=%d" % n)
    assert stats["fused_path"] == 0


@pytest.mark.parametrize("n,dtype", [(1024, np.float64), (1030, np.float64), (1152, np.float32)])
def test_ps_rounds_128_tiles(ex, n, dtype):
    """From n = 1024 on the Paterson-Stockmeyer rounds run in 128x128 tiles behind a preparation pass (top Horner
    block): full tiles (operands straight into LDS) and a ragged size, eight matrices so the shape is kept."""
    from paper_2512_20777_amd import workloads
    _, m, s, _, stats = _run(ex, workloads.random_stack(720 + n, 8, n, dtype, 0.05, 25.0), label="ps rounds 128-tiles n=%d" % n)
    assert stats["fused_path"] == 0 and len(set(int(x) for x in m)) >= 2


@pytest.mark.parametrize("n", [40, 144])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_ps_all_orders_in_one_batch(ex, n, dtype):
    from paper_2512_20777_amd import workloads
    norms = np.array([0.0, 1e-10, 1e-9, 1e-6, 1e-4, 2e-3, 2e-2, 0.1, 0.3, 0.8, 2.0, 5.0, 20.0, 80.0, 300.0])
    a = workloads.random_stack(78, len(norms), n, np.float64, 1.0, 1.0)
    a = (a * norms[:, None, None]).astype(dtype)
    _, m, s, info, stats = _run(ex, a, label="ps all-orders n=%d" % n)
    assert set(np.unique(m)) >= {0, 1, 2, 4, 6, 9, 12, 16}
    assert stats["products"] == int(workloads.products_for(m, s, scheme="ps").sum())


def test_ps_workloads_c1_c2_c3(ex):
    from paper_2512_20777_amd import workloads
    for name in ("C1", "C2", "C3"):
        _run(ex, workloads.make_workload(name), label="ps " + name)


def test_ps_workload_c4(ex):
    from paper_2512_20777_amd import workloads
    _run(ex, workloads.make_workload("C4"), label="ps C4")


def test_ps_and_main_scheme_agree_and_ps_costs_more_products(ex):
    """On-device cross-check of the two schemes, and the paper's observation that Paterson-Stockmeyer needs
    more products for the same tolerance (about 1.2x on its test-bed, Sec. 4.1)."""
    import torch
    from paper_2512_20777_amd import workloads
    a = workloads.make_workload("C3")
    d = torch.from_numpy(a).cuda()
    xa, _ = ex.expm(d)
    xa = xa.clone()
    pa = ex.expm_get_stats()["products"]
    xb, _ = ex.expm(d, scheme=ex.SCHEME_PS)
    pb = ex.expm_get_stats()["products"]
    rel = (torch.linalg.norm((xa - xb).double(), dim=(1, 2)) / torch.linalg.norm(xa.double(), dim=(1, 2))).max()
    assert float(rel) < 5e-5
    assert pb > pa
    print("   products: formulas of Sec. 3.1 %d, Paterson-Stockmeyer %d (ratio %.2f)" % (pa, pb, pb / pa), flush=True)
