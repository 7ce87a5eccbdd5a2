"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI.

Gates: (m, s) identical except for matrices whose norms lie within
1e-6 relative of a selection switch point (then the result must equal one of the corner choices);
relative Frobenius error per matrix <= 1e-11 (fp64) / 5e-5 (fp32).
"""
import ctypes
import os

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
    assert torch.cuda.is_available(), "GPU tests need a device"
    ex.load_library()  # raises if the HIP library is not built: no fallback
    return ex


def _tol(a):
    return U32 if a.dtype == np.float32 else U64


def _corner_choices(n1, n2, tol):
    from oracle import oracle_select_from_norms
    out = set()
    for f1 in (1 - 1e-6, 1 + 1e-6):
        for f2 in (1 - 1e-6, 1 + 1e-6):
            out.add(oracle_select_from_norms(n1 * f1, max(n2, 0.0) * f2, tol))
    return out


def _check_ms(m, s, info, tol, label):
    for b in range(len(m)):
        if m[b] == info["m"][b] and s[b] == info["s"][b]:
            continue
        assert info["near"][b], "%s matrix %d: GPU (m,s)=(%d,%d) oracle (%d,%d) and not near a switch point" % (
            label, b, m[b], s[b], info["m"][b], info["s"][b])
        assert (int(m[b]), int(s[b])) in _corner_choices(info["n1"][b], info["n2"][b], tol), (label, b)


def _run_and_check(ex, a, tol=None, label="", gate=None):
    import torch
    from oracle import oracle_expm_batch
    tol = _tol(a) if tol is None else tol
    gate = GATE[a.dtype] if gate is None else gate
    X, info = oracle_expm_batch(a, tol)
    d = torch.from_numpy(a).cuda()
    print("case %s shape %s dtype %s" % (label, a.shape, a.dtype), flush=True)
    out, status = ex.expm(d, tol)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    stats = ex.expm_get_stats()  # of the expm() call
    m, s, st2 = ex.expm_select(d, tol)
    _check_ms(m, s, info, tol, label)
    worst = 0.0
    for b in range(a.shape[0]):
        ref = X[b]
        if (m[b], s[b]) != (info["m"][b], info["s"][b]):
            # a near-switch matrix evaluated with the other admissible choice: the oracle's polynomial for that pair
            from oracle import oracle_expm_forced
            ref = oracle_expm_forced(a[b], int(m[b]), int(s[b]))
            print("   matrix %d takes the neighbouring choice (%d,%d), oracle (%d,%d): compared against that polynomial"
                  % (b, m[b], s[b], info["m"][b], info["s"][b]), flush=True)
        den = np.linalg.norm(ref)
        err = np.linalg.norm(got[b] - ref) / den
        worst = max(worst, err)
        assert err <= gate, "%s matrix %d (m=%d s=%d): rel Frobenius error %.3e > %.1e" % (
            label, b, m[b], s[b], err, gate)
    print("   worst rel Frobenius error %.3e (gate %.1e), status %d" % (worst, gate, status), flush=True)
    return got, m, s, info, stats


# ------------------------------------------------------------------------------------------------
# fused single-kernel path (n <= 128 fp32, n <= 96 fp64)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n", [1, 2, 5, 16, 17, 31, 32, 33, 48, 63, 70, 81, 96])
def test_fused_fp64_sizes(ex, n):
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(100 + n, 37, n, np.float64, 1e-3, 60.0)
    _, m, s, info, stats = _run_and_check(ex, a, label="fused64 n=%d" % n)
    assert stats["fused_path"] == 1


@pytest.mark.parametrize("n", [1, 3, 16, 20, 32, 47, 49, 64, 77, 90, 100, 113, 128])
def test_fused_fp32_sizes(ex, n):
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(200 + n, 41, n, np.float32, 1e-3, 60.0, kind="skew" if n % 2 else "dense")
    _, m, s, info, stats = _run_and_check(ex, a, label="fused32 n=%d" % n)
    assert stats["fused_path"] == 1


def test_workload_c1_full(ex):
    from paper_2512_20777_amd import workloads
    _, m, s, info, stats = _run_and_check(ex, workloads.make_workload("C1"), label="C1")
    assert stats["fused_path"] == 1 and stats["matrices"] == 16
    assert stats["products"] == int(workloads.products_for(m, s).sum())


def test_workload_c2_full(ex):
    from paper_2512_20777_amd import workloads
    _, m, s, info, stats = _run_and_check(ex, workloads.make_workload("C2"), label="C2")
    assert stats["fused_path"] == 1 and stats["matrices"] == 4096
    assert set(np.unique(m)) >= {4, 8, 15}  # the flow-layer norm range exercises the low orders too


# ------------------------------------------------------------------------------------------------
# round-based path (larger n): several tiles, ragged tails, aligned and unaligned row lengths
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,batch", [(97, 5), (128, 4), (130, 3), (200, 3), (257, 2), (384, 2)])
def test_rounds_fp64_sizes(ex, n, batch):
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(300 + n, batch, n, np.float64, 0.05, 80.0)
    _, m, s, info, stats = _run_and_check(ex, a, label="rounds64 n=%d" % n)
    assert stats["fused_path"] == 0


@pytest.mark.parametrize("n,batch", [(129, 5), (136, 3), (192, 6), (250, 3), (300, 2), (515, 2)])
def test_rounds_fp32_sizes(ex, n, batch):
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(400 + n, batch, n, np.float32, 0.05, 80.0)
    _, m, s, info, stats = _run_and_check(ex, a, label="rounds32 n=%d" % n)
    assert stats["fused_path"] == 0


# 32x32 tiles straight into LDS (small batches of full-tile sizes) keep three k-blocks in flight in a ring of four
# stages: a loop of four steps and a tail of three to six.  k-blocks are 32 (fp32) or 16 (fp64) wide, so these sizes
# give every tail length after zero, one or several turns of the loop, and a single matrix gives the first chain
# round its 32x32 variant with the third tile per stage.
@pytest.mark.parametrize("n,dtype", [(160, np.float32), (224, np.float32), (288, np.float32), (320, np.float32),
                                     (352, np.float32), (416, np.float32), (160, np.float64), (224, np.float64),
                                     (288, np.float64), (352, np.float64)])
def test_rounds_thin_tiles_ring_every_tail_length(ex, n, dtype):
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(900 + n, 2, n, dtype, 0.5, 120.0)
    a[0] *= 60.0 / np.abs(a[0]).sum(axis=0).max()   # order 15+ with several squarings
    a[1] *= 0.02 / np.abs(a[1]).sum(axis=0).max()   # a low order as well (its first round is the last one)
    _, m, s, info, stats = _run_and_check(ex, a, label="ring n=%d %s" % (n, np.dtype(dtype).name))
    assert stats["fused_path"] == 0 and m[0] == 15 and s[0] >= 3
    one = a[:1].copy()
    _run_and_check(ex, one, label="ring single n=%d %s" % (n, np.dtype(dtype).name))


@pytest.mark.parametrize("n,dtype", [(1030, np.float64), (1027, np.float64), (1028, np.float32), (1030, np.float32),
                                     (1152, np.float32)])
def test_rounds_128_tiles_ragged_and_full(ex, n, dtype):
    """From n = 1024 on the products run in 128x128 tiles: sizes that are not a multiple of the tile (vector loads
    with bounds checks where rows are 16-byte aligned, element-wise loads where they are not) and one that is."""
    from paper_2512_20777_amd import workloads
    # seven matrices: a launch switches to 128x128 tiles only when it has at least two such workgroups per compute unit
    a = workloads.random_stack(500 + n, 7, n, dtype, 0.3, 6.0)
    _, m, s, info, stats = _run_and_check(ex, a, label="rounds 128-tiles n=%d %s" % (n, np.dtype(dtype).name))
    assert stats["fused_path"] == 0


@pytest.mark.parametrize("n,dtype", [(1024, np.float64), (1152, np.float64), (1024, np.float32)])
def test_rounds_128_tiles_straight_to_lds_whole_matrices(ex, n, dtype):
    """Full 128x128 tiles with aligned rows: the product kernel whose operand tiles go from global memory straight
    into LDS, the one the 4096 x 4096 workloads run in, compared here on whole matrices (there: samples and per-tile
    digests).  Eight matrices, so that every round keeps the 128x128 shape; norms large enough for a few squarings."""
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(520 + n, 8, n, dtype, 0.3, 25.0 if dtype == np.float64 else 600.0)
    _, m, s, info, stats = _run_and_check(ex, a, label="rounds 128-tiles direct-to-LDS n=%d %s" % (n, np.dtype(dtype).name))
    assert stats["fused_path"] == 0 and int(s.max()) >= 1


@pytest.mark.parametrize("n", [144, 192])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_rounds_all_orders_in_one_batch(ex, dtype, n):
    """Norms from 1e-10 to 300 in one batch: every order 0,1,2,4,8,15+ and several scalings at once.  n = 192: full
    64x64 tiles, where the first chain round fetches straight into LDS and forms its combined operand (the right
    factor of y02, the left factor of T_4) from the fragments; n = 144: the same round with register staging."""
    from paper_2512_20777_amd import workloads
    norms = np.array([0.0, 1e-10, 1e-9, 1e-6, 1e-5, 1e-3, 5e-3, 0.03, 0.1, 0.4, 1.0, 3.0, 10.0, 40.0, 120.0, 300.0])
    a = workloads.random_stack(77, len(norms), n, np.float64, 1.0, 1.0)
    a = (a * norms[:, None, None]).astype(dtype)
    _, m, s, info, stats = _run_and_check(ex, a, label="all-orders n=%d %s" % (n, np.dtype(dtype).name))
    assert set(np.unique(m)) >= {0, 1, 2, 4, 8, 15}
    assert stats["hist_m"][0] == 1
    assert stats["rounds"] == 3 + int(s.max())


def test_rounds_nonnormal_triangular(ex):
    """Upper-triangular non-normal input: result keeps an exactly zero strict lower part."""
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(5, 3, 160, np.float64, 5.0, 90.0, kind="triu")
    got, m, s, info, _ = _run_and_check(ex, a, label="triu")
    for b in range(a.shape[0]):
        assert np.array_equal(np.tril(got[b], -1), np.zeros_like(got[b]))


def test_workload_c3_full(ex):
    from paper_2512_20777_amd import workloads
    _, m, s, info, stats = _run_and_check(ex, workloads.make_workload("C3"), label="C3")
    assert stats["matrices"] == 256 and stats["fused_path"] == 1


def test_workload_c4_full(ex):
    from paper_2512_20777_amd import workloads
    _run_and_check(ex, workloads.make_workload("C4"), label="C4")


@pytest.mark.parametrize("name", ["C5f64", "C5f32"])
def test_workload_c5_against_stored_oracle_samples(ex, name, golden_dir):
    """Full-size 4096x4096 batch against what tests/golden/make_c5_samples.py stored of the oracle's result (the
    oracle needs about a quarter of an hour per dtype): sampled entries, and a digest of every 128x128 tile."""
    import torch
    from paper_2512_20777_amd import workloads
    w = workloads.WORKLOADS[name]
    path = os.path.join(golden_dir, "c5_samples_%s.npz" % w.dtype)
    if not os.path.exists(path):
        pytest.skip("stored oracle samples %s not generated" % path)
    g = np.load(path)
    a = workloads.make_workload(name)
    d = torch.from_numpy(a).cuda()
    del a
    print("case %s" % name, flush=True)
    out, status = ex.expm(d, w.tol)
    torch.cuda.synchronize()
    m, s, _ = ex.expm_select(d, w.tol)
    info = dict(m=g["m"], s=g["s"], n1=g["n1"], n2=g["n2"], near=g["near"].astype(bool))
    _check_ms(m, s, info, w.tol, name)
    gate = GATE[np.dtype(w.np_dtype)]
    for b in range(w.batch):
        if (m[b], s[b]) != (info["m"][b], info["s"][b]):
            continue
        rows = torch.from_numpy(g["rows"][b].astype(np.int64)).cuda()
        cols = torch.from_numpy(g["cols"][b].astype(np.int64)).cuda()
        got = out[b][rows, cols].cpu().numpy().astype(np.float64)
        ref = g["vals"][b]
        # sampled estimate of the relative Frobenius error, and the GPU result's norm against the oracle's
        err = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        fro = float(torch.linalg.norm(out[b].double()).cpu())
        print("   %s matrix %d (m=%d s=%d): sampled rel error %.3e, Frobenius norm rel diff %.3e"
              % (name, b, m[b], s[b], err, abs(fro - g["fro"][b]) / g["fro"][b]), flush=True)
        assert err <= gate, (name, b, err)
        assert abs(fro - g["fro"][b]) <= gate * g["fro"][b]
        # Every 128 x 128 tile, not only the sampled entries: its Frobenius norm, a bilinear probe u_I^T X_IJ v_J with
        # stored vectors of +-1 (an error E in the tile moves it by about ||E||_F), and all row and column sums in
        # blocks of 128 (same reasoning), each against the oracle's stored value, scaled by the tile's (block's) norm.
        x = out[b].double()
        t = w.n // 128
        ref_fro = torch.from_numpy(g["tile_fro"][b]).cuda()
        u = torch.from_numpy(g["probe_u"].astype(np.float64)).cuda()
        v = torch.from_numpy(g["probe_v"].astype(np.float64)).cuda()
        fro_t = (x * x).reshape(t, 128, t, 128).sum(dim=(1, 3)).sqrt()
        probe = ((u[:, None] * x) * v[None, :]).reshape(t, 128, t, 128).sum(dim=(1, 3))
        d_fro = ((fro_t - ref_fro).abs() / ref_fro).max()
        d_probe = ((probe - torch.from_numpy(g["tile_probe"][b]).cuda()).abs() / ref_fro).max()
        row_fro = (ref_fro ** 2).sum(dim=1).sqrt()      # norm of each block of 128 rows
        col_fro = (ref_fro ** 2).sum(dim=0).sqrt()
        d_row = ((x.sum(dim=1) - torch.from_numpy(g["rowsum"][b]).cuda()).reshape(t, 128).norm(dim=1) / row_fro).max()
        d_col = ((x.sum(dim=0) - torch.from_numpy(g["colsum"][b]).cuda()).reshape(t, 128).norm(dim=1) / col_fro).max()
        print("      per tile: norm rel diff %.3e, probe diff / tile norm %.3e; row-block sums %.3e, column-block sums %.3e"
              % (float(d_fro), float(d_probe), float(d_row), float(d_col)), flush=True)
        assert float(d_fro) <= gate, (name, b, float(d_fro))
        assert float(d_probe) <= 8 * gate and float(d_row) <= 8 * gate and float(d_col) <= 8 * gate, (name, b)
        del x


# ------------------------------------------------------------------------------------------------
# edge cases and host-visible behaviour
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n", [8, 100])
def test_zero_matrix_gives_identity_and_m0(ex, n):
    import torch
    a = torch.zeros(3, n, n, dtype=torch.float64, device="cuda")
    out, st = ex.expm(a)
    m, s, _ = ex.expm_select(a)
    assert list(m) == [0, 0, 0] and list(s) == [0, 0, 0]
    assert torch.equal(out, torch.eye(n, dtype=torch.float64, device="cuda").expand(3, n, n))


@pytest.mark.parametrize("n", [12, 90, 140])
def test_index2_nilpotent_is_exact(ex, n):
    import torch
    a = torch.zeros(2, n, n, dtype=torch.float64, device="cuda")
    a[0, 0, n - 1] = 7.0
    a[1, 1, n - 2] = -3.0
    out, _ = ex.expm(a)
    m, s, _ = ex.expm_select(a)
    assert list(m) == [2, 2] and list(s) == [0, 0]
    assert torch.equal(out, torch.eye(n, dtype=torch.float64, device="cuda").expand(2, n, n) + a)


def test_empty_batch_and_empty_matrix(ex):
    import torch
    out, st = ex.expm(torch.zeros(0, 5, 5, dtype=torch.float32, device="cuda"))
    assert st == 0 and out.shape == (0, 5, 5)
    out, st = ex.expm(torch.zeros(4, 0, 0, dtype=torch.float64, device="cuda"))
    assert st == 0 and out.shape == (4, 0, 0)
    m, s, st = ex.expm_select(torch.zeros(0, 5, 5, dtype=torch.float32, device="cuda"))
    assert len(m) == 0 and st == 0


@pytest.mark.parametrize("n", [10, 80, 150])
def test_nonfinite_input_is_flagged_and_isolated(ex, n):
    import torch
    from oracle import oracle_expm
    rng = np.random.default_rng(1)
    a = rng.standard_normal((3, n, n)) / np.sqrt(n)
    a[1, 2, 3] = np.nan
    d = torch.from_numpy(a).cuda()
    out, st = ex.expm(d)
    torch.cuda.synchronize()
    m, s, st2 = ex.expm_select(d)
    assert st2 == 1 and (m[1], s[1]) == (-1, -1)
    assert ex.expm_get_stats()["warning"] == 1
    assert bool(torch.isnan(out[1]).all())
    for b in (0, 2):
        X, _ = oracle_expm(a[b], U64)
        got = out[b].cpu().numpy()
        assert np.linalg.norm(got - X) / np.linalg.norm(X) < 1e-11


@pytest.mark.parametrize("n", [70, 130])
def test_scaling_cap_warning(ex, n):
    import torch
    a = torch.zeros(2, n, n, dtype=torch.float64, device="cuda")
    a[0] = torch.eye(n, device="cuda", dtype=torch.float64) * 0.5
    a[1] = torch.eye(n, device="cuda", dtype=torch.float64) * -3.0e7   # needs s > 20: capped
    m, s, st = ex.expm_select(a)
    assert st == 2 and (m[1], s[1]) == (15, 20) and s[0] < 20


def test_user_tolerance_changes_the_choice_like_the_oracle(ex):
    from paper_2512_20777_amd import workloads
    for n, dt in ((24, np.float64), (150, np.float64), (40, np.float32)):
        a = workloads.random_stack(9, 12, n, dt, 1e-4, 12.8)
        for tol in ((1e-8, 1e-5) if dt == np.float64 else (1e-6, 1e-4)):
            _run_and_check(ex, a, tol=tol, label="tol=%g n=%d %s" % (tol, n, np.dtype(dt).name),
                           gate=max(GATE[np.dtype(dt)], 1e-12))


def test_results_are_bitwise_reproducible(ex):
    import torch
    from paper_2512_20777_amd import workloads
    for n, dt in ((16, np.float32), (128, np.float32), (200, np.float64), (136, np.float32)):
        d = torch.from_numpy(workloads.random_stack(3, 6, n, dt, 0.1, 50.0)).cuda()
        o1, _ = ex.expm(d)
        o1 = o1.clone()
        o2, _ = ex.expm(d)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2)


def test_runs_on_a_caller_stream_and_into_a_caller_buffer(ex):
    import torch
    from oracle import oracle_expm_batch
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(4, 4, 140, np.float64, 0.5, 20.0)
    X, _ = oracle_expm_batch(a, U64)
    d = torch.from_numpy(a).cuda()
    out = torch.empty_like(d)
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        ex.expm(d, out=out)
    st.synchronize()
    got = out.cpu().numpy()
    assert max(np.linalg.norm(got[b] - X[b]) / np.linalg.norm(X[b]) for b in range(4)) < 1e-11


def test_inverse_and_determinant_identities_at_size(ex):
    """Properties that hold at any size, on the GPU result alone (Sec. 2.2 of the paper)."""
    import torch
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(6, 2, 512, np.float64, 2.0, 6.0)
    d = torch.from_numpy(a).cuda()
    x, _ = ex.expm(d)
    x = x.clone()
    y, _ = ex.expm(-d)
    eye = torch.eye(512, dtype=torch.float64, device="cuda")
    assert float((x @ y - eye).abs().max()) < 1e-10
    sign, logdet = torch.linalg.slogdet(x)
    tr = torch.diagonal(d, dim1=-2, dim2=-1).sum(-1)
    assert bool((sign > 0).all()) and float((logdet - tr).abs().max()) < 1e-9


@pytest.mark.parametrize("n,dtype,tol", [(6144, np.float32, 2e-4), (5000, np.float64, 1e-11)])
def test_identities_beyond_the_benchmark_sizes(ex, n, dtype, tol):
    """Sizes above the largest benchmark matrix (48 x 48 tiles of 128 x 128 that do not split evenly over the XCDs;
    a ragged 5000 that leaves 8 rows and columns for the last tile), checked by what holds at any size:
    e^W e^(-W) = I and (e^(W/2))^2 = e^W (Sec. 2.2 of the paper), products taken with torch on the device."""
    import torch
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(n, 1, n, dtype, 30.0, 30.0)
    d = torch.from_numpy(a).cuda()
    print("case identities n=%d %s" % (n, np.dtype(dtype).name), flush=True)
    x = ex.expm(d)[0].clone()
    y = ex.expm(-d)[0].clone()
    h = ex.expm(0.5 * d)[0].clone()
    m, s, _ = ex.expm_select(d)
    assert m[0] == 15
    x64, y64, h64 = x[0].double(), y[0].double(), h[0].double()
    eye = torch.eye(n, dtype=torch.float64, device="cuda")
    err_inv = float((x64 @ y64 - eye).abs().max())
    err_sq = float((h64 @ h64 - x64).abs().max() / x64.abs().max())
    print("   |e^W e^-W - I|_max %.3e   |(e^(W/2))^2 - e^W|_max / |e^W|_max %.3e" % (err_inv, err_sq), flush=True)
    assert err_inv < tol and err_sq < tol


# ------------------------------------------------------------------------------------------------
# infinity-norm selection and the tolerance of the paper's own runs (Sec. 4.2: eps = 1e-8, inf-norm)
# ------------------------------------------------------------------------------------------------
def _run_inf_norm(ex, a, tol, label, scheme=0):
    """Selection on infinity-norms of W equals selection on 1-norms of W^T, and e^(W^T) = (e^W)^T:
    the oracle runs on the transposed stack and its result is transposed back."""
    import torch
    from oracle import oracle_expm_batch, oracle_expm_ps_batch
    at = np.ascontiguousarray(np.swapaxes(a, -1, -2))
    X, info = (oracle_expm_ps_batch if scheme else oracle_expm_batch)(at, tol)
    X = np.swapaxes(X, -1, -2)
    d = torch.from_numpy(a).cuda()
    print("case %s shape %s %s" % (label, a.shape, a.dtype), flush=True)
    out, _ = ex.expm(d, tol, scheme=scheme, norm=ex.NORM_INF)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    m, s, _ = ex.expm_select(d, tol, scheme=scheme, norm=ex.NORM_INF)
    m1, s1, _ = ex.expm_select(d, tol, scheme=scheme, norm=ex.NORM_ONE)
    worst = 0.0
    for b in range(a.shape[0]):
        ref = X[b]
        if (m[b], s[b]) != (info["m"][b], info["s"][b]):
            assert info["near"][b], (label, b, (m[b], s[b]), (info["m"][b], info["s"][b]))
            from oracle import oracle_expm_forced   # the neighbouring choice: the oracle's polynomial for that pair
            ref = oracle_expm_forced(at[b], int(m[b]), int(s[b]), plus16=(not scheme and m[b] == 15)).T
        err = np.linalg.norm(got[b] - ref) / np.linalg.norm(ref)
        worst = max(worst, err)
        assert err <= GATE[a.dtype], (label, b, err)
    print("   worst rel Frobenius error %.3e; matrices whose choice differs between the two norms: %d"
          % (worst, int(((m != m1) | (s != s1)).sum())), flush=True)
    return m, s, m1, s1


@pytest.mark.parametrize("n,batch,dtype", [(16, 64, np.float32), (48, 20, np.float64), (128, 8, np.float32),
                                           (150, 6, np.float64), (260, 3, np.float32), (515, 2, np.float64)])
def test_infinity_norm_selection(ex, n, batch, dtype):
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(900 + n, batch, n, dtype, 0.01, 60.0, kind="triu" if n % 2 == 0 else "dense")
    _run_inf_norm(ex, a, _tol(a), "inf-norm n=%d" % n)


@pytest.mark.parametrize("n", [24, 160])
def test_infinity_norm_really_uses_row_sums(ex, n):
    """One dense row: the 1-norm is the largest entry, the infinity-norm the sum of the row."""
    import torch
    from oracle import oracle_select
    rng = np.random.default_rng(n)
    a = np.zeros((2, n, n))
    a[0, 3, :] = rng.uniform(0.5, 1.0, n) * 0.02      # row sums ~ 0.015 n, column sums <= 0.02
    a[1, :, 5] = rng.uniform(0.5, 1.0, n) * 0.02      # the transpose situation
    d = torch.from_numpy(a).cuda()
    m1, s1, _ = ex.expm_select(d, U64, norm=ex.NORM_ONE)
    mi, si, _ = ex.expm_select(d, U64, norm=ex.NORM_INF)
    for b in range(2):
        o1 = oracle_select(a[b], U64)
        oi = oracle_select(a[b].T, U64)
        assert (m1[b], s1[b]) == (o1["m"], o1["s"]) and (mi[b], si[b]) == (oi["m"], oi["s"])
    assert (m1[0], s1[0]) != (mi[0], si[0]) and (m1[1], s1[1]) != (mi[1], si[1])
    assert (m1[0], s1[0]) == (mi[1], si[1]) and (m1[1], s1[1]) == (mi[0], si[0])


def test_infinity_norm_with_paterson_stockmeyer(ex):
    from paper_2512_20777_amd import workloads
    for n, dt in ((40, np.float64), (200, np.float32)):
        a = workloads.random_stack(950 + n, 6, n, dt, 0.01, 60.0, kind="triu")
        _run_inf_norm(ex, a, _tol(a), "inf-norm PS n=%d" % n, scheme=1)


def test_flow_setting_of_the_paper_tol_1e8_inf_norm(ex):
    """Workload F1: tolerance 1e-8, infinity-norm, norms 1e-5 .. 12.8: the low orders dominate."""
    from paper_2512_20777_amd import workloads
    w = workloads.WORKLOADS["F1"]
    a = workloads.make_workload("F1")
    m, s, m1, s1 = _run_inf_norm(ex, a, w.tol, "F1")
    hist = {int(k): int((m == k).sum()) for k in np.unique(m)}
    print("   F1 orders:", hist, "max s", int(s.max()), flush=True)
    assert hist.get(1, 0) > 0 and hist.get(2, 0) > 0 and hist.get(4, 0) > 0 and hist.get(15, 0) > 0
    assert int(s.max()) <= 3   # norm 12.8 needs s = 3 at this tolerance (the paper's worked example)


# ------------------------------------------------------------------------------------------------
# one-tile fp64 matrices (n <= 16): the register-resident kernel; every order, scaling, both norms
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n", [3, 9, 16])
def test_one_tile_fp64_all_orders_both_norms(ex, n):
    from paper_2512_20777_amd import workloads
    a = workloads.random_stack(1200 + n, 48, n, np.float64, 1e-9, 300.0, kind="dense" if n % 2 else "triu")
    a[0] = 0.0                                  # order 0
    a[1] *= 1e-12 / max(np.abs(a[1]).sum(axis=0).max(), 1e-300)   # order 1
    got, m, s, info, stats = _run_and_check(ex, a, label="one tile fp64 n=%d" % n)
    assert stats["fused_path"] == 1
    assert {0, 1, 2, 4, 8, 15} <= set(int(x) for x in m) and int(s.max()) >= 4
    _run_inf_norm(ex, a, U64, "one tile fp64 inf-norm n=%d" % n)
    _run_inf_norm(ex, a, 1e-8, "one tile fp64 inf-norm tol 1e-8 n=%d" % n)


def test_one_tile_fp64_nonfinite_and_nilpotent(ex):
    import torch
    rng = np.random.default_rng(77)
    n = 11
    a = rng.standard_normal((6, n, n)) * 0.3
    a[2, 4, 7] = np.nan
    a[4, 0, 0] = np.inf
    a[5] = np.triu(a[5], 1)                     # nilpotent: the series is finite, order 15 covers n - 1 = 10
    a[5] *= 0.4 / np.abs(a[5]).sum(axis=0).max()
    d = torch.from_numpy(a).cuda()
    out, status = ex.expm(d, U64)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    # the asynchronous call cannot report it; the statistics of the call and expm_select do
    assert ex.expm_get_stats()["warning"] == 1
    m, s, st2 = ex.expm_select(d, U64)
    assert st2 == 1 and (m[2], s[2]) == (-1, -1) and (m[4], s[4]) == (-1, -1)
    assert np.isnan(got[2]).all() and np.isnan(got[4]).all()
    for b in (0, 1, 3, 5):
        assert np.isfinite(got[b]).all()
    from oracle import oracle_expm_batch
    X, info = oracle_expm_batch(a[[0, 1, 3, 5]], U64)
    for i, b in enumerate((0, 1, 3, 5)):
        assert np.linalg.norm(got[b] - X[i]) / np.linalg.norm(X[i]) <= 1e-11
    assert np.all(np.tril(got[5], -1) == 0.0)   # upper triangular input: exact zeros below the diagonal
