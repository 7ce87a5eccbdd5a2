"""Host-side checks that need no GPU: the shared library loads, exports every symbol the public
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "expm_mi355x.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2512_20777_amd as ex
    if not os.path.exists(ex.library_path()):
        from paper_2512_20777_amd.build import build_library
        build_library()
    return ex.load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:int|size_t|const char \*)\s*\*?\s*(expm\w*)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_header_declares_the_boundary():
    names = _declared_functions()
    for must in ("expm", "expm_select", "expm_workspace_bytes", "expm_get_stats", "expm_status_string"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in _declared_functions():
        assert hasattr(lib, name), name


def test_status_strings(lib):
    for code in (0, 1, 2, -1, -2, -3, -4):
        s = lib.expm_status_string(code).decode()
        assert s and s != "unknown status"
    assert lib.expm_status_string(77).decode() == "unknown status"


def test_argument_validation_happens_before_any_device_work(lib):
    i32p = ctypes.POINTER(ctypes.c_int32)
    m = (ctypes.c_int32 * 4)()
    s = (ctypes.c_int32 * 4)()
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: every call below must fail in validation
    null = ctypes.c_void_p(0)
    mp, sp = ctypes.cast(m, i32p), ctypes.cast(s, i32p)
    assert lib.expm_select(null, 8, 4, 1, 0.0, mp, sp) == -1          # null input
    assert lib.expm_select(fake, -1, 4, 1, 0.0, mp, sp) == -1         # n < 0
    assert lib.expm_select(fake, 8, -2, 1, 0.0, mp, sp) == -1         # batch < 0
    assert lib.expm_select(fake, 8, 4, 7, 0.0, mp, sp) == -1          # unknown dtype
    assert lib.expm_select(fake, 8, 4, 1, -1e-8, mp, sp) == -2        # negative tolerance
    assert lib.expm_select(fake, 8, 4, 1, float("nan"), mp, sp) == -2
    assert lib.expm_select(fake, 8, 4, 1, 1e-17, mp, sp) == -2        # below fp64 unit roundoff
    assert lib.expm_select(fake, 8, 4, 0, 1e-9, mp, sp) == -2         # below fp32 unit roundoff
    assert lib.expm_select(fake, 8, 4, 1, 0.0, ctypes.cast(None, i32p), sp) == -1
    assert lib.expm(fake, 8, 4, 1, 0.0, null, null) == -1             # null output
    assert lib.expm(fake, 8, 4, 1, 0.0, fake, null) == -1             # output overlaps input
    assert lib.expm(fake, 8, 4, 1, 0.0, ctypes.c_void_p(0x1000 + 8 * 64), null) == -1  # partial overlap
    assert lib.expm(fake, 8, 4, 1, 1e-20, ctypes.c_void_p(0x100000), null) == -2
    # empty problems succeed without work
    assert lib.expm(null, 0, 4, 1, 0.0, null, null) == 0
    assert lib.expm(null, 8, 0, 1, 0.0, null, null) == 0
    assert lib.expm_select(null, 8, 0, 1, 0.0, mp, sp) == 0
    assert lib.expm_select(null, 0, 4, 1, 0.0, mp, sp) == 0 and list(m) == [0, 0, 0, 0]


def test_noalloc_entry_point_refuses_oversized_shapes_without_a_device(lib):
    fake = ctypes.c_void_p(0x1000)
    far = ctypes.c_void_p(0x1000 + (1 << 40))
    assert lib.expm_workspace_bytes(512, 32, 1) > (64 << 20)
    assert lib.expm_noalloc(fake, 512, 32, 1, 0.0, far, None) == -6
    assert lib.expm_noalloc(fake, -1, 32, 1, 0.0, far, None) == -1
    assert "workspace" in lib.expm_status_string(-6).decode()


def test_workspace_size_formula(lib):
    assert lib.expm_workspace_bytes(0, 4, 1) == 0
    assert lib.expm_workspace_bytes(16, -1, 0) == 0
    small = lib.expm_workspace_bytes(16, 4096, 0)
    assert 0 < small < 1 << 20                       # fused path: control records only
    big = lib.expm_workspace_bytes(4096, 4, 1)
    assert big >= 7 * 4 * 4096 * 4096 * 8            # W2 and six temporaries per matrix
    assert big < 7.2 * 4 * 4096 * 4096 * 8


def test_binding_refuses_host_tensors():
    import torch
    import paper_2512_20777_amd as ex
    with pytest.raises(ex.ExpmError):
        ex.expm(torch.zeros(2, 4, 4, dtype=torch.float64))
    with pytest.raises(ex.ExpmError):
        ex.expm_select(torch.zeros(2, 4, 4, dtype=torch.float64))


def test_coefficient_tables_in_the_kernel_header_are_the_printed_ones(golden_dir):
    """The literals compiled into the HIP kernels equal the paper's tables (tests/golden fixture)."""
    from conftest import read_coefficients
    co = read_coefficients(os.path.join(golden_dir, "paper_coefficients.txt"))
    text = open(os.path.join(ROOT, "paper_2512_20777_amd", "csrc", "expm_internal.h")).read()
    defs = dict(re.findall(r"#define\s+(EXPM_T(?:8|15)_C\d+)\s+(\S+)", text))
    assert len(defs) == 6 + 16
    for k, v in co["T8"].items():
        assert float(defs["EXPM_T8_" + k.upper()]) == v
    for k, v in co["T15+"].items():
        assert float(defs["EXPM_T15_" + k.upper()]) == v


def test_selection_rule_of_the_library_matches_the_oracle_on_a_grid_of_norms(tmp_path):
    """The library's scalar selection (host+device inline function) compiled for the host against
    the oracle's, on a grid of (n1, n2) pairs and three tolerances: identical away from switch points."""
    import subprocess
    import numpy as np
    from oracle import oracle_select_from_norms
    src = tmp_path / "sel.cpp"
    src.write_text(
        '#include <cstdio>\n#include <cstdlib>\n#include <cmath>\n'
        '#define __host__\n#define __device__\n#define __forceinline__ inline\n'
        'namespace hipstub {}\n'
        + _selection_source() +
        'int main() { double n1, n2, eps; while (scanf("%lf %lf %lf", &n1, &n2, &eps) == 3) {'
        ' int m, s, f; expmk::select_order_scaling(n1, n2, eps, m, s, f); printf("%d %d %d\\n", m, s, f); } return 0; }\n')
    exe = tmp_path / "sel"
    subprocess.run(["g++", "-O1", "-o", str(exe), str(src)], check=True)
    rng = np.random.default_rng(17)
    cases = []
    for eps in (2.0 ** -53, 2.0 ** -24, 1e-8):
        for _ in range(1500):
            n1 = float(10.0 ** rng.uniform(-9, 7))
            n2 = float(n1 * n1 * 10.0 ** rng.uniform(-3, 0))
            cases.append((n1, n2, eps))
        # the scaling switches exactly where a term equals eps * 2^(16 k) or eps * 2^(17 k): hit those points
        # (n2 = n1^2: E1 = |1/16! - b16| n1^16) and their neighbours
        d16 = 2.1711086342891295e-14
        for k in range(1, 22):
            x = (eps * 2.0 ** (16 * k) / d16) ** (1.0 / 16.0)
            for f in (1 - 3e-6, 1 - 1e-9, 1.0, 1 + 1e-9, 1 + 3e-6):
                cases.append((x * f, (x * f) ** 2, eps))
    out = subprocess.run([str(exe)], input="".join("%r %r %r\n" % c for c in cases), capture_output=True, text=True,
                         check=True)
    got = [tuple(int(x) for x in ln.split()[:2]) for ln in out.stdout.splitlines()]
    assert len(got) == len(cases)
    seen_s = set()
    for (n1, n2, eps), (m, s) in zip(cases, got):
        exp = oracle_select_from_norms(n1, n2, eps)
        corners = {oracle_select_from_norms(n1 * a, n2 * b, eps) for a in (1 - 1e-6, 1 + 1e-6) for b in (1 - 1e-6, 1 + 1e-6)}
        if len(corners) == 1:
            assert (m, s) == exp, (n1, n2, eps, (m, s), exp)
        else:
            assert (m, s) in corners, (n1, n2, eps, (m, s), corners)
        seen_s.add(s)
    assert seen_s >= set(range(0, 21))   # every scaling up to the cap was exercised


def test_cap_warning_only_when_more_than_twenty_squarings_are_asked_for(tmp_path):
    """Algorithm 4 clips s to 20 only when more is asked for: a scaling of exactly 20 meets the tolerance and is not
    flagged; 21 and beyond (or an error term that is not finite) are clipped to 20 and flagged.  Expected values from
    an exact rational evaluation of the two error terms."""
    import math
    import subprocess
    from fractions import Fraction
    src = tmp_path / "cap.cpp"
    src.write_text(
        '#include <cstdio>\n#include <cstdlib>\n#include <cmath>\n'
        '#define __host__\n#define __device__\n#define __forceinline__ inline\n'
        + _selection_source() +
        'int main() { double n1, n2, eps; while (scanf("%lf %lf %lf", &n1, &n2, &eps) == 3) {'
        ' int m, s, f; expmk::select_order_scaling(n1, n2, eps, m, s, f); printf("%d %d %d\\n", m, s, f); } return 0; }\n')
    exe = tmp_path / "cap"
    subprocess.run(["g++", "-O1", "-o", str(exe), str(src)], check=True)
    c1 = Fraction(4.018761610201036e-4)
    d16 = abs(Fraction(1, math.factorial(16)) - c1 ** 4)

    def exact(n1, n2, eps):
        e1 = d16 * Fraction(n2) ** 8
        e2 = Fraction(n2) ** 8 * Fraction(n1) / math.factorial(17)
        s = 0
        while e1 > Fraction(eps) * 2 ** (16 * s) or e2 > Fraction(eps) * 2 ** (17 * s):
            s += 1
        return s

    cases = []
    for eps in (2.0 ** -53, 1e-8):
        x20 = (eps * 2.0 ** (16 * 20) / float(d16)) ** (1.0 / 16.0)      # E1 = eps 2^(16 20) for W = x I
        for f in (0.5, 0.97, 1 - 1e-4, 1 + 1e-4, 1.05, 2.0, 1e3):
            cases.append((x20 * f, (x20 * f) ** 2, eps))
    cases.append((1e200, 1e300, 2.0 ** -53))                               # n2^8 overflows: not finite
    out = subprocess.run([str(exe)], input="".join("%r %r %r\n" % c for c in cases), capture_output=True, text=True,
                         check=True)
    got = [tuple(int(x) for x in ln.split()) for ln in out.stdout.splitlines()]
    seen = set()
    for (n1, n2, eps), (m, s, flag) in zip(cases[:-1], got[:-1]):
        want = exact(n1, n2, eps)
        assert m == 15 and s == min(want, 20), (n1, eps, s, want)
        assert flag == (2 if want > 20 else 0), (n1, eps, s, want, flag)
        seen.add(min(want, 21))
    assert {20, 21} <= seen and min(seen) < 20
    assert got[-1] == (15, 20, 2)


def test_term_rounds_enqueued_for_the_baseline_cover_the_tolerance(tmp_path):
    """Rounds the baseline (Algorithm 1) enqueues above the on-chip sizes: ||Y_t|| <= (1/2)^t / t!, so once that
    bound is at most eps no further term can be added; checked in exact rationals."""
    import math
    import subprocess
    from fractions import Fraction
    text = open(os.path.join(ROOT, "paper_2512_20777_amd", "csrc", "expm_internal.h")).read()
    a = text.index("__host__ __device__ inline int baseline_max_terms(double eps)")
    b = text.index("template <typename T>", a)
    src = tmp_path / "terms.cpp"
    src.write_text('#include <cstdio>\n#define __host__\n#define __device__\n' + text[a:b] +
                   'int main() { double e; while (scanf("%lf", &e) == 1) printf("%d\\n", baseline_max_terms(e)); return 0; }\n')
    exe = tmp_path / "terms"
    subprocess.run(["g++", "-O1", "-o", str(exe), str(src)], check=True)
    eps_list = [2.0 ** -53, 2.0 ** -24, 1e-8, 1e-3, 0.2]   # tolerances below the fp64 unit roundoff are rejected earlier
    out = subprocess.run([str(exe)], input="".join("%r\n" % e for e in eps_list), capture_output=True, text=True, check=True)
    got = [int(x) for x in out.stdout.split()]
    for eps, rounds in zip(eps_list, got):
        t = 1
        while Fraction(1, 2) ** t / math.factorial(t) > Fraction(eps):
            t += 1
        # term t is never added, so t - 1 rounds do the work; the library keeps two spare
        assert t - 1 <= rounds <= t + 2, (eps, t, rounds)
    assert got[0] > got[2] > got[4]


def test_paterson_stockmeyer_selection_of_the_library_matches_the_oracle(tmp_path):
    """Same check for the selection of the Paterson-Stockmeyer variant (four power norms)."""
    import subprocess
    import numpy as np
    from oracle import oracle_select_ps_from_norms
    src = tmp_path / "selps.cpp"
    src.write_text(
        '#include <cstdio>\n#include <cstdlib>\n#include <cmath>\n'
        '#define __host__\n#define __device__\n#define __forceinline__ inline\n'
        + _selection_source("// Products after the powers") +
        'int main() { double n[4], eps; while (scanf("%lf %lf %lf %lf %lf", &n[0], &n[1], &n[2], &n[3], &eps) == 5) {'
        ' int m, s, f; bool more; expmk::select_ps_order_scaling(n, 4, eps, m, s, f, more); printf("%d %d\\n", m, s); }'
        ' return 0; }\n')
    exe = tmp_path / "selps"
    subprocess.run(["g++", "-O1", "-o", str(exe), str(src)], check=True)
    rng = np.random.default_rng(23)
    cases = []
    for eps in (2.0 ** -53, 2.0 ** -24, 1e-8):
        for _ in range(1200):
            n1 = float(10.0 ** rng.uniform(-9, 7))
            n2 = float(n1 ** 2 * 10.0 ** rng.uniform(-2, 0))
            n3 = float(n1 * n2 * 10.0 ** rng.uniform(-1, 0))
            n4 = float(n2 * n2 * 10.0 ** rng.uniform(-1, 0))
            cases.append((n1, n2, n3, n4, eps))
    out = subprocess.run([str(exe)], input="".join("%r %r %r %r %r\n" % c for c in cases), capture_output=True,
                         text=True, check=True)
    got = [tuple(int(x) for x in ln.split()) for ln in out.stdout.splitlines()]
    assert len(got) == len(cases)
    seen_s = set()
    for c, ms in zip(cases, got):
        n1, n2, n3, n4, eps = c
        exp = oracle_select_ps_from_norms(n1, n2, n3, n4, eps)
        corners = {oracle_select_ps_from_norms(n1 * a, n2 * b, n3 * b, n4 * b, eps)
                   for a in (1 - 1e-6, 1 + 1e-6) for b in (1 - 1e-6, 1 + 1e-6)}
        if len(corners) == 1:
            assert ms == exp, (c, ms, exp)
        seen_s.add(ms[1])
    assert seen_s >= set(range(0, 21))


def _selection_source(end_marker="// Rounds after the W^2 product"):
    """The selection function and its constants cut out of the kernel header (plain C++ once the
    HIP qualifiers are defined away)."""
    text = open(os.path.join(ROOT, "paper_2512_20777_amd", "csrc", "expm_internal.h")).read()
    start = text.index("#define EXPM_T8_C1")
    end = text.index(end_marker)
    return "namespace expmk {\n" + text[start:end] + "}\n"
