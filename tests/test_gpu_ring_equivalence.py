"""The 32 x 32 tiles' k-loop (ring of four LDS stages, counted waits, bare barrier) against the 64 x 64 tiles'
(two stages, full waits): two independent pipelines that add up every element's products in the same order, so for
sizes that are a multiple of 64 (both fetch straight into LDS, the first chain round included) the results have to
agree bit for bit -- a much sharper check on the ring's synchronisation than the oracle's tolerance."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.gpu
def test_thin_tile_ring_matches_the_two_stage_kernel_bit_for_bit(tmp_path):
    child = os.path.join(HERE, "ring_equivalence_child.py")
    path = str(tmp_path / "thin.npz")
    env = dict(os.environ)
    env.pop("EXPM_FORCE_WT", None)   # small batches: the library picks the 32 x 32 tiles itself
    r = subprocess.run([sys.executable, child, "write", path], env=env, capture_output=True, text=True, timeout=300)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0
    env["EXPM_FORCE_WT"] = "2"
    r = subprocess.run([sys.executable, child, "check", path], env=env, capture_output=True, text=True, timeout=300)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0
