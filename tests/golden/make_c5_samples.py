"""Write tests/golden/c5_samples_{f64,f32}.npz: sampled entries of the ORACLE's result on the
largest workload (4 matrices of order 4096), for the full-size GPU parity test.

Calls only the CPU oracle and the seeded input generator; nothing here touches the GPU library.
Takes roughly ten minutes per dtype on 8 host cores.  Usage (from the repository root):

    python tests/golden/make_c5_samples.py [f64|f32|both] [threads]

Stored per dtype: sample index pairs (seeded), the oracle values at those entries, the Frobenius
norm of each full oracle result, and the oracle's (m, s, ||W||_1, ||W^2||_1, near) per matrix; and, so that
every 128 x 128 tile of the result is gated and not only the sampled entries: the Frobenius norm of every tile,
one bilinear probe u_I^T X_IJ v_J per tile (u, v seeded vectors of +-1, stored), and all row and column sums.
"""
import importlib.util
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import oracle_expm_batch  # noqa: E402

_spec = importlib.util.spec_from_file_location(
    "expm_workloads", os.path.join(ROOT, "paper_2512_20777_amd", "workloads.py"))
workloads = importlib.util.module_from_spec(_spec)
sys.modules["expm_workloads"] = workloads
_spec.loader.exec_module(workloads)

N_SAMPLES = 4096
SAMPLE_SEED = 20251220
TILE = 128


def tile_digest(X: np.ndarray, u: np.ndarray, v: np.ndarray):
    """Per 128 x 128 tile of X: Frobenius norm and the probe u_I^T X_IJ v_J; plus row and column sums of X."""
    n = X.shape[0]
    t = n // TILE
    sq = (X * X).reshape(t, TILE, t, TILE).sum(axis=(1, 3))
    probe = ((u[:, None] * X) * v[None, :]).reshape(t, TILE, t, TILE).sum(axis=(1, 3))
    return np.sqrt(sq), probe, X.sum(axis=1), X.sum(axis=0)


def sample_indices(n: int, batch: int):
    rng = np.random.default_rng(SAMPLE_SEED)
    rows = rng.integers(0, n, size=(batch, N_SAMPLES))
    cols = rng.integers(0, n, size=(batch, N_SAMPLES))
    # always include the diagonal corners and a few diagonal entries
    rows[:, :4] = np.array([0, n - 1, 0, n - 1])
    cols[:, :4] = np.array([0, n - 1, n - 1, 0])
    return rows, cols


def main():
    which = sys.argv[1] if len(sys.argv) > 1 else "both"
    threads = int(sys.argv[2]) if len(sys.argv) > 2 else 0
    names = {"f64": ["C5f64"], "f32": ["C5f32"], "both": ["C5f64", "C5f32"]}[which]
    for name in names:
        w = workloads.WORKLOADS[name]
        a = workloads.make_workload(name)
        t0 = time.time()
        X, info = oracle_expm_batch(a, w.tol, threads)
        dt = time.time() - t0
        rows, cols = sample_indices(w.n, w.batch)
        vals = np.stack([X[b, rows[b], cols[b]] for b in range(w.batch)])
        fro = np.array([np.linalg.norm(X[b]) for b in range(w.batch)])
        prng = np.random.default_rng(SAMPLE_SEED + 1)
        u = prng.integers(0, 2, size=w.n).astype(np.float64) * 2.0 - 1.0
        v = prng.integers(0, 2, size=w.n).astype(np.float64) * 2.0 - 1.0
        dig = [tile_digest(X[b], u, v) for b in range(w.batch)]
        out = os.path.join(ROOT, "tests", "golden", "c5_samples_%s.npz" % w.dtype)
        np.savez_compressed(out, rows=rows.astype(np.int32), cols=cols.astype(np.int32), vals=vals, fro=fro,
                            m=info["m"], s=info["s"], n1=info["n1"], n2=info["n2"],
                            near=info["near"].astype(np.int8), oracle_seconds=np.array([dt]),
                            probe_u=u.astype(np.int8), probe_v=v.astype(np.int8),
                            tile_fro=np.stack([d[0] for d in dig]), tile_probe=np.stack([d[1] for d in dig]),
                            rowsum=np.stack([d[2] for d in dig]), colsum=np.stack([d[3] for d in dig]),
                            oracle_threads=np.array([info["threads"]]))
        print(name, "m", info["m"], "s", info["s"], "seconds %.1f" % dt, "threads", info["threads"], "->", out,
              flush=True)


if __name__ == "__main__":
    main()
