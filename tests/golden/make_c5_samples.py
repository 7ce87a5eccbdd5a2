"""Write tests/golden/c5_samples_{f64,f32}.npz: sampled entries of the ORACLE's result on the
largest workload (4 matrices of order 4096), for the full-size GPU parity test.

Calls only the CPU oracle and the seeded input generator; nothing here touches the GPU library.
Takes roughly ten minutes per dtype on 8 host cores.  Usage (from the repository root):

    python tests/golden/make_c5_samples.py [f64|f32|both] [threads]

Stored per dtype: sample index pairs (seeded), the oracle values at those entries, the Frobenius
norm of each full oracle result, and the oracle's (m, s, ||W||_1, ||W^2||_1, near) per matrix.
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
        out = os.path.join(ROOT, "tests", "golden", "c5_samples_%s.npz" % w.dtype)
        np.savez_compressed(out, rows=rows.astype(np.int32), cols=cols.astype(np.int32), vals=vals, fro=fro,
                            m=info["m"], s=info["s"], n1=info["n1"], n2=info["n2"],
                            near=info["near"].astype(np.int8), oracle_seconds=np.array([dt]),
                            oracle_threads=np.array([info["threads"]]))
        print(name, "m", info["m"], "s", info["s"], "seconds %.1f" % dt, "threads", info["threads"], "->", out,
              flush=True)


if __name__ == "__main__":
    main()
