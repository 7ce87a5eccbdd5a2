"""Child process of test_gpu_ring_equivalence.py: runs expm() on fixed seeded inputs and either stores the results
or compares them, bit for bit, with the stored ones.  The tile shape is pinned by the parent through the
library's EXPM_FORCE_WT debugging aid, which is read once per process -- hence a process of its own per shape."""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

CASES = [(192, np.float32, 2), (256, np.float32, 1), (320, np.float32, 3), (512, np.float32, 1), (192, np.float64, 1),
         (256, np.float64, 2), (448, np.float64, 1), (512, np.float64, 4), (768, np.float64, 1)]


def main():
    import torch
    import paper_2512_20777_amd as ex
    from paper_2512_20777_amd import workloads
    mode, path = sys.argv[1], sys.argv[2]
    ex.load_library()
    stored = dict(np.load(path)) if mode == "check" else {}
    results, bad = {}, 0
    for n, dtype, batch in CASES:
        a = workloads.random_stack(77 + n, batch, n, dtype, 5.0, 90.0)
        d = torch.from_numpy(a).cuda()
        key = "%d_%s_%d" % (n, np.dtype(dtype).name, batch)
        print("case %s (%s)" % (key, mode), flush=True)
        first = None
        for rep in range(10):
            x = ex.expm(d)[0].cpu().numpy()
            if first is None:
                first = x
            elif not np.array_equal(first.view(np.uint8), x.view(np.uint8)):
                print("   repetition %d differs from the first" % rep, flush=True)
                bad += 1
        results[key] = first
        if mode == "check" and not np.array_equal(stored[key].view(np.uint8), first.view(np.uint8)):
            diff = np.abs(stored[key].astype(np.float64) - first.astype(np.float64)).max()
            print("   differs from the other tile shape, max abs difference %.3e" % diff, flush=True)
            bad += 1
    if mode == "write":
        np.savez(path, **results)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main())
