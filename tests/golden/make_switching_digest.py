"""Writes ``mid_switching_digest.txt``: the digest of the switching-aware partitioner's
assignment on the ``mid`` workload, computed by the oracle alone (about half an hour of numpy).

    python tests/golden/make_switching_digest.py

The full-size GPU test compares the library's assignment with this digest, because running
the oracle's partitioner at that size inside the test would take far longer than the test may.
"""
import hashlib
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import partition as op          # noqa: E402
from synth import make_config               # noqa: E402


def main():
    cfg, rowptr, colidx = make_config("mid")
    k, seed = cfg["k"], cfg["seed"]
    t0 = time.time()
    done = [0]

    def iteration(rp, ci, part, kk, workers):
        done[0] += 1
        print("iteration %d (%.0f s)" % (done[0], time.time() - t0), flush=True)
        return op.switching_iteration_fast(rp, ci, part, kk, workers)

    part, hist = op.assign_switching(rowptr, colidx, k, seed, workers=16, iteration=iteration,
                                     objective=op.switching_objective_fast)
    part = np.ascontiguousarray(part, dtype="<i4")
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "mid_switching_digest.txt")
    with open(out, "w") as f:
        f.write("# written by make_switching_digest.py from the oracle's partitioner; config mid\n")
        f.write("n %d\nk %d\nseed %d\nworkers 16\n" % (cfg["n"], k, seed))
        f.write("iterations %d\n" % (len(hist) - 1))
        f.write("sizes %s\n" % " ".join(str(int(x)) for x in np.bincount(part, minlength=k)))
        f.write("sha256 %s\n" % hashlib.sha256(part.tobytes()).hexdigest())
    print("wrote", out)


if __name__ == "__main__":
    main()
