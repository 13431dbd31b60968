"""Writes the stored expectations for the full-size parity tests of configs 3 and 5.

Calls ONLY the CPU oracle (oracle/) and the seeded input generators; nothing here touches the
HIP path.  For matrix 0 of the batch it stores the oracle's iteration count, residual and alpha
histories, the Frobenius norm of the result and the result at seeded sample positions.

    python tests/golden/make_full_size_golden.py c3     (about 3 minutes on 8 cores)
    python tests/golden/make_full_size_golden.py c5     (about 15 minutes on 8 cores)
    python tests/golden/make_full_size_golden.py c5 2   (matrix 2 of the batch -> c5_full_matrix2.txt)
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import prism_ref as O                      # noqa: E402
from paper_2601_22137_amd import workloads as W        # noqa: E402

N_SAMPLES = 4096
N_DIAG = 512


def sample_positions(n_rows, n_cols, seed=7):
    """4096 random positions followed by 512 evenly spaced diagonal positions (the square roots of
    SPD matrices are diagonally dominant, so the diagonal is sampled separately)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    r, c = rng.integers(0, n_rows, N_SAMPLES), rng.integers(0, n_cols, N_SAMPLES)
    d = (np.arange(N_DIAG) * (min(n_rows, n_cols) // N_DIAG)).astype(np.int64)
    return np.concatenate([r, d]), np.concatenate([c, d])


def write(path, header, info, outputs):
    with open(path, "w") as f:
        f.write("# " + header + "\n")
        f.write("iters %d\nstatus %d\n" % (info["iters"], info["status"]))
        f.write("residual " + " ".join("%.17g" % r for r in info["residual"]) + "\n")
        f.write("alpha " + " ".join("%.17g" % a for a in info["alpha"]) + "\n")
        for name, X in outputs:
            r, c = sample_positions(*X.shape)
            f.write("%s_fro %.17g\n" % (name, np.linalg.norm(X)))
            f.write("%s_samples " % name + " ".join("%.17g" % v for v in X[r, c]) + "\n")


def main():
    which = sys.argv[1]
    t0 = time.time()
    if which == "c3":
        bits = W.c3_polar_large(batch=1)[0]
        X, info = O.polar(W.from_bf16_bits(bits), 5, 40, 32, W.SKETCH_SEED, 1e-2)
        write(os.path.join(HERE, "c3_full_matrix0.txt"),
              "oracle.polar on workloads.c3_polar_large(batch=1)[0]: degree 5, sketch 32, tol 1e-2, max 40, seed 22137",
              info, [("polar", X)])
    elif which == "c5":
        b = int(sys.argv[2]) if len(sys.argv) > 2 else 0      # matrix b of the batch is drawn with data_seed 1005 + b
        A = W.c5_wishart_spd(batch=1, data_seed=1005 + b)[0]
        S, Si, info = O.sqrt(A, 5, 40, 64, W.SKETCH_SEED, 1e-5)
        write(os.path.join(HERE, "c5_full_matrix%d.txt" % b),
              "oracle.sqrt on workloads.c5_wishart_spd(batch=1%s)[0]: degree 5, sketch 64, tol 1e-5, max 40, seed 22137"
              % ("" if b == 0 else ", data_seed=%d" % (1005 + b)),
              info, [("root", S), ("inv_root", Si)])
    else:
        raise SystemExit("usage: make_full_size_golden.py c3|c5")
    print("done in %.0f s" % (time.time() - t0))


if __name__ == "__main__":
    main()
