"""Writes tests/golden/gauss_recipe_digests.txt: SHA-256 digests of the oracle's Box-Muller
building blocks over their whole 24-bit input domains.  Calls only oracle/.  The GPU parity
test hashes the device's output over the same domain and compares, which makes the bit-exact
check exhaustive without running the slow oracle inside the test.

    python tests/golden/make_gauss_digests.py
"""
import hashlib
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import gauss  # noqa: E402

SUBSET_STRIDE = 37


def digest(arr):
    return hashlib.sha256(np.ascontiguousarray(arr).view(np.uint32).tobytes()).hexdigest()


def main():
    lines = [
        "# SHA-256 of the binary32 bit patterns (little-endian uint32, index order) produced by the",
        "# oracle's Gaussian recipe: radius_from_word(n << 8) and cos_sin_from_word(n << 8) for",
        "# n = 0 .. 2^24-1 ('full'), and for n = 0, stride, 2*stride, ... ('subset').",
        "# Written by tests/golden/make_gauss_digests.py, which calls only oracle/.",
        "# The recipe implements Algorithm 1's 'P_t <- N_seed(0, 1/r)' draw.",
        "subset_stride: %d" % SUBSET_STRIDE,
    ]
    out = {}
    chunks_r, chunks_c, chunks_s = [], [], []
    step = 1 << 20
    for lo in range(0, 1 << 24, step):
        n = np.arange(lo, lo + step, dtype=np.uint32) << np.uint32(8)
        chunks_r.append(gauss.radius_from_word(n))
        c, s = gauss.cos_sin_from_word(n)
        chunks_c.append(c)
        chunks_s.append(s)
        print("done", lo + step, flush=True)
    full = {"radius": np.concatenate(chunks_r), "cos": np.concatenate(chunks_c),
            "sin": np.concatenate(chunks_s)}
    for name, arr in full.items():
        out["full_%s_sha256" % name] = digest(arr)
        out["subset_%s_sha256" % name] = digest(arr[::SUBSET_STRIDE])
    for k in sorted(out):
        lines.append("%s: %s" % (k, out[k]))
    with open(os.path.join(HERE, "gauss_recipe_digests.txt"), "w") as fh:
        fh.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
