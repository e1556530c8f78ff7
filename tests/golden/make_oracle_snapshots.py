"""Writes tests/golden/oracle_snapshots.txt: small worked examples computed by the CPU oracle and by nothing else.

The paper prints no numbers for its random choices (App. B.4.1 only says that indices and signs are sampled), so these
values are not the paper's: they freeze the readings this repository takes (hash streams, Random-Mask order, SJLT
block construction and sign rule, Kronecker order of Eq. (3), Box-Muller bits of the Gaussian baseline) so that a later
change to any of them shows up as a changed fixture, and they give the GPU library a stored target that no GPU code
produced.  Inputs are small integers, so every sum is exact in binary floating point and is written exactly.

Run from the repository root:  python tests/golden/make_oracle_snapshots.py
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", ".."))
from oracle import grass_oracle as orc  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_snapshots.txt")


def small_ints(rows, cols, mod, shift):
    """Deterministic small integers (no generator involved): ((7 i + 3 j + i j) mod `mod`) - shift, zero where the
    value is odd and j is a multiple of 3 (some exact zeros, as in ReLU gradients)."""
    i = np.arange(rows)[:, None]
    j = np.arange(cols)[None, :]
    v = (7 * i + 3 * j + i * j) % mod - shift
    return np.where((v % 2 != 0) & (j % 3 == 0), 0, v).astype(np.float64)


def cases():
    out = []
    # Sec. 3.2, Random Mask: k' smallest hash keys, ascending
    for (seed, stream, p, kp) in [(0, 0, 1000, 12), (7, 16, 4096, 8), (3, 17, 50, 50)]:
        out.append((f"mask_indices seed={seed} stream={stream} p={p} kprime={kp}",
                    orc.mask_indices(seed, stream, p, kp).astype(np.int64)))
    # Sec. 3.1, SJLT tables: bucket and sign of every (position, r)
    for (seed, stream, d, k, s) in [(0, 1, 12, 8, 1), (5, 18, 6, 12, 3)]:
        b, g = orc.sjlt_tables(seed, stream, d, k, s)
        out.append((f"sjlt_bucket seed={seed} stream={stream} d={d} k={k} s={s}", b.astype(np.int64).reshape(-1)))
        out.append((f"sjlt_sign seed={seed} stream={stream} d={d} k={k} s={s}", g.astype(np.int64).reshape(-1)))
    # Sec. 3.1, SJLT of small integer rows (s = 1 and s = 4: the scale 1/2 is exact)
    g = small_ints(3, 40, 9, 4)
    out.append(("sjlt seed=0 stream=1 n=3 d=40 k=8 s=1", orc.sjlt(g, 8, 1, 0, 1).reshape(-1)))
    out.append(("sjlt seed=2 stream=1 n=3 d=40 k=16 s=4", orc.sjlt(g, 16, 4, 2, 1).reshape(-1)))
    # Sec. 3.3.1, GraSS = SJLT o Mask
    idx = orc.mask_indices(1, 0, 40, 10)
    out.append(("grass seed=1 n=3 p=40 kprime=10 k=4 s=1 (mask seed 1 stream 0, sjlt stream 1)",
                orc.grass(g, idx, 4, 1, 1, 1).reshape(-1)))
    # Sec. 3.3.2 / Eq. (3), FactGraSS on one tiny layer (layer 0: streams 16, 17, 18)
    x = small_ints(2 * 3, 10, 5, 2).reshape(2, 3, 10)
    go = small_ints(2 * 3, 6, 7, 3).reshape(2, 3, 6)
    s_in, s_out, s_sj = orc.layer_streams(0)
    ii = orc.mask_indices(4, s_in, 10, 4)
    io = orc.mask_indices(4, s_out, 6, 3)
    out.append(("factgrass seed=4 layer=0 n=2 T=3 d_in=10 d_out=6 kin=4 kout=3 k=6 s=1",
                orc.factgrass_linear(x, go, ii, io, 6, 1, 4, s_sj).reshape(-1)))
    # Sec. 2.2, Gaussian baseline: the uniforms are exact, the normals are written to 12 significant digits
    out.append(("gauss_matrix seed=0 stream=1 p=5 k=4 (row-major 4 x 5, 12 significant digits)",
                orc.gauss_matrix(0, 1, 5, 4).reshape(-1)))
    return out


def fmt(v):
    if v.dtype.kind in "iu":
        return " ".join(str(int(x)) for x in v)
    return " ".join(repr(float(x)) if float(x) == round(float(x) * 4) / 4 else f"{float(x):.12g}" for x in v)


def main():
    lines = ["# Worked examples computed by oracle/grass_oracle.py (script: tests/golden/make_oracle_snapshots.py).",
             "# Not the paper's numbers (it prints none for its random choices): they freeze this repository's readings.",
             "# format: one '@ name' line, then one line of values"]
    for name, v in cases():
        lines.append("@ " + name)
        lines.append(fmt(np.asarray(v)))
    with open(OUT, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", OUT, len(lines), "lines")


if __name__ == "__main__":
    main()
