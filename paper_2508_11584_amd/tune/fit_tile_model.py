"""Fits the tile-choice time model of csrc/gemm_bf16.hip to the output of gemm_shapes (read from stdin).

Model per tiling:  t [us] = alpha * max(r, 1) + beta * r * (bm * bn * K / 1e6),  r = ceil(tiles / 256) / held.
Prints alpha, beta per tiling (relative least squares) and, per shape, the model's pick against the measured best.
"""
import re
import sys

import numpy as np

KINDS = [("d256x128", 256, 128, 2), ("d256x256", 256, 256, 1), ("d384x256", 384, 256, 1),
         ("r128x128", 128, 128, 2), ("r64x128", 64, 128, 3), ("r64x64", 64, 64, 4),
         ("d64x64", 64, 64, 4), ("d64x128", 64, 128, 3)]


def cdiv(a, b):
    return -(-a // b)


def rounds(m, n, bm, bn, held):
    return cdiv(cdiv(m, bm) * cdiv(n, bn), 256) / held


def main():
    rows = []
    for line in sys.stdin:
        m = re.search(r"^(.*?)\s+M=\s*(\d+) N=\s*(\d+) K=\s*(\d+) \|(.*)$", line)
        if not m:
            continue
        times = [float(t) for t in re.findall(r"([0-9.]+)us", m.group(5))]
        if len(times) == len(KINDS):
            rows.append((m.group(1).strip(), int(m.group(2)), int(m.group(3)), int(m.group(4)), times))
    if not rows:
        sys.exit("no gemm_shapes lines on stdin")
    fit = {}
    for ki, (name, bm, bn, held) in enumerate(KINDS):
        x = np.array([[max(rounds(M, N, bm, bn, held), 1.0), rounds(M, N, bm, bn, held) * bm * bn * K / 1e6]
                      for _, M, N, K, _ in rows])
        y = np.array([t[ki] for *_, t in rows])
        coef, *_ = np.linalg.lstsq(x / y[:, None], np.ones_like(y), rcond=None)
        fit[name] = coef
        print(f"{name:9s} alpha {coef[0]:6.2f}  beta {coef[1]:7.4f}  max relative error {np.max(np.abs(x @ coef / y - 1)):.2f}")
    tot_pick = tot_best = 0.0
    for shape, M, N, K, times in rows:
        pred = [fit[n][0] * max(rounds(M, N, bm, bn, h), 1.0) + fit[n][1] * rounds(M, N, bm, bn, h) * bm * bn * K / 1e6
                for n, bm, bn, h in KINDS]
        pick, best = int(np.argmin(pred)), int(np.argmin(times))
        tot_pick += times[pick]
        tot_best += times[best]
        print(f"{shape:24s} pick {KINDS[pick][0]:9s} {times[pick]:7.1f} us   best {KINDS[best][0]:9s} {times[best]:7.1f} us   x{times[pick] / times[best]:.3f}")
    print(f"total time of the picks / total of the best: {tot_pick / tot_best:.4f}")


if __name__ == "__main__":
    main()
