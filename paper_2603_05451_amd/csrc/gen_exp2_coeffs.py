#!/usr/bin/env python3
"""Prints the fp32 polynomial coefficients used by exp2_emulation.h.

2^f on [0, 1) is approximated by 1 + p1 f + ... + pn f^n with the maximum RELATIVE error
minimised and p0 fixed to 1 (paper Sec. 3.1.3 states the criterion; it prints no coefficients).
Method: Remez exchange on the weighted error e(f) = (1 + sum p_i f^i) / 2^f - 1 with n + 1
alternation points.  Run: python3 gen_exp2_coeffs.py
"""
import numpy as np


def remez(n, iters=40):
    k = np.arange(n + 1)
    pts = 0.5 - 0.5 * np.cos(np.pi * (k + 0.5) / (n + 1))            # initial reference in (0, 1)
    grid = np.linspace(0.0, 1.0, 200001)
    for _ in range(iters):
        w = 2.0 ** pts
        # sum_i p_i x^i - (-1)^k E 2^x = 2^x - 1
        A = np.hstack([np.stack([pts ** i for i in range(1, n + 1)], 1), (-(-1.0) ** k * w)[:, None]])
        sol = np.linalg.solve(A, w - 1.0)
        p, E = sol[:n], sol[n]
        err = (1.0 + sum(p[i - 1] * grid ** i for i in range(1, n + 1))) / 2.0 ** grid - 1.0
        # new reference: the extremum of each sign-constant segment of the error
        sign_change = np.where(np.diff(np.sign(err)) != 0)[0]
        bounds = np.concatenate([[0], sign_change + 1, [len(grid)]])
        new = [lo + np.argmax(np.abs(err[lo:hi])) for lo, hi in zip(bounds[:-1], bounds[1:]) if hi > lo]
        while len(new) > n + 1:          # too many alternations: drop the weaker end point
            new = new[1:] if abs(err[new[0]]) < abs(err[new[-1]]) else new[:-1]
        if len(new) < n + 1:
            break
        new_pts = grid[new]
        if np.max(np.abs(new_pts - pts)) < 1e-7:
            pts = new_pts
            break
        pts = new_pts
    return p, abs(E)


if __name__ == "__main__":
    for n in (3, 4, 5):
        p, E = remez(n)
        lits = ", ".join(f"{np.float32(v):.9e}f" for v in p)
        print(f"degree {n}: max rel err {E:.3e}: {{{lits}}}")
