"""Case study of Section 6.1 on the GPU library: nonconvex logistic regression (eq. (7), lambda = 0.1,
n = 20 workers, full-batch local gradients) with the four strategies the paper compares - no
compression, CD-Adam (Algorithm 1), error feedback, naive compression - and prints the norm of the
full gradient against the iteration, the quantity the paper plots.

The LibSVM sets of the paper are not available here; workloads.logreg_problem makes data of their shape
(a few hundred binary features, +-1 labels from a noisy linear rule).  Settings: block-wise scaled
sign with 16 coordinates per block, nu = 1e-3 inside the root (Algorithm 1), alpha = 0.003.  On such
data the ordering uncompressed < CD-Adam < error feedback < naive shows with these settings; it is
not universal (with nu = 1e-8, or the whole-vector sign, CD-Adam ends behind error feedback).

    python -m paper_2111_00705_amd.examples.logreg_case_study [--iterations 1500] [--block 16]
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--iterations", type=int, default=1500)
    ap.add_argument("--block", type=int, default=16)
    ap.add_argument("--nu", type=float, default=1e-3)
    ap.add_argument("--alpha", type=float, default=0.003)
    ap.add_argument("--every", type=int, default=100)
    args = ap.parse_args()

    import torch

    import paper_2111_00705_amd as P
    import workloads as W

    assert torch.cuda.is_available(), "this example needs a GPU"
    a, y = W.logreg_problem()
    n, _, d = a.shape
    arms = (("uncompressed", P.METHOD_NONE), ("CD-Adam", P.METHOD_CD), ("error feedback", P.METHOD_EF),
            ("naive", P.METHOD_NAIVE))
    curves = {}
    for name, method in arms:
        h = P.CompAms(d, n, P.BLOCKSIGN, args.block, 0.9, 0.999, args.nu, args.alpha)
        h.set_method(method)
        h.set_eps_mode(1)
        theta = np.zeros(d, np.float32)
        rows = []
        for t in range(args.iterations + 1):
            g = W.logreg_grads(a, y, theta)
            if t % args.every == 0:
                rows.append((t, float(np.linalg.norm(g.astype(np.float64).mean(axis=0)))))
            if t == args.iterations:
                break
            h.step(torch.from_numpy(g).cuda())
            theta = h.get_theta()
        up, down = h.message_bits()
        curves[name] = (rows, up, down)
        h.destroy()
    print(f"nonconvex logistic regression, n = {n}, d = {d}; norm of the full gradient")
    print("iteration " + " ".join(f"{name:>15s}" for name, _ in arms))
    for q in range(len(curves[arms[0][0]][0])):
        print(f"{curves[arms[0][0]][0][q][0]:9d} " + " ".join(f"{curves[name][0][q][1]:15.3e}" for name, _ in arms))
    print("bits per step and worker (up + down): " +
          ", ".join(f"{name} {curves[name][1] + curves[name][2]}" for name, _ in arms))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
