#!/usr/bin/env python3
"""Signal swamping on synthetic data (Sec. 3.2.1, the example with uniform signals).

A tensor of 1000 unsigned EMA states, quantized tensor-wise (one block); initial states and
every received signal are drawn from U[0, 1].  The exact EMA converges to 0.5 on every element;
a quantized EMA whose levels are wider apart than the signal's contribution (1 - beta) z never
leaves its initial codes.  Prints, per quantizer and code width: the fraction of codes that are
still the initial ones, the spread of the final states, and the RMS distance to the exact EMA.

This is test infrastructure like the rest of oracle/: it runs the CPU oracle only.
"""
import argparse
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from oracle import solo_oracle as so  # noqa: E402

KINDS = ((so.U_LINEAR, "linear"), (so.U_LINEAR_NOZERO, "linear, no zero"), (so.U_DE, "dynamic exponent"),
         (so.U_LOG, "logarithmic + SR (SOLO)"))


def run(n, steps, beta, bits, kind, seed=0, block=None):
    rng = np.random.default_rng(seed)
    x0 = rng.random(n).astype(np.float32)
    ema = so.UnsignedEma(x0, block or n, bits, kind)
    first = ema.codes.copy()
    exact = x0.astype(np.float64)
    for _ in range(steps):
        z = rng.random(n).astype(np.float32)
        ema.step(z, beta)
        exact = beta * exact + (1 - beta) * z
    v = ema.values().astype(np.float64)
    return {"unchanged": float(np.mean(ema.codes == first)), "std": float(v.std()),
            "rms": float(np.sqrt(np.mean((v - exact) ** 2))), "exact_std": float(exact.std())}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=1000)
    ap.add_argument("--block", type=int, default=None, help="block size (default: the whole tensor)")
    ap.add_argument("--betas", type=float, nargs="+", default=[0.9, 0.99, 0.999])
    args = ap.parse_args()
    for beta in args.betas:
        steps = int(round(3.0 / (1.0 - beta)))          # three time constants of the EMA
        print(f"beta = {beta}, {steps} steps")
        for bits in (2, 3, 4, 8):
            for kind, name in KINDS:
                r = run(args.n, steps, beta, bits, kind, block=args.block)
                print(f"  {bits}-bit {name:26s} codes unchanged {100 * r['unchanged']:5.1f} %   "
                      f"std of states {r['std']:.3f} (exact {r['exact_std']:.3f})   rms to exact {r['rms']:.3f}")


if __name__ == "__main__":
    main()
