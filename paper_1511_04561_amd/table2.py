"""Approximation errors of the four 8-bit data types on synthetic samples (Sec. 3.4, Table 2 of
arXiv 1511.04561): 25 million draws from U(0,1), N(0,1), N(0,10^2) and N(0,0.2^2); the dynamic tree and
the linear type are normalised by the sample's absolute maximum, the two static-exponent types use a
decade as scale (10^2 for N(0,10^2), 10^1 otherwise).

    python -m paper_1511_04561_amd.table2 [--samples N] [--seed S]

Samples are drawn on the device with torch's generator; the statistics come from dq8_error_stats.
Prints one line per (distribution, data type): mean absolute error, mean relative error in percent
(over the non-zero samples) and the largest absolute error.
"""
import argparse

import torch

from . import dq8

TYPES = [(dq8.DYNAMIC_TREE, "8-bit dynamic tree", False), (dq8.LINEAR, "8-bit linear quant", False),
         (dq8.MANTISSA, "8-bit mantissa", True), (dq8.STATIC_TREE, "8-bit static tree", True)]
DISTRIBUTIONS = [("U(0,1)", None, 1.0, 1), ("N(0,1)", 0.0, 1.0, 1), ("N(0,10^2)", 0.0, 10.0, 2), ("N(0,0.2^2)", 0.0, 0.2, 1)]


def rows(samples=25_000_000, seed=1511):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    out = []
    for name, mean, std, decade in DISTRIBUTIONS:
        x = torch.empty(samples, dtype=torch.float32, device="cuda")
        if mean is None:
            x.uniform_(0.0, 1.0, generator=gen)
        else:
            x.normal_(mean, std, generator=gen)
        for kind, label, static in TYPES:
            if static:
                scale = torch.full((1,), 10.0 ** decade, dtype=torch.float32, device="cuda")
                stats, means = dq8.error_stats(kind, x, 0, scales=scale, scales_given=True)
            else:
                stats, means = dq8.error_stats(kind, x, 0)
            m, s = means.cpu().tolist(), stats.cpu().tolist()[0]
            out.append((name, label, m[0], 100.0 * m[1], s[3]))
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--samples", type=int, default=25_000_000)
    ap.add_argument("--seed", type=int, default=1511)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("needs a GPU")
    dq8.init()
    print("%-12s %-20s %14s %12s %14s" % ("distribution", "data type", "mean abs err", "mean rel %", "max abs err"))
    for name, label, mae, mre, worst in rows(args.samples, args.seed):
        print("%-12s %-20s %14.6g %12.3f %14.6g" % (name, label, mae, mre, worst))


if __name__ == "__main__":
    main()
