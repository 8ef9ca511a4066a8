"""Writes tests/golden/worked_example_d8.json.  Calls neither the oracle nor the GPU library.

The paper prints no numerical example, so this is a hand-derived one.  The inputs
are chosen so that every corrected gradient x = e + g, residual e, block scale mu,
averaged gradient gbar, index set and sign bit is a short binary fraction: those
entries are written below as literals, derived with pencil from Definition 1,
Definition 2 and the worker/server lines of Algorithm 2 (ties: larger |x| first,
then the lower index; sign(0) = +1).  The moments and theta are the server lines
of Algorithm 2 evaluated on the exact gbar in 50-digit decimal arithmetic, for both
placements of epsilon, with the hyper-parameters taken as the fp32 numbers nearest
to 0.9, 0.999, 1e-8 and 1e-3 (what an fp32 implementation is actually handed), and
rounded to 10 significant digits.  An fp32 implementation must reproduce the
literal parts exactly and the computed parts to about 1e-6 relative.
"""
import json
import os
import struct
from decimal import Decimal as D, getcontext

getcontext().prec = 50


def f32(x):
    return D(struct.unpack("f", struct.pack("f", x))[0])


B1, B2, EPS, LR = f32(0.9), f32(0.999), f32(1e-8), f32(1e-3)

G = [[[4, -2, 2, 0.5, -1, 0, 0.25, 1], [-1, 3, 0.5, 0, -3, 1, 2, -0.5]],
     [[1, 1, 0, -0.5, -1, 3, -0.25, 1], [1, -2, -0.5, 0, 2, 1, 0, 0.5]]]

TOPK = {
    "k": 2,
    # step 1: worker 0 |x| = 4,2,2,.5,1,0,.25,1 -> {0, then the tie |2| at 1,2 goes to 1}; worker 1: |3| at 1 and 4
    # step 2: x0 = 1,1,2,0,-2,3,0,2 -> {5, tie |2| at 2,4,7 -> 2}; x1 = 0,-2,0,0,2,2,2,0 -> tie |2| at 1,4,5,6 -> {1,4}
    "idx": [[[0, 1], [1, 4]], [[2, 5], [1, 4]]],
    "e": [[[0, 0, 2, 0.5, -1, 0, 0.25, 1], [-1, 0, 0.5, 0, 0, 1, 2, -0.5]],
          [[1, 1, 0, 0, -2, 0, 0, 2], [0, 0, 0, 0, 0, 2, 2, 0]]],
    "gbar": [[2, 0.5, 0, 0, -1.5, 0, 0, 0], [0, -1, 1, 0, 1, 1.5, 0, 0]],
}

BLOCKSIGN = {
    "block_offsets": [0, 4, 8],
    "mu": [[[2.125, 0.5625], [1.125, 1.625]], [[1.5625, 1.46875], [0.875, 0.75]]],
    "neg": [[[0, 1, 0, 0, 1, 0, 0, 0], [1, 0, 0, 0, 1, 0, 0, 1]], [[0, 0, 1, 1, 1, 0, 1, 0], [0, 1, 1, 1, 0, 0, 0, 0]]],
    "e": [[[1.875, 0.125, -0.125, -1.625, -0.4375, -0.5625, -0.3125, 0.4375],
           [0.125, 1.875, -0.625, -1.125, -1.375, -0.625, 0.375, 1.125]],
          [[1.3125, -0.4375, 1.4375, -0.5625, 0.03125, 0.96875, 0.90625, -0.03125],
           [0.25, 0.75, -0.25, -0.25, -0.125, -0.375, -0.375, 0.875]]],
    "gbar": [[0.5, -0.5, 1.625, 1.625, -1.09375, 1.09375, 1.09375, -0.53125],
             [1.21875, 0.34375, -1.21875, -1.21875, -0.359375, 1.109375, -0.359375, 1.109375]],
}


def server(gbars, eps_in):
    d = len(gbars[0])
    m = [D(0)] * d; v = [D(0)] * d; vh = [D(0)] * d; th = [D(0)] * d
    out = {"m": [], "v": [], "vhat": [], "theta": []}
    for gb in gbars:
        for j in range(d):
            g = D(str(gb[j]))
            m[j] = B1 * m[j] + (1 - B1) * g
            v[j] = B2 * v[j] + (1 - B2) * g * g
            vh[j] = max(vh[j], v[j])
            den = (vh[j] + EPS).sqrt() if eps_in else vh[j].sqrt() + EPS
            th[j] = th[j] - LR * m[j] / den
        for name, a in (("m", m), ("v", v), ("vhat", vh), ("theta", th)):
            out[name].append([float("%.9e" % t) for t in a])
    return out


def main():
    doc = {"_provenance": __doc__.strip(), "n": 2, "d": 8, "lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8,
           "theta1": [0] * 8, "g": G}
    for name, part in (("topk", TOPK), ("blocksign", BLOCKSIGN)):
        part = dict(part)
        s_in, s_out = server(part["gbar"], True), server(part["gbar"], False)
        part.update(m=s_in["m"], v=s_in["v"], vhat=s_in["vhat"],
                    theta_eps_in=s_in["theta"], theta_eps_out=s_out["theta"])
        doc[name] = part
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "worked_example_d8.json")
    with open(path, "w") as f:
        json.dump(doc, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
