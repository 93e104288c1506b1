#!/usr/bin/env python3
"""Writes tests/golden/codec_golden.json: a frozen record of what the CPU oracle computes for a
few tiny encode/decode cases (inputs and results as exact bit patterns).  It calls only oracle/.
Purpose: the oracle cannot drift unnoticed, and the HIP library is checked against the same record.
Run from the repository root:  python tests/golden/make_codec_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import tng_oracle as O  # noqa: E402


def bits(a):
    return [int(x) for x in np.asarray(a, dtype=np.float32).view(np.uint32).reshape(-1)]


def main():
    rng = np.random.default_rng(20190123)
    cases = []
    for d, M in [(20, 2), (37, 3)]:
        gref = rng.standard_normal(d).astype(np.float32)
        gref[3] = 0.0
        gref2 = (rng.standard_normal(d) + 2.5).astype(np.float32)
        g = (gref + 0.25 * rng.standard_normal((M, d))).astype(np.float32)
        g[M - 1, 5] = gref[5]
        for bits_ in (2, 4):
            for norm in (O.NORM_NONE, O.NORM_SUB, O.NORM_QUOT, O.NORM_COMB):
                cfg = O.Config(d=d, M=M, bits=bits_, norm=norm, seed=0x1901_08227, lr=0.05)
                it = 7
                codes, scales = O.normalize_encode(cfg, it, g, gref, gref2)
                vbar = O.decode_aggregate(cfg, codes, scales, gref, d, gref2)
                w = np.linspace(-1, 1, d).astype(np.float32)
                cases.append({
                    "d": d, "M": M, "bits": bits_, "norm": norm, "seed": cfg.seed, "iter": it, "lr": cfg.lr,
                    "g": bits(g), "gref": bits(gref), "gref2": bits(gref2), "w": bits(w),
                    "codes": [int(x) for x in codes.reshape(-1)], "scales": bits(scales), "vbar": bits(vbar),
                    "w_next": bits(O.update_iterate(w, vbar, cfg.lr)),
                })
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "codec_golden.json")
    with open(out, "w") as fh:
        json.dump({"note": "written by tests/golden/make_codec_golden.py from oracle/ only; float arrays are IEEE "
                           "binary32 bit patterns", "cases": cases}, fh)
    print(f"wrote {out}: {len(cases)} cases")


if __name__ == "__main__":
    main()
