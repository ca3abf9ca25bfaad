#!/usr/bin/env python3
"""Writes tests/golden/oracle_digests.txt from the CPU oracle alone (never from the HIP path)."""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from workloads import configs  # noqa: E402


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:16]


def entries():
    out = []
    for name, w in (("cfg1", configs.config1()), ("cfg2_b1_hw8", configs.config2(batch=1, HW=8)),
                    ("cfg3_b4", configs.config3(batch=4)), ("cfg4_b1_hw6", configs.config4(batch=1, HW=6)),
                    ("cfg5_b1_hw32_w16", configs.config5(batch=1, HW=32, width=16, blocks=(1, 1, 1, 1)))):
        rounded, _ = oracle.run_stack(w.x_exact, w.layers, w.dtype)
        y = rounded[-1]
        out.append("%s output sha=%s sum=%.10e abssum=%.10e" % (name, digest(y), y.sum(), np.abs(y).sum()))
        for i, L in enumerate(w.layers):
            if L.kind not in ("conv", "fc"):
                continue
            Bf = 1 if L.scheme == "pattern" else min(L.Bf, L.F)
            grp, kpos, wc = oracle.pack_block_punched(L.w_exact, L.mask, Bf)
            out.append("%s layer%d meta grp=%s kpos=%s w=%s K=%d" % (name, i, digest(grp), digest(kpos), digest(wc), len(kpos)))
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_digests.txt")
    with open(path, "w") as f:
        f.write("\n".join(entries()) + "\n")
    print("wrote", path)
