#!/usr/bin/env python3
"""Writes tests/golden/oracle_small_cases.json: outputs of the CPU oracle on small seeded inputs.

The paper prints no worked numeric example of this path (its tables report accuracies and run times that need datasets
and trained weights), so there is no paper fixture; this file freezes what the pinned oracle computes, so that an
unintended change of its arithmetic shows up as a diff here.  It calls nothing but `oracle/` and the seeded input
generators.  Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.abspath(os.path.join(os.path.dirname(__file__), "..", ".."))
sys.path.insert(0, ROOT)

import oracle as orc  # noqa: E402
from paper_2203_04071_amd import workloads as wl  # noqa: E402


def cases():
    rng = np.random.default_rng(20220304)
    out = {}
    lut4 = wl.make_lut(4)
    A = wl.random_i8(rng, (3, 7), 4)
    W = wl.random_i8(rng, (2, 7), 4)
    out["linear_4bit"] = dict(A=A.tolist(), W=W.tolist(), acc=orc.approx_linear(lut4, 4, A, W).tolist())
    x = wl.random_i8(rng, (1, 2, 4, 4), 4)
    w = wl.random_i8(rng, (2, 2, 3, 3), 4)
    out["conv2d_4bit_pad1"] = dict(x=x.tolist(), w=w.tolist(), acc=orc.approx_conv2d(lut4, 4, x, w, pad=(1, 1)).tolist())
    wt = wl.random_i8(rng, (2, 2, 4, 4), 4)
    out["conv_transpose2d_4bit_s2_p1"] = dict(x=x.tolist(), w=wt.tolist(),
                                              acc=orc.approx_conv_transpose2d(lut4, 4, x, wt, 2, 1).tolist())
    v = (rng.standard_normal(12) * 2).astype(np.float32)
    out["quantize_8bit"] = dict(x=[float(t) for t in v], scale=0.03125, q=orc.quantize(v, 0.03125, 8).tolist())
    a1 = rng.integers(-5000, 5000, (2, 8)).astype(np.int32)
    a2 = rng.integers(-5000, 5000, (2, 8)).astype(np.int32)
    c = rng.standard_normal((2, 2)).astype(np.float32)
    h, c2 = orc.lstm_cell(a1, a2, 1e-3, 2e-3, None, c)
    out["lstm_cell"] = dict(acc_ih=a1.tolist(), acc_hh=a2.tolist(), c=[[float(t) for t in r] for r in c],
                            h_bits=h.view(np.uint32).tolist(), c_bits=c2.view(np.uint32).tolist())
    g1, g2 = a1[:, :6].copy(), a2[:, :6].copy()
    hp = rng.uniform(-1, 1, (2, 2)).astype(np.float32)
    out["gru_cell"] = dict(acc_ih=g1.tolist(), acc_hh=g2.tolist(), h=[[float(t) for t in r] for r in hp],
                           h_bits=orc.gru_cell(g1, g2, 1e-3, 2e-3, None, None, hp).view(np.uint32).tolist())
    out["mitchell_6bit_row_of_21"] = [orc.mul_func(orc.FUNC_MITCHELL, 0, 21, w_) for w_ in range(-32, 32)]
    cnt = orc.histogram_abs(v, float(np.abs(v).max()), 8)
    out["histogram_8_bins"] = dict(counts=cnt.tolist(),
                                   p75=float(orc.percentile_from_histogram(cnt, float(np.abs(v).max()), 3, 4)))
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(__file__), "oracle_small_cases.json")
    with open(path, "w") as f:
        json.dump(cases(), f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", path)
