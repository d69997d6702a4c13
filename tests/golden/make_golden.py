"""Writes tests/golden/tiny_stage_fp64.txt: a few values of the ORACLE's output on the tiny seeded stage.

Calls only oracle/ and the input generator.  The paper prints no worked numeric example of the decoder layer
(it names the architecture only, Sec. 7.1), so these are regression values of the pinned oracle, not paper values;
they guard against an unnoticed change of the oracle or of the generator."""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import synth  # noqa: E402
from oracle import stage as O  # noqa: E402


def values():
    sh = synth.CONFIGS["tiny"]
    _, p64 = synth.make_params(sh, 1000)
    W = [synth.split_params(sh, p64, l) for l in range(sh.layers)]
    _, x = synth.make_x(sh, 2000, 0)
    _, dy = synth.make_dy(sh, 3000, 0)
    y, caches = O.stage_forward(x, W, sh)
    dx, g = O.stage_backward(dy, W, caches, sh)
    out = {"x[0,0,0]": x[0, 0, 0], "w_qkv[0][3,5]": W[0]["w_qkv"][3, 5], "norm(y)": np.linalg.norm(y),
           "y[1,127,255]": y[1, 127, 255], "y[0,5,17]": y[0, 5, 17], "norm(dx)": np.linalg.norm(dx),
           "dx[1,0,3]": dx[1, 0, 3], "norm(g0.w_qkv)": np.linalg.norm(g[0]["w_qkv"]),
           "g1.w_d[100,200]": g[1]["w_d"][100, 200], "g0.gamma1[7]": g[0]["gamma1"][7],
           "norm(g1.w_gu)": np.linalg.norm(g[1]["w_gu"]), "g1.gamma2[255]": g[1]["gamma2"][255]}
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_stage_fp64.txt")
    with open(path, "w") as f:
        f.write("# oracle regression values, tiny stage (2 layers, 1 micro-batch), seeds 1000/2000/3000; written by make_golden.py\n")
        for k, v in values().items():
            f.write(f"{k}\t{float(v)!r}\n")
    print("wrote", path)
