"""Writes tests/golden/bf16_rounding_distances.txt: how far bf16 roundings ALONE move the stage's results.

CPU only; calls nothing but the oracle (oracle/stage.py), the seeded input generator (synth/) and the test
helpers that wrap them.  For a configuration (layer shape, depth, micro-batch index) it runs the exact fp64 oracle
once, then the same oracle with a hook that rounds a set of its named intermediate tensors
(oracle.stage.ROUNDING_POINTS) to bf16, and records the relative Frobenius distance of y, dX and of the worst
parameter gradient from the exact run.  Sets:

    one name at a time          the ablation: which tensor's rounding costs how much at depth
    "operands"                  the tensors that are operands of a matrix product; a path that multiplies in bf16
                                has to round these whatever else it does
    "library"                   the tensors the HIP library keeps in bf16 (LIBRARY_BF16 below, maintained by hand
                                from the library's data layout)
    "library_fp32_stream"       the same without the residual stream (h, y forward; dh, dx backward), i.e. what keeping
                                that stream in fp32 would leave.  (dh is also an operand of two products; rounding
                                only that use is not expressible with the hook, so this set is a lower bound.)
    "all"                       every named tensor

The paper prints no numeric value for this computation (it names the architecture only, Sec. 7.1), so these are
measurements of the pinned oracle, not paper values.  The GPU tests read the file for the bounds of their
regression guards; the parity bar itself stays the benchmark spec's tolerance against the exact oracle.

Usage:  python tests/golden/make_bf16_floors.py --config 7b [--layers 4] [--mb 0] [--sets operands,library,all,singles]
Appends to the file (one line per run), so configurations can be added one at a time; a (config, layers, mb, set)
that is already there is skipped unless --redo is given.
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import synth  # noqa: E402
from oracle import stage as O  # noqa: E402
from tests.helpers import grad_errors, rel_err, rounding_hook  # noqa: E402

PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "bf16_rounding_distances.txt")

# operands of the matrix products of one layer, forward and backward
OPERANDS = ("a", "qk", "v", "p", "o", "b", "z", "dgu", "dh", "dc", "p_dv", "ds", "dqk", "dv")
# what the library holds in bf16 between kernels or feeds to its matrix units
LIBRARY_BF16 = OPERANDS + ("h", "y", "gu_kept", "dz", "db", "da", "dx")
SEEDS = (1001, 2001, 3001)      # weights, x, dY: the seeds of the full-size GPU tests and of bench.py


def read(path=PATH):
    """{(config, layers, mb, set): (y, dx, grad, worst gradient)}"""
    out = {}
    if os.path.exists(path):
        for line in open(path):
            if line.startswith("#") or not line.strip():
                continue
            c, k, mb, s, y, dx, g, worst = line.rstrip("\n").split("\t")
            out[(c, int(k), int(mb), s)] = (float(y), float(dx), float(g), worst)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", required=True, choices=sorted(synth.CONFIGS))
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--mb", type=int, default=0, help="index of the micro-batch whose x and dY are used")
    ap.add_argument("--sets", default="operands,library,all")
    ap.add_argument("--redo", action="store_true")
    ap.add_argument("--out", default=PATH, help="file to append to (default: the golden file beside this script)")
    a = ap.parse_args()
    base = synth.CONFIGS[a.config]
    K = a.layers or base.layers
    sh = base.with_(layers=K, microbatches=1)
    sets = []
    for s in a.sets.split(","):
        if s == "singles":
            sets += [(n, (n,)) for n in O.ROUNDING_POINTS]
        elif s == "operands":
            sets.append((s, OPERANDS))
        elif s == "library":
            sets.append((s, LIBRARY_BF16))
        elif s == "all":
            sets.append((s, O.ROUNDING_POINTS))
        elif s == "library_fp32_stream":      # what an fp32 residual stream (forward h, y; backward dh, dx) would leave
            sets.append((s, tuple(n for n in LIBRARY_BF16 if n not in ("h", "y", "dh", "dx"))))
        else:
            sets.append((s, tuple(s.split("+"))))      # e.g. h+y
    out_path = a.out
    have = read(out_path)
    if not a.redo:
        sets = [(n, m) for n, m in sets if (a.config, K, a.mb, n) not in have]
    if not sets:
        print("nothing to do")
        return
    if not os.path.exists(out_path):
        with open(out_path, "w") as f:
            f.write("# bf16 roundings alone: relative Frobenius distance from the exact fp64 oracle (oracle only, CPU);\n"
                    "# written by tests/golden/make_bf16_floors.py; seeds weights/x/dY = %d/%d/%d\n"
                    "# config\tlayers\tmicro-batch\trounded set\ty\tdX\tworst gradient\twhich\n" % SEEDS)
    _, p64 = synth.make_params(sh, SEEDS[0])
    xs, dys = SEEDS[1], SEEDS[2]
    t0 = time.time()
    ey, edx, eg = _run(sh, p64, xs, dys, K, a.mb, None)
    print(f"[{a.config} x{K} mb{a.mb}] exact run {time.time() - t0:.0f} s", flush=True)
    for name, members in sets:
        t0 = time.time()
        y, dx, g = _run(sh, p64, xs, dys, K, a.mb, rounding_hook(members))
        worst, errs = grad_errors(sh, g, eg, K)
        (wl, wn), _ = max(errs.items(), key=lambda kv: kv[1])
        line = "%s\t%d\t%d\t%s\t%.3e\t%.3e\t%.3e\t%s" % (a.config, K, a.mb, name, rel_err(y, ey), rel_err(dx, edx),
                                                        worst, f"{wn}[{wl}]")
        with open(out_path, "a") as f:
            f.write(line + "\n")
        print(line, f"({time.time() - t0:.0f} s)", flush=True)


def _run(sh, p64, xseed, dyseed, K, mb, hook):
    """One micro-batch (index mb of the seeded stream) through K layers and back.  To bound the memory (a layer's
    cache holds its S x S probabilities: 4 to 5 GB at these shapes) only the layer inputs are kept on the way up and
    each layer's forward is run again on the way down; the hook is a pure function, so this changes no value."""
    W = [synth.split_params(sh, p64, l) for l in range(K)]
    _, x = synth.make_x(sh, xseed, mb)
    _, dy = synth.make_dy(sh, dyseed, mb)
    xs = [np.array(x, dtype=np.float64)]
    for l in range(K):
        y, _ = O.layer_forward(xs[l], W[l], sh, hook)
        xs.append(y)
        print(f"  forward layer {l} done", flush=True)
    per = synth.layer_param_elems(sh)
    flat = np.zeros(K * per, dtype=np.float32)     # distances of 1e-3 and more: fp32 storage of the result is ample
    d = np.array(dy, dtype=np.float64)
    for l in range(K - 1, -1, -1):
        _, cache = O.layer_forward(xs[l], W[l], sh, hook)
        d, g = O.layer_backward(d, W[l], cache, sh, hook)
        del cache
        for name, tid, r, c, off in synth.param_layout(sh):
            flat[l * per + off: l * per + off + r * c] = g[name].reshape(-1)
        del g
        print(f"  backward layer {l} done", flush=True)
    return xs[K], d, flat


if __name__ == "__main__":
    main()
