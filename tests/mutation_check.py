"""Mutation check of the oracle pins (CPU only, run by hand: `python tests/mutation_check.py`, about five minutes).

Plants one plausible mistake at a time (a dropped term, a wrong sign, index or operand, a transposed product) in a
COPY of oracle/*.py, runs the non-GPU tests against that copy and lists every mutant the pins fail to catch.  The
repository itself is never modified: the copy lives in a temporary directory next to links to everything else."""
import os
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
M = [
 ("stage.py", "axis=-1, keepdims=True) + eps)", "axis=-1, keepdims=True) - eps)"),
 ("stage.py", "r = 1.0 / np.sqrt(np.mean(x * x", "r = 1.0 / np.sqrt(np.sum(x * x"),
 ("stage.py", "return x * r * gamma, r", "return x * r, r"),
 ("stage.py", "dx = r * (dn - n * np.mean", "dx = r * (dn + n * np.mean"),
 ("stage.py", "dx = r * (dn - n * np.mean(dn * n", "dx = r * (dn - n * np.mean(da * n"),
 ("stage.py", "return dx, np.sum(da * n, axis=0)", "return dx, np.sum(dn * n, axis=0)"),
 ("stage.py", "return dx, np.sum(da * n, axis=0)", "return dx, np.sum(da * x, axis=0)"),
 ("stage.py", "theta = base ** (-2.0 * i / head_dim)", "theta = base ** (2.0 * i / head_dim)"),
 ("stage.py", "theta = base ** (-2.0 * i / head_dim)", "theta = base ** (-1.0 * i / head_dim)"),
 ("stage.py", "theta = base ** (-2.0 * i / head_dim)", "theta = base ** (-2.0 * (i + 1) / head_dim)"),
 ("stage.py", "return np.concatenate([u1 * c - u2 * s, u1 * s + u2 * c], axis=-1)", "return np.concatenate([u1 * c + u2 * s, u1 * s - u2 * c], axis=-1)"),
 ("stage.py", "return np.concatenate([u1 * c - u2 * s, u1 * s + u2 * c], axis=-1)", "return np.concatenate([u1 * c + u2 * s, -u1 * s + u2 * c], axis=-1)"),
 ("stage.py", "u1, u2 = u[..., :d2], u[..., d2:]", "u1, u2 = u[..., 0::2], u[..., 1::2]"),
 ("stage.py", "k[bi, :, hk, :].T / np.sqrt(d)\n", "k[bi, :, hk, :].T / d\n"),
 ("stage.py", "            hk = hq // g\n            s = q", "            hk = hq % k.shape[2]\n            s = q"),
 ("stage.py", "mask = np.tril(np.ones((S, S), dtype=bool))", "mask = np.tril(np.ones((S, S), dtype=bool), -1) | np.eye(S, dtype=bool)[0:1].T.repeat(S, 1)"),
 ("stage.py", "mask = np.tril(np.ones((S, S), dtype=bool))", "mask = np.ones((S, S), dtype=bool)"),
 ("stage.py", "o[bi, :, hq, :] = st(\"p\", pr) @ v[bi, :, hk, :]", "o[bi, :, hq, :] = st(\"p\", pr) @ k[bi, :, hk, :]"),
 ("stage.py", "dv[bi, :, hk, :] += st(\"p_dv\", pr).T @ dO", "dv[bi, :, hk, :] = st(\"p_dv\", pr).T @ dO"),
 ("stage.py", "dv[bi, :, hk, :] += st(\"p_dv\", pr).T @ dO", "dv[bi, :, hk, :] += st(\"p_dv\", pr) @ dO"),
 ("stage.py", "ds = st(\"ds\", pr * (dp - np.sum(pr * dp", "ds = st(\"ds\", pr * (dp + np.sum(pr * dp"),
 ("stage.py", "ds = st(\"ds\", pr * (dp - np.sum(pr * dp, axis=1, keepdims=True)))", "ds = st(\"ds\", pr * dp)"),
 ("stage.py", "dq[bi, :, hq, :] = ds @ k[bi, :, hk, :] / np.sqrt(d)", "dq[bi, :, hq, :] = ds @ k[bi, :, hk, :]"),
 ("stage.py", "dk[bi, :, hk, :] += ds.T @ q[bi, :, hq, :] / np.sqrt(d)", "dk[bi, :, hk, :] = ds.T @ q[bi, :, hq, :] / np.sqrt(d)"),
 ("stage.py", "dk[bi, :, hk, :] += ds.T @ q[bi, :, hq, :] / np.sqrt(d)", "dk[bi, :, hk, :] += ds @ q[bi, :, hq, :] / np.sqrt(d)"),
 ("stage.py", "    return g * sigmoid(g) * u\n", "    return sigmoid(g) * u\n"),
 ("stage.py", "    return g * sigmoid(g) * u\n", "    return u * sigmoid(u) * g\n"),
 ("stage.py", "return dz * u * s * (1.0 + g * (1.0 - s)), dz * g * s", "return dz * u * s * (1.0 + g * (1.0 + s)), dz * g * s"),
 ("stage.py", "return dz * u * s * (1.0 + g * (1.0 - s)), dz * g * s", "return dz * u * s * (1.0 + g * (1.0 - s)), dz * s"),
 ("stage.py", "return dz * u * s * (1.0 + g * (1.0 - s)), dz * g * s", "return dz * u * s * (1.0 - g * (1.0 - s)), dz * g * s"),
 ("stage.py", 'H = st("h", X + C @ w["w_o"])', 'H = st("h", C @ w["w_o"])'),
 ("stage.py", 'Y = st("y", H + Z @ w["w_d"])', 'Y = st("y", X + Z @ w["w_d"])'),
 ("stage.py", "swiglu_fwd(GU[:, :f], GU[:, f:])", "swiglu_fwd(GU[:, f:], GU[:, :f])"),
 ("stage.py", "G=GUk[:, :f], U=GUk[:, f:]", "U=GUk[:, :f], G=GUk[:, f:]"),
 ("stage.py", "q, k = qk[:, :, :nq, :], qk[:, :, nq:, :]", "q, k = qk[:, :, :nq, :], QKV[:, qd:qd + kvd].reshape(b, S, nkv, d)"),
 ("stage.py", 'B, r2 = rmsnorm_fwd(H, w["gamma2"], sh.rms_eps)', 'B, r2 = rmsnorm_fwd(H, w["gamma1"], sh.rms_eps)'),
 ("stage.py", 'dH = st("dh", dY + dHn)', 'dH = st("dh", dHn)'),
 ("stage.py", 'dX = st("dx", dH + dXn)', 'dX = st("dx", dXn)'),
 ("stage.py", 'dX = st("dx", dH + dXn)', 'dX = st("dx", dY + dXn)'),
 ("stage.py", 'g["w_d"] = c["Z"].T @ dY', 'g["w_d"] = c["Z"].T @ dZ[:, :h] if False else c["Z"].T @ (dY * 1.0001)'),
 ("stage.py", 'g["w_gu"] = c["B"].T @ dGU', 'g["w_gu"] = c["H"].T @ dGU'),
 ("stage.py", 'g["w_o"] = c["C"].T @ dH', 'g["w_o"] = c["C"].T @ dY'),
 ("stage.py", 'g["w_qkv"] = c["A"].T @ dQKV', 'g["w_qkv"] = c["X"].T @ dQKV'),
 ("stage.py", 'dq = st("dqk", rope_apply(dq, c["ang"], sign=-1.0))', 'dq = st("dqk", rope_apply(dq, c["ang"], sign=1.0))'),
 ("stage.py", 'dk = st("dqk", rope_apply(dk, c["ang"], sign=-1.0))', 'dk = st("dqk", dk)'),
 ("stage.py", 'dHn, g["gamma2"] = rmsnorm_bwd(dB, c["H"], w["gamma2"], c["r2"])', 'dHn, g["gamma2"] = rmsnorm_bwd(dB, c["H"], w["gamma2"], c["r1"])'),
 ("stage.py", "    for l in range(k - 1, -1, -1):\n        d, grads[l]", "    for l in range(k):\n        d, grads[l]"),
 ("stage.py", "                total[l][n] += grads[l][n]", "                total[l][n] = grads[l][n]"),
 # ends
 ("ends.py", "ok = (tok >= 0) & (tok < embed.shape[0])", "ok = (tok > 0) & (tok < embed.shape[0])"),
 ("ends.py", "            g[tok[t]] += dx[t]", "            g[tok[t]] = dx[t]"),
 ("ends.py", "lse = m[:, 0] + np.log(np.exp(logits - m).sum(axis=1))", "lse = np.log(np.exp(logits - m).sum(axis=1))"),
 ("ends.py", "loss = float(np.sum((lse - picked)[ok]) / tgt.size)", "loss = float(np.sum((lse - picked)[ok]) / max(1, ok.sum()))"),
 ("ends.py", "loss = float(np.sum((lse - picked)[ok]) / tgt.size)", "loss = float(np.sum((lse + picked)[ok]) / tgt.size)"),
 ("ends.py", "dlogits[np.nonzero(ok)[0], tgt[ok]] -= 1.0", "dlogits[np.nonzero(ok)[0], tgt[ok]] += 1.0"),
 ("ends.py", "dlogits[~ok] = 0.0", "pass"),
 ("ends.py", "dlogits * (loss_weight / T))", "dlogits * loss_weight)"),
 ("ends.py", 'g_wlm = cache["nrm"].T @ dlogits', 'g_wlm = cache["y"].T @ dlogits'),
 ("ends.py", 'dn = st("dn", dlogits @ p["w_lm"].T)', 'dn = st("dn", prob @ p["w_lm"].T)'),
 # optim
 ("optim.py", "m = b1 * m + (1.0 - b1) * g", "m = b1 * m + g"),
 ("optim.py", "v = b2 * v + (1.0 - b2) * g * g", "v = b2 * v + (1.0 - b2) * g"),
 ("optim.py", "mhat = m / (1.0 - b1 ** t)", "mhat = m"),
 ("optim.py", "vhat = v / (1.0 - b2 ** t)", "vhat = v / (1.0 - b1 ** t)"),
 ("optim.py", "(np.sqrt(vhat) + eps)", "np.sqrt(vhat + eps)"),
 ("optim.py", "+ wd * w)", "- wd * w)"),
 ("optim.py", "+ wd * w)", "+ wd * mhat)"),
 ("optim.py", "x = (e / u) / tau_ref_ms", "x = e / tau_ref_ms"),
 ("optim.py", "abs(x - prev) / prev > threshold", "abs(x - prev) > threshold"),
 ("optim.py", "abs(x - prev) / prev > threshold", "(x - prev) / prev > threshold"),
 # plan
 ("plan.py", "v = max(yj * lj for yj, lj in zip(y, l))", "v = sum(yj * lj for yj, lj in zip(y, l))"),
 ("plan.py", "        if best is None or v < best:\n            best, arg = v, [l]", "        if best is None or v > best:\n            best, arg = v, [l]"),
 ("plan.py", "for first in range(hi + 1):", "for first in range(1, hi + 1):"),
 ("plan.py", "zip(pipelines, ls, m)) * tau", "zip(pipelines, ls, m))"),
 ("plan.py", "a_ub[j, j] = y[j]", "a_ub[j, j] = 1.0 / y[j]"),
 ("plan.py", "acc + 1.0 / (rho[g] * max(x[i] for i in members))", "acc + 1.0 / (rho[g] * min(x[i] for i in members))"),
 ("plan.py", "acc + 1.0 / (rho[g] * max(x[i] for i in members))", "acc + 1.0 / max(x[i] for i in members)"),
 ("plan.py", "            if best is None or acc > best:", "            if best is None or acc < best:"),
 ("plan.py", "runs[g] = tuple(range(at, at + sizes[g]))", "runs[g] = tuple(range(at, at + sizes[order[0]]))"),
]


def main():
    survivors = []
    with tempfile.TemporaryDirectory() as tmp:
        for name in os.listdir(ROOT):
            if name == "oracle" or name.startswith((".", "_")) or not (name.endswith(".py") or os.path.isdir(os.path.join(ROOT, name))):
                continue
            os.symlink(os.path.join(ROOT, name), os.path.join(tmp, name))
        os.mkdir(os.path.join(tmp, "oracle"))
        for i, (f, old, new) in enumerate([("", "", "")] + M):
            i -= 1  # -1: the control run on an unchanged copy, which must pass
            for name in os.listdir(os.path.join(ROOT, "oracle")):
                if name.endswith(".py"):
                    src = open(os.path.join(ROOT, "oracle", name)).read()
                    if name == f:
                        assert src.count(old) == 1, (f, old)
                        src = src.replace(old, new)
                    open(os.path.join(tmp, "oracle", name), "w").write(src)
            r = subprocess.run([sys.executable, "-m", "pytest", "tests", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                               cwd=tmp, capture_output=True, text=True, env=dict(os.environ, PYTHONDONTWRITEBYTECODE="1"))
            killed = r.returncode != 0
            if i < 0:
                assert not killed, "the unchanged copy fails:\n" + r.stdout[-2000:]
                print("control run on the unchanged copy passes", flush=True)
                continue
            print(f"[{i:2d}] {f}: {'caught  ' if killed else 'SURVIVED'} {old.strip()[:48]!r} -> {new.strip()[:48]!r}", flush=True)
            if not killed:
                survivors.append(i)
    print(f"{len(M) - len(survivors)} of {len(M)} planted mistakes caught; survivors: {survivors}")
    return 1 if survivors else 0


if __name__ == "__main__":
    sys.exit(main())
