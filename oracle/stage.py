"""Plain fp64 CPU oracle for one GPU's pipeline stage: forward and backward of `l` LLaMA-style decoder
layers over `m` accumulated micro-batches.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's cpu_baseline leg may call
this; it shares no code with the HIP library and is not tuned.

What the paper fixes: the stage's cost is t = y * l * tau(b) and a pipeline's step takes about
m * max t (Sec. 4.2, time cost model), with l layers and m micro-batches assigned per GPU (Sec. 4.2,
Eq. 1; Table 1 of notations), on models of the LLaMA-2 architecture with context 4K and micro-batch 1 (Sec. 7.1).  The paper
does not write the layer's arithmetic out; the definitions below are the textbook ones of that
architecture (pre-norm residual block, RMSNorm, rotary position embedding with half-split pairing,
causal softmax attention with grouped KV heads, SwiGLU feed-forward, no biases).  The method is exact
mathematics, so the oracle is the plain definition: the full S x S score matrix is materialised, nothing
is blocked, fused or reordered.  All arithmetic is fp64; callers pass values already rounded to the
storage type when they model a bf16 run.

Rounding hook.  The layer functions take an optional `store(name, tensor)` hook, called at every named
intermediate tensor of the definition (ROUNDING_POINTS).  With the default (identity) the oracle is the exact fp64
function that the pins below fix, and that is what parity is judged against.  A hook that rounds some of the names
to bf16 states what an otherwise exact path computes when it keeps those tensors in bf16; the tests use it only to
measure, on the CPU, how far such roundings alone move a result (one name at a time, or a set of names), never as
the function the library has to match.  The arithmetic between two hook calls is the same fp64 code either way.

Parity pins (tests/test_oracle_*.py): central finite differences on every parameter and on dX, softmax
rows summing to one, causality, RoPE norm preservation / relative-position property, the RMSNorm closed
form, attention special cases, a brute-force scalar-loop re-derivation on tiny shapes, linearity of
gradient accumulation and layer composition.
"""
from __future__ import annotations

import numpy as np


def _identity(name, t):
    return t

# ---------------------------------------------------------------- RMSNorm


def rmsnorm_fwd(x, gamma, eps):
    """a[t,i] = x[t,i] * r[t] * gamma[i],  r[t] = (mean_i x[t,i]^2 + eps)^(-1/2).  x: [T,h]."""
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x * r * gamma, r


def rmsnorm_bwd(da, x, gamma, r):
    """Reverse mode of rmsnorm_fwd: returns (dx, dgamma).  With n = x*r and dn = da*gamma:
    dx = r * (dn - n * mean_i(dn*n)),  dgamma = sum_t da*n."""
    n = x * r
    dn = da * gamma
    dx = r * (dn - n * np.mean(dn * n, axis=-1, keepdims=True))
    return dx, np.sum(da * n, axis=0)

# ---------------------------------------------------------------- RoPE


def rope_angles(seq, head_dim, base):
    """angle[p,i] = p * base^(-2i/d), p = 0..seq-1, i = 0..d/2-1."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    theta = base ** (-2.0 * i / head_dim)
    return np.arange(seq, dtype=np.float64)[:, None] * theta[None, :]


def rope_apply(u, angle, sign=1.0):
    """Rotate the pairs (u_i, u_{i+d/2}) of every head vector by sign*angle[p,i].
    u: [b, S, n_heads, d]; position p is the index inside the sequence."""
    d2 = u.shape[-1] // 2
    c = np.cos(angle)[None, :, None, :]
    s = sign * np.sin(angle)[None, :, None, :]
    u1, u2 = u[..., :d2], u[..., d2:]
    return np.concatenate([u1 * c - u2 * s, u1 * s + u2 * c], axis=-1)

# ---------------------------------------------------------------- attention


def attention_fwd(q, k, v, store=None):
    """Causal softmax attention with grouped KV heads.
    q: [b,S,n_q,d], k,v: [b,S,n_kv,d].  Query head hq reads KV head hq // (n_q/n_kv).
    Returns o [b,S,n_q,d] and the probabilities p [b,n_q,S,S] (zero above the diagonal).
    store: optional rounding hook (see the module header); "p" is the probability operand of the product with V."""
    st = store or _identity
    b, S, nq, d = q.shape
    g = nq // k.shape[2]
    mask = np.tril(np.ones((S, S), dtype=bool))
    o = np.empty_like(q)
    p = np.zeros((b, nq, S, S))
    for bi in range(b):
        for hq in range(nq):
            hk = hq // g
            s = q[bi, :, hq, :] @ k[bi, :, hk, :].T / np.sqrt(d)
            s = np.where(mask, s, -np.inf)
            e = np.exp(s - s.max(axis=1, keepdims=True))      # masked entries are exactly 0
            pr = e / e.sum(axis=1, keepdims=True)
            p[bi, hq] = pr
            o[bi, :, hq, :] = st("p", pr) @ v[bi, :, hk, :]
    return o, p


def attention_bwd(do, q, k, v, p, store=None):
    """Reverse mode of attention_fwd.  dV_j += sum_i p_ij dO_i; dp_ij = dO_i . V_j;
    ds_ij = p_ij (dp_ij - sum_j' p_ij' dp_ij'); dQ_i = sum_j ds_ij K_j / sqrt(d);
    dK_j += sum_i ds_ij Q_i / sqrt(d), the KV gradients summed over the query heads of a group.
    store: optional rounding hook; "p_dv" is the probability operand of the dV product, "ds" the score-gradient
    operand of the dQ and dK products."""
    st = store or _identity
    b, S, nq, d = q.shape
    g = nq // k.shape[2]
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for bi in range(b):
        for hq in range(nq):
            hk = hq // g
            pr = p[bi, hq]
            dO = do[bi, :, hq, :]
            dv[bi, :, hk, :] += st("p_dv", pr).T @ dO
            dp = dO @ v[bi, :, hk, :].T
            ds = st("ds", pr * (dp - np.sum(pr * dp, axis=1, keepdims=True)))
            dq[bi, :, hq, :] = ds @ k[bi, :, hk, :] / np.sqrt(d)
            dk[bi, :, hk, :] += ds.T @ q[bi, :, hq, :] / np.sqrt(d)
    return dq, dk, dv

# ---------------------------------------------------------------- SwiGLU


def sigmoid(g):
    return 1.0 / (1.0 + np.exp(-g))


def swiglu_fwd(g, u):
    """z = g * sigmoid(g) * u."""
    return g * sigmoid(g) * u


def swiglu_bwd(dz, g, u):
    """dg = dz*u*sigma(g)*(1 + g*(1 - sigma(g))),  du = dz*g*sigma(g)."""
    s = sigmoid(g)
    return dz * u * s * (1.0 + g * (1.0 - s)), dz * g * s

# ---------------------------------------------------------------- one decoder layer

# Rounding points: every intermediate tensor of one layer's definition has a name, in order forward then
# backward.  "_pre" = before the rotary step (which changes q and k, not v); "gu" is what the forward's SwiGLU
# consumes, "gu_kept" what the backward's SwiGLU derivative consumes; "p", "p_dv", "ds" are the matrix operands
# inside the attention (see attention_fwd / attention_bwd).  A hook sees (name, tensor) and returns the tensor
# its consumers read.
ROUNDING_POINTS = ("a", "qk_pre", "v", "qk", "p", "o", "h", "b", "gu", "gu_kept", "z", "y",
                   "dz", "dgu", "db", "dh", "dc", "p_dv", "ds", "dqk_pre", "dv", "dqk", "da", "dx")


def layer_forward(x, w, sh, store=None):
    """x: [b,S,h]; w: dict gamma1,w_qkv,w_o,gamma2,w_gu,w_d (row-major [in,out]); sh: shape object with
    hidden,n_q_heads,n_kv_heads,head_dim,ffn,rms_eps,rope_base.  Returns (y, cache)."""
    st = store or _identity
    b, S, h = x.shape
    nq, nkv, d, f = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.ffn
    qd, kvd = nq * d, nkv * d
    X = x.reshape(b * S, h)
    A, r1 = rmsnorm_fwd(X, w["gamma1"], sh.rms_eps)
    A = st("a", A)
    QKV = A @ w["w_qkv"]
    ang = rope_angles(S, d, sh.rope_base)
    qk = st("qk", rope_apply(st("qk_pre", QKV[:, :qd + kvd]).reshape(b, S, nq + nkv, d), ang))
    q, k = qk[:, :, :nq, :], qk[:, :, nq:, :]
    v = st("v", QKV[:, qd + kvd:]).reshape(b, S, nkv, d)
    o, p = attention_fwd(q, k, v, store)
    o = st("o", o)
    C = o.reshape(b * S, qd)
    H = st("h", X + C @ w["w_o"])
    B, r2 = rmsnorm_fwd(H, w["gamma2"], sh.rms_eps)
    B = st("b", B)
    GU = st("gu", B @ w["w_gu"])
    Z = st("z", swiglu_fwd(GU[:, :f], GU[:, f:]))
    Y = st("y", H + Z @ w["w_d"])
    GUk = st("gu_kept", GU)
    cache = dict(X=X, A=A, r1=r1, q=q, k=k, v=v, p=p, C=C, H=H, B=B, r2=r2, G=GUk[:, :f], U=GUk[:, f:], Z=Z, ang=ang)
    return Y.reshape(b, S, h), cache


def layer_backward(dy, w, cache, sh, store=None):
    """Reverse mode of layer_forward.  Returns (dx, grads dict with the same keys as w)."""
    st = store or _identity
    b, S, h = dy.shape
    nq, nkv, d, f = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.ffn
    qd, kvd = nq * d, nkv * d
    c = cache
    dY = dy.reshape(b * S, h)
    g = {}
    dZ = st("dz", dY @ w["w_d"].T)
    g["w_d"] = c["Z"].T @ dY
    dG, dU = swiglu_bwd(dZ, c["G"], c["U"])
    dGU = st("dgu", np.concatenate([dG, dU], axis=1))
    dB = st("db", dGU @ w["w_gu"].T)
    g["w_gu"] = c["B"].T @ dGU
    dHn, g["gamma2"] = rmsnorm_bwd(dB, c["H"], w["gamma2"], c["r2"])
    dH = st("dh", dY + dHn)
    dC = st("dc", dH @ w["w_o"].T)
    g["w_o"] = c["C"].T @ dH
    dq, dk, dv = attention_bwd(dC.reshape(b, S, nq, d), c["q"], c["k"], c["v"], c["p"], store)
    dq, dk, dv = st("dqk_pre", dq), st("dqk_pre", dk), st("dv", dv)
    dq = st("dqk", rope_apply(dq, c["ang"], sign=-1.0))
    dk = st("dqk", rope_apply(dk, c["ang"], sign=-1.0))
    dQKV = np.concatenate([dq.reshape(b * S, qd), dk.reshape(b * S, kvd), dv.reshape(b * S, kvd)], axis=1)
    dA = st("da", dQKV @ w["w_qkv"].T)
    g["w_qkv"] = c["A"].T @ dQKV
    dXn, g["gamma1"] = rmsnorm_bwd(dA, c["X"], w["gamma1"], c["r1"])
    dX = st("dx", dH + dXn)
    return dX.reshape(b, S, h), g

# ---------------------------------------------------------------- the stage


def stage_forward(x, weights, sh, k_layers=None, store=None):
    """Layers 0..k-1 composed.  weights: list of per-layer dicts.  k = 0 is the identity.
    Returns (y, list of per-layer caches)."""
    k = len(weights) if k_layers is None else k_layers
    caches = []
    y = np.array(x, dtype=np.float64)
    for l in range(k):
        y, c = layer_forward(y, weights[l], sh, store)
        caches.append(c)
    return y, caches


def stage_backward(dy, weights, caches, sh, store=None):
    """Reverse of stage_forward for one micro-batch: returns (dx, list of per-layer grad dicts)."""
    k = len(caches)
    grads = [None] * k
    d = np.array(dy, dtype=np.float64)
    for l in range(k - 1, -1, -1):
        d, grads[l] = layer_backward(d, weights[l], caches[l], sh, store)
    return d, grads


def stage_step(xs, dys, weights, sh, k_layers=None):
    """One stage step: m micro-batches forward, then backward with the parameter gradients summed over
    the micro-batches in ascending order.  xs, dys: lists of [b,S,h].  Returns (ys, dxs, grads)."""
    k = len(weights) if k_layers is None else k_layers
    total = [{n: np.zeros_like(v) for n, v in weights[l].items()} for l in range(k)]
    ys, dxs = [], []
    for x, dy in zip(xs, dys):
        y, caches = stage_forward(x, weights, sh, k)
        dx, grads = stage_backward(dy, weights, caches, sh)
        for l in range(k):
            for n in total[l]:
                total[l][n] += grads[l][n]
        ys.append(y)
        dxs.append(dx)
    return ys, dxs, total
