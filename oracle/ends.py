"""Oracle for the first/last-stage layers (token embedding; final RMSNorm, LM head, mean cross-entropy):
TEST INFRASTRUCTURE, not a product path.  Plain numpy in fp64, written from the definitions; no blocking, no fusion,
no online softmax.  Only tests, the smoke test and the benchmark's CPU-baseline leg may import it.

The paper (Appendix B.4) only names these layers (the non-uniform layers of the first and last pipeline stage of a
model of the LLaMA-2 architecture, Sec. 7.1); their arithmetic is the textbook one:
    x_t      = embed[token_t]                                   (a token outside [0, V) gives a zero row)
    nrm      = y * rsqrt(mean(y^2) + eps) * gamma_f             (row-wise, like the layer norms of the stage oracle)
    logits   = nrm w_lm
    loss     = (1/T) sum_t [ log sum_v exp(logits_tv) - logits_t[target_t] ]   (targets outside [0, V) are skipped,
                                                                                 the divisor stays T)
"""
import numpy as np

from oracle.stage import rmsnorm_bwd, rmsnorm_fwd


def embed_forward(tokens, embed):
    tok = np.asarray(tokens).reshape(-1)
    x = np.zeros((tok.size, embed.shape[1]), dtype=np.float64)
    ok = (tok >= 0) & (tok < embed.shape[0])
    x[ok] = embed[tok[ok]]
    return x


def embed_backward(tokens, dx, vocab):
    """d embed[v] = sum of dx rows at the positions holding token v (positions in ascending order)."""
    tok = np.asarray(tokens).reshape(-1)
    g = np.zeros((vocab, dx.shape[1]), dtype=np.float64)
    for t in range(tok.size):
        if 0 <= tok[t] < vocab:
            g[tok[t]] += dx[t]
    return g


def head_forward(y, targets, p, eps, store=None):
    """Returns (loss, cache).  `store(name, array)`, if given, stands for writing a tensor to memory in the storage
    type (names: nrm, logits, dlogits, dn, dy), like the hook of the stage oracle."""
    st = store or (lambda name, a: a)
    tgt = np.asarray(targets).reshape(-1)
    nrm, r = rmsnorm_fwd(y, p["gamma_f"], eps)
    nrm = st("nrm", nrm)
    logits = st("logits", nrm @ p["w_lm"])
    m = logits.max(axis=1, keepdims=True)
    lse = m[:, 0] + np.log(np.exp(logits - m).sum(axis=1))
    ok = (tgt >= 0) & (tgt < logits.shape[1])
    picked = np.zeros(tgt.size)
    picked[ok] = logits[np.nonzero(ok)[0], tgt[ok]]
    loss = float(np.sum((lse - picked)[ok]) / tgt.size)
    return loss, dict(y=y, r=r, nrm=nrm, logits=logits, lse=lse, tgt=tgt, ok=ok)


def head_backward(cache, p, loss_weight, store=None):
    """Gradient of loss_weight * loss: returns (dy, grads dict gamma_f, w_lm, dlogits)."""
    st = store or (lambda name, a: a)
    logits, lse, tgt, ok = cache["logits"], cache["lse"], cache["tgt"], cache["ok"]
    T = tgt.size
    prob = np.exp(logits - lse[:, None])
    dlogits = prob.copy()
    dlogits[np.nonzero(ok)[0], tgt[ok]] -= 1.0
    dlogits[~ok] = 0.0
    dlogits = st("dlogits", dlogits * (loss_weight / T))
    g_wlm = cache["nrm"].T @ dlogits
    dn = st("dn", dlogits @ p["w_lm"].T)
    dy, g_gamma = rmsnorm_bwd(dn, cache["y"], p["gamma_f"], cache["r"])
    return st("dy", dy), dict(gamma_f=g_gamma, w_lm=g_wlm), dlogits
