"""Counter-based N(0,1) generator and the parameter layout of a decoder stage.

Generator (stated once here; the HIP library carries its own implementation of the same text):

    mix(z):  z += 0x9E3779B97F4A7C15            (all arithmetic modulo 2**64)
             z  = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9
             z  = (z ^ (z >> 27)) * 0x94D049BB133111EB
             return z ^ (z >> 31)
    stream(seed, tensor_id, layer) = mix(mix(seed) ^ ((tensor_id << 32) | layer))
    r1 = mix(stream + 2*i), r2 = mix(stream + 2*i + 1)          for flat element index i
    u1 = ((r1 >> 11) + 1) * 2**-53   in (0, 1]
    u2 =  (r2 >> 11)      * 2**-53   in [0, 1)
    z  = sqrt(-2 ln u1) * cos(2 pi u2)                           (Box-Muller, fp64)

Projection weights are 0.02*z, RMSNorm gains 1 + 0.02*z, activations and upstream gradients z; each value
is then rounded once (nearest-even) to the storage type, bf16 or fp32.  The workloads are the
LLaMA-2-architecture shapes of the paper's experimental setup (Sec. 7.1: context length 4K, micro-batch
size 1), which names no dataset for this compute; seeded Gaussians stand in for activations and weights.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

TID_GAMMA1, TID_WQKV, TID_WO, TID_GAMMA2, TID_WGU, TID_WD = 0, 1, 2, 3, 4, 5
TID_X, TID_DY, TID_PLAN = 16, 17, 18

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


@dataclass(frozen=True)
class StageShape:
    """Shape of one GPU's pipeline stage: the layer shape plus the two integers a plan assigns to it,
    the layer count (l_{i,j} in the paper's notation table) and the micro-batch count (m_i)."""
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    seq: int
    micro_batch: int
    layers: int
    microbatches: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    dtype: str = "bf16"          # storage type: "bf16" or "fp32"

    @property
    def q_dim(self): return self.n_q_heads * self.head_dim
    @property
    def kv_dim(self): return self.n_kv_heads * self.head_dim
    @property
    def tokens(self): return self.seq * self.micro_batch
    def with_(self, **kw): return replace(self, **kw)

    def matrix_params(self):
        return self.hidden * (self.q_dim + 2 * self.kv_dim) + self.q_dim * self.hidden + 3 * self.hidden * self.ffn

    def model_flops_layer_mb(self):
        """fwd+bwd model FLOPs of one layer on one micro-batch: 3 x (dense GEMMs + causal attention)."""
        gemm = 2 * self.tokens * self.matrix_params()
        attn = 4 * self.micro_batch * self.n_q_heads * self.head_dim * self.seq * (self.seq + 1) // 2
        return 3 * (gemm + attn)


CONFIGS = {
    "tiny": StageShape(256, 4, 4, 64, 688, 128, 2, 2, 1),
    "7b": StageShape(4096, 32, 32, 128, 11008, 4096, 1, 4, 4),
    "13b": StageShape(5120, 40, 40, 128, 13824, 4096, 1, 5, 7),
    "70b_tp4": StageShape(8192, 16, 2, 128, 7168, 4096, 1, 3, 8),
    "sweep": StageShape(4096, 32, 32, 128, 11008, 2048, 1, 9, 16),
}


def mix64(z):
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = z + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def _stream(seed, tensor_id, layer):
    return mix64(mix64(np.uint64(seed)) ^ np.uint64((int(tensor_id) << 32) | int(layer)))


def normal(seed, tensor_id, layer, n, start=0):
    """n standard normals (fp64) for flat indices start .. start+n-1 of tensor (tensor_id, layer).
    Large requests are cut into chunks that a small thread pool fills (the value of an element depends on
    its index only, never on the chunking)."""
    s = _stream(seed, tensor_id, layer)
    out = np.empty(n, dtype=np.float64)
    chunk = 1 << 20

    def fill(lo):
        hi = min(n, lo + chunk)
        i = np.arange(start + lo, start + hi, dtype=np.uint64)
        with np.errstate(over="ignore"):
            c = s + np.uint64(2) * i
            r1 = mix64(c)
            r2 = mix64(c + np.uint64(1))
        u1 = ((r1 >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53
        u2 = (r2 >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
        out[lo:hi] = np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * np.pi) * u2)

    starts = range(0, n, chunk)
    if n <= 4 * chunk:
        for lo in starts:
            fill(lo)
    else:
        from concurrent.futures import ThreadPoolExecutor
        import os
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(fill, starts))
    return out


def uniform_u64(seed, tensor_id, layer, i):
    """The raw 64-bit draw r1 for element i (used for the integer plan sweep)."""
    s = _stream(seed, tensor_id, layer)
    with np.errstate(over="ignore"):
        return int(mix64(s + np.uint64(2) * np.uint64(i)))


def f32_to_bf16_bits(a):
    """fp32 array -> uint16 bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(a64, dtype):
    """Round an fp64 array once to the storage type; returns (storage array, fp64 value of it).
    bf16 storage is returned as uint16 bit patterns."""
    if dtype == "fp32":
        s = a64.astype(np.float32)
        return s, s.astype(np.float64)
    if dtype == "bf16":
        # fp64 -> bf16 in ONE rounding (going through fp32 first would round twice).
        b = _f64_to_bf16_bits(a64)
        return b, bf16_bits_to_f32(b).astype(np.float64)
    raise ValueError(dtype)


def _f64_to_bf16_bits(a64):
    """fp64 -> bf16 bit patterns with a single round-to-nearest-even (values well inside bf16's normal
    range, which holds for every tensor generated here; zeros map to zero)."""
    a = np.ascontiguousarray(a64, dtype=np.float64)
    m, e = np.frexp(a)                       # a = m * 2**e, 0.5 <= |m| < 1
    q = np.rint(np.ldexp(m, 8))              # 8 significant bits, ties to even
    v = np.ldexp(q, e - 8).astype(np.float32)   # exactly representable in bf16 (and fp32)
    return (v.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def param_layout(sh: StageShape):
    """Public per-layer parameter order: (name, tensor_id, rows, cols, offset), each row-major [in, out]."""
    h, qd, kvd, f = sh.hidden, sh.q_dim, sh.kv_dim, sh.ffn
    items = [("gamma1", TID_GAMMA1, 1, h), ("w_qkv", TID_WQKV, h, qd + 2 * kvd), ("w_o", TID_WO, qd, h),
             ("gamma2", TID_GAMMA2, 1, h), ("w_gu", TID_WGU, h, 2 * f), ("w_d", TID_WD, f, h)]
    out, off = [], 0
    for name, tid, r, c in items:
        out.append((name, tid, r, c, off))
        off += r * c
    return out


def layer_param_elems(sh: StageShape):
    name, tid, r, c, off = param_layout(sh)[-1]
    return off + r * c


def make_params(sh: StageShape, seed, layers=None):
    """Flat parameter vector for `layers` layers in the public layout.
    Returns (storage array [uint16 bits or fp32], fp64 values)."""
    L = sh.layers if layers is None else layers
    per = layer_param_elems(sh)
    vals = np.empty(L * per, dtype=np.float64)
    for l in range(L):
        for name, tid, r, c, off in param_layout(sh):
            z = normal(seed, tid, l, r * c)
            vals[l * per + off: l * per + off + r * c] = (1.0 + 0.02 * z) if name.startswith("gamma") else 0.02 * z
    return round_to_storage(vals, sh.dtype)


def split_params(sh: StageShape, flat64, layer):
    """Views of one layer's tensors (dict name -> 2-D/1-D fp64 array) inside a flat vector."""
    per = layer_param_elems(sh)
    base = layer * per
    d = {}
    for name, tid, r, c, off in param_layout(sh):
        v = flat64[base + off: base + off + r * c]
        d[name] = v.reshape(c) if r == 1 and name.startswith("gamma") else v.reshape(r, c)
    return d


def make_x(sh: StageShape, seed, mb):
    """Stage input of micro-batch mb: [micro_batch, seq, hidden] ~ N(0,1), rounded to storage."""
    n = sh.tokens * sh.hidden
    s, v = round_to_storage(normal(seed, TID_X, mb, n), sh.dtype)
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    return s.reshape(shape), v.reshape(shape)


def make_dy(sh: StageShape, seed, mb):
    """Upstream gradient of micro-batch mb: same shape as the stage output."""
    n = sh.tokens * sh.hidden
    s, v = round_to_storage(normal(seed, TID_DY, mb, n), sh.dtype)
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    return s.reshape(shape), v.reshape(shape)


def plan_sweep(seed=4000, n_plans=16, layer_range=(2, 9), mb_range=(1, 16)):
    """Seeded (layers, micro-batches) pairs, uniform in the given inclusive ranges: the two integers the
    lower-level problem (Eq. 1) assigns per GPU."""
    plans = []
    for i in range(n_plans):
        k = layer_range[0] + uniform_u64(seed, TID_PLAN, 0, 2 * i) % (layer_range[1] - layer_range[0] + 1)
        m = mb_range[0] + uniform_u64(seed, TID_PLAN, 0, 2 * i + 1) % (mb_range[1] - mb_range[0] + 1)
        plans.append((int(k), int(m)))
    return plans


# ---------------------------------------------------------------- first / last stage (embedding, final norm, LM head)
TID_EMBED, TID_GAMMA_F, TID_WLM = 6, 7, 8
TID_TOKENS, TID_TARGETS = 19, 20


@dataclass(frozen=True)
class EndsShape:
    """Shape of the non-uniform layers of the first and last pipeline stage (Appendix B.4): token embedding, final
    RMSNorm, LM head, mean cross-entropy loss.  LLaMA-2 (Sec. 7.1) has a vocabulary of 32000."""
    hidden: int
    vocab: int
    seq: int
    micro_batch: int
    microbatches: int
    rms_eps: float = 1e-5
    dtype: str = "bf16"

    @property
    def tokens(self): return self.seq * self.micro_batch
    def with_(self, **kw): return replace(self, **kw)

    def model_flops_mb(self):
        """fwd+bwd model FLOPs of the LM head on one micro-batch (the embedding and the loss are not contractions)."""
        return 3 * 2 * self.tokens * self.hidden * self.vocab


ENDS_CONFIGS = {
    "tiny": EndsShape(256, 1000, 128, 2, 2),
    "7b": EndsShape(4096, 32000, 4096, 1, 4),
}


def ends_param_layout(sh: EndsShape):
    """(name, tensor_id, rows, cols, offset) of embed [V, h], gamma_f [h], w_lm [h, V]."""
    items = [("embed", TID_EMBED, sh.vocab, sh.hidden), ("gamma_f", TID_GAMMA_F, 1, sh.hidden),
             ("w_lm", TID_WLM, sh.hidden, sh.vocab)]
    out, off = [], 0
    for name, tid, r, c in items:
        out.append((name, tid, r, c, off))
        off += r * c
    return out


def make_ends_params(sh: EndsShape, seed):
    """Flat parameter vector (storage array, fp64 values) of the first/last-stage layers."""
    lay = ends_param_layout(sh)
    total = lay[-1][4] + lay[-1][2] * lay[-1][3]
    vals = np.empty(total, dtype=np.float64)
    for name, tid, r, c, off in lay:
        z = normal(seed, tid, 0, r * c)
        vals[off:off + r * c] = (1.0 + 0.02 * z) if name.startswith("gamma") else 0.02 * z
    return round_to_storage(vals, sh.dtype)


def split_ends_params(sh: EndsShape, flat64):
    d = {}
    for name, tid, r, c, off in ends_param_layout(sh):
        v = flat64[off:off + r * c]
        d[name] = v.reshape(c) if r == 1 else v.reshape(r, c)
    return d


def _token_draws(seed, tid, mb, n, vocab):
    s = _stream(seed, tid, mb)
    with np.errstate(over="ignore"):
        r = mix64(s + np.uint64(2) * np.arange(n, dtype=np.uint64))
    return (r % np.uint64(vocab)).astype(np.int32)


def make_tokens(sh: EndsShape, seed, mb, skew=False):
    """Token ids [b, S] of micro-batch mb, uniform over the vocabulary; skew=True folds them onto a 64th of it so
    that many positions share a token (the embedding gradient then sums several rows per table row)."""
    t = _token_draws(seed, TID_TOKENS, mb, sh.tokens, sh.vocab)
    if skew:
        t = t % np.int32(max(1, sh.vocab // 64))
    return t.reshape(sh.micro_batch, sh.seq)


def make_targets(sh: EndsShape, seed, mb):
    return _token_draws(seed, TID_TARGETS, mb, sh.tokens, sh.vocab).reshape(sh.micro_batch, sh.seq)


def to_device(storage, dtype):
    """Storage array of this generator (uint16 bf16 bit patterns, or fp32) -> CUDA tensor of the storage type.
    Plumbing only; torch is imported here so that the generator itself stays importable without it."""
    import torch
    if dtype == "bf16":
        return torch.from_numpy(storage.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(storage)).cuda()
