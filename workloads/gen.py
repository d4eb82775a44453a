"""Seeded tensor generators shared by the oracle-side and HIP-side harness code.

Every tensor is a pure function of (seed, tensor id, fixed chunking), independent of thread count.
bf16 workloads get values already rounded (round-to-nearest-even) onto the bf16 grid and returned as
float32, so the same numbers can be uploaded exactly as bf16 and read exactly by a float64 oracle.
"""
from concurrent.futures import ThreadPoolExecutor
import os
import numpy as np

_CHUNK = 1 << 22   # elements per independently keyed chunk (fixed: results do not depend on threads)
_POOL = None


def _pool():
    global _POOL
    if _POOL is None:
        _POOL = ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1))
    return _POOL


def _round_bf16_inplace(v):
    u = v.view(np.uint32)
    t = u >> np.uint32(16)
    t &= np.uint32(1)
    t += np.uint32(0x7FFF)
    u += t
    u &= np.uint32(0xFFFF0000)


def to_bf16_grid(x):
    """Round float32 values to the nearest bf16-representable value (ties to even); returns float32."""
    v = np.array(x, dtype=np.float32, copy=True)
    _round_bf16_inplace(v.reshape(-1))
    return v


def _fill_chunk(out, lo, hi, key, mean, std, bf16):
    g = np.random.Generator(np.random.Philox(key=key))
    v = out[lo:hi]
    g.standard_normal(hi - lo, dtype=np.float32, out=v)
    v *= np.float32(std)
    if mean:
        v += np.float32(mean)
    if bf16:
        _round_bf16_inplace(v)


def normal_tensor(seed, tensor_id, shape, std, mean=0.0, bf16=False, out=None):
    """float32 tensor ~ N(mean, std^2); chunk c of the flattened tensor uses Philox key
    (seed, tensor_id * 2^20 + c).  `out` (flat float32 of the right size) is filled if given."""
    n = int(np.prod(shape))
    if out is None:
        out = np.empty(n, dtype=np.float32)
    assert out.size == n and out.dtype == np.float32
    jobs = []
    for c, lo in enumerate(range(0, n, _CHUNK)):
        hi = min(n, lo + _CHUNK)
        key = [np.uint64(seed), np.uint64(tensor_id) * np.uint64(1 << 20) + np.uint64(c)]
        jobs.append((out, lo, hi, key, mean, std, bf16))
    if len(jobs) == 1:
        _fill_chunk(*jobs[0])
    else:
        list(_pool().map(lambda a: _fill_chunk(*a), jobs))
    return out.reshape(shape)


# tensor ids: 1 tok_emb, 2 norm_final, 3 lm_head, 16*(layer+1)+k for the per-layer tensors
_LAYER_TENSORS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "norm_attn", "norm_ffn")


class Weights:
    """Random-init decoder weights: matrices and embeddings ~ N(0, 0.02^2), RMSNorm gains
    ~ 1 + N(0, 0.02^2).  All matrices are row-major [out][in].  Layers are generated on demand so a
    13B model never has to sit in host memory at once."""

    def __init__(self, model, seed, reuse_buffers=False):
        """reuse_buffers: layer() hands back the same arrays on every call, overwritten in place
        (saves the page-fault cost of fresh allocations when streaming a large model)."""
        self.model = model
        self.seed = seed
        self.bf16 = model.dtype != "fp32"
        self._bufs = {} if reuse_buffers else None

    def _mat(self, tid, shape, name=None):
        out = None
        if self._bufs is not None and name is not None:
            out = self._bufs.get(name)
            if out is None:
                out = self._bufs[name] = np.empty(int(np.prod(shape)), np.float32)
        return normal_tensor(self.seed, tid, shape, 0.02, 0.0, self.bf16, out=out)

    def _gain(self, tid, n):
        return normal_tensor(self.seed, tid, (n,), 0.02, 1.0, self.bf16)

    def tok_emb(self):
        return self._mat(1, (self.model.vocab, self.model.d_model))

    def norm_final(self):
        return self._gain(2, self.model.d_model)

    def lm_head(self):
        return self._mat(3, (self.model.vocab, self.model.d_model))

    def layer(self, l):
        m = self.model
        d, f, hd = m.d_model, m.d_ff, m.n_heads * m.head_dim
        shapes = {"wq": (hd, d), "wk": (hd, d), "wv": (hd, d), "wo": (d, hd),
                  "wgate": (f, d), "wup": (f, d), "wdown": (d, f)}
        out = {}
        for k, name in enumerate(_LAYER_TENSORS):
            tid = 16 * (l + 1) + k
            out[name] = self._gain(tid, d) if name.startswith("norm") else self._mat(tid, shapes[name], name)
        return out


def prefix_tokens(wl):
    """S shared-prefix token ids, uniform over the vocabulary."""
    g = np.random.Generator(np.random.Philox(key=[np.uint64(wl.seed + 1), np.uint64(0)]))
    return g.integers(0, wl.model.vocab, size=wl.S, dtype=np.int64).astype(np.int32)


def private_tokens(wl):
    """[N][R] branch-private context token ids (true-prefix protocol only)."""
    g = np.random.Generator(np.random.Philox(key=[np.uint64(wl.seed + 1), np.uint64(1)]))
    return g.integers(0, wl.model.vocab, size=(wl.N, wl.R), dtype=np.int64).astype(np.int32)


def pending_tokens(wl):
    """[N] last validated token of each branch (its KV is not yet cached)."""
    g = np.random.Generator(np.random.Philox(key=[np.uint64(wl.seed + 1), np.uint64(2)]))
    return g.integers(0, wl.model.vocab, size=wl.N, dtype=np.int64).astype(np.int32)


def private_lens(wl):
    """[N] valid tokens of each branch's private context: all R, or seeded in [R_min, R] for ragged workloads
    (then branch 0 gets R_min and branch N-1 gets R, so both ends occur)."""
    if wl.R_min < 0 or wl.R_min >= wl.R:
        return np.full(wl.N, wl.R, np.int32)
    g = np.random.Generator(np.random.Philox(key=[np.uint64(wl.seed + 1), np.uint64(3)]))
    lens = g.integers(wl.R_min, wl.R + 1, size=wl.N, dtype=np.int64).astype(np.int32)
    lens[0] = wl.R_min
    lens[-1] = wl.R
    return lens


def synthetic_kv(wl, layer):
    """Synthetic-KV protocol: post-RoPE K and V ~ N(0,1) for the shared prefix [H][S][dh] and the
    private contexts [N][H][R][dh] of one layer, on the storage grid of the model dtype."""
    m = wl.model
    bf16 = m.dtype != "fp32"
    H, dh = m.n_heads, m.head_dim
    base = 1000 + 4 * layer
    ks = normal_tensor(wl.seed + 1, base + 0, (H, wl.S, dh), 1.0, 0.0, bf16) if wl.S else \
        np.zeros((H, 0, dh), np.float32)
    vs = normal_tensor(wl.seed + 1, base + 1, (H, wl.S, dh), 1.0, 0.0, bf16) if wl.S else \
        np.zeros((H, 0, dh), np.float32)
    kp = normal_tensor(wl.seed + 1, base + 2, (wl.N, H, wl.R, dh), 1.0, 0.0, bf16) if wl.R else \
        np.zeros((wl.N, H, 0, dh), np.float32)
    vp = normal_tensor(wl.seed + 1, base + 3, (wl.N, H, wl.R, dh), 1.0, 0.0, bf16) if wl.R else \
        np.zeros((wl.N, H, 0, dh), np.float32)
    return ks, vs, kp, vp


def _softmax64(z):
    z = z.astype(np.float64)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def random_draft_q(wl):
    """Draft distributions q[N][gamma][V] = softmax(z / q_temp), z ~ N(0,1) iid, as float32."""
    z = normal_tensor(wl.seed + 2, 1, (wl.N, wl.gamma, wl.model.vocab), 1.0)
    return _softmax64(z / np.float32(wl.q_temp)).astype(np.float32)


def perturbed_draft_q(wl, target_logits_row, b, j):
    """q for (branch b, draft position j) = softmax((target logits + N(0, noise_std^2)) / q_temp)."""
    eps = normal_tensor(wl.seed + 2, 2 + b * 64 + j, (wl.model.vocab,), wl.q_noise_std)
    return _softmax64((np.asarray(target_logits_row, np.float32) + eps) / np.float32(wl.q_temp)).astype(np.float32)


def draw_tokens(q, u):
    """Generic inverse-CDF draw (float64 cumulative sum + searchsorted) used only to manufacture
    draft tokens that are distributed like q; not the library's fixed-point sampler."""
    q = np.asarray(q, np.float64)
    flat = q.reshape(-1, q.shape[-1])
    uu = np.asarray(u, np.float64).reshape(-1)
    out = np.empty(flat.shape[0], np.int32)
    for i in range(flat.shape[0]):
        c = np.cumsum(flat[i])
        out[i] = min(int(np.searchsorted(c, uu[i] * c[-1], side="right")), flat.shape[1] - 1)
    return out.reshape(q.shape[:-1])
