"""CPU oracle: the decoder-only transformer whose next-token argmax is the paper's LLM(.).

TEST INFRASTRUCTURE ONLY.  Plain numpy, no blocking or fusion, written so it can be
checked against the definitions by eye.  Nothing in the product path may import this
package; it shares no code with the HIP implementation.

The paper treats the model as a black box that maps a token prefix to the most probable
next token (Method, Eq. 2 and Eq. 3).  The architecture here is the LLaMA-style one the
benchmark configurations fix: RMSNorm, rotary position embedding, causal multi-head
attention with a key/value cache, SwiGLU feed-forward, no biases, untied input embedding
and output head.

Arithmetic precision is a constructor argument: float64 by default (every pin and every
small-configuration parity test), float32 permitted for the 7B/13B shapes where float64
copies of the weights would not fit in host memory.  The arg-max decision is always taken
on logits rounded to float32, lowest token id winning exact ties, because that is the
precision the GPU path decides in.

Where even float32 copies do not fit (the 13B shape: 51 GB), `lazy=True` keeps the layers'
matrices in the form they arrive in (bfloat16 bit patterns) and widens one layer at a time
inside forward(); the arithmetic is the same, only the moment of the (exact) format
conversion differs.
"""
from __future__ import annotations

import numpy as np


def _widen(a: np.ndarray, dtype) -> np.ndarray:
    """Weights arrive as float32 or as bfloat16 bit patterns (uint16); both widen exactly."""
    if a.dtype == np.uint16:
        # the 16 stored bits are the upper half of the float32 pattern
        return np.left_shift(a, 16, dtype=np.uint32, casting="unsafe").view(np.float32).astype(dtype, copy=False)
    return a.astype(dtype)


class _LayersWidenedOnDemand:
    """The per-layer weight dicts of a model whose matrices stay in their storage format;
    iterating yields one layer at a time, widened to the arithmetic dtype.  The widened
    matrices of consecutive layers share one set of buffers (same shapes), so a yielded
    layer is only valid until the next one is asked for -- which is how forward() uses it."""

    def __init__(self, raw_layers, dtype):
        self.raw, self.dtype = raw_layers, dtype
        self.buf = {}

    def __len__(self):
        return len(self.raw)

    def _widen_into_buffer(self, name, a):
        if a.dtype != np.uint16 or self.dtype != np.float32:
            return _widen(a, self.dtype)
        b = self.buf.get(name)
        if b is None or b.shape != a.shape:
            b = self.buf[name] = np.empty(a.shape, dtype=np.float32)
        np.left_shift(a, 16, out=b.view(np.uint32), dtype=np.uint32, casting="unsafe")   # same exact widening as _widen
        return b

    def __iter__(self):
        for lw in self.raw:
            yield {k: (self._widen_into_buffer(k, v) if v.ndim == 2 else v.astype(self.dtype)) for k, v in lw.items()}


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """RMSNorm(x; g) = g * x / sqrt(mean(x^2) + eps), per row."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return g * x / np.sqrt(ms + eps)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding.  x: [rows, heads, d_h]; pos: [rows] absolute positions.
    Feature i (i < d_h/2) is paired with i + d_h/2 and the pair is rotated by the angle
    pos * theta^(-2i/d_h)."""
    half = x.shape[-1] // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / x.shape[-1])
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]        # [rows, half]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


class KVCache:
    """Keys (already rotated) and values per layer: [layers][heads, capacity, d_h]."""

    def __init__(self, n_layers, n_heads, capacity, head_dim, dtype):
        self.k = [np.zeros((n_heads, capacity, head_dim), dtype=dtype) for _ in range(n_layers)]
        self.v = [np.zeros((n_heads, capacity, head_dim), dtype=dtype) for _ in range(n_layers)]
        self.capacity = capacity


class OracleModel:
    def __init__(self, cfg, weights: dict, dtype=np.float64, lazy: bool = False):
        self.cfg = cfg
        self.dtype = dtype
        self.embed = _widen(weights["embed"], dtype)
        self.lm_head = _widen(weights["lm_head"], dtype)
        self.final_norm = weights["final_norm"].astype(dtype)
        if lazy:
            self.layers = _LayersWidenedOnDemand(weights["layers"], dtype)
        else:
            self.layers = [{k: (_widen(v, dtype) if v.ndim == 2 else v.astype(dtype)) for k, v in lw.items()}
                           for lw in weights["layers"]]

    def new_cache(self, capacity: int) -> KVCache:
        c = self.cfg
        return KVCache(len(self.layers), c.n_heads, capacity, c.head_dim, self.dtype)

    def forward(self, tokens, cache: KVCache, T: int) -> np.ndarray:
        """Feed `tokens` (m ids) at absolute positions T..T+m-1 on top of the T cached
        positions.  Returns logits [m, vocab]: row j is the next-token distribution's
        logits given everything up to and including tokens[j] (Eq. 3: all k+1 outputs of
        one step come from one causal forward).  Cache rows T..T+m-1 are (over)written."""
        c = self.cfg
        tokens = np.asarray(tokens, dtype=np.int64)
        m = len(tokens)
        H, dh, d = c.n_heads, c.head_dim, c.d_model
        pos = np.arange(T, T + m)
        h = self.embed[tokens]                                          # [m, d]
        for l, w in enumerate(self.layers):
            u = rmsnorm(h, w["norm1"], c.rms_eps)
            qkv = u @ w["wqkv"].T                                       # [m, 3d]
            q = rope(qkv[:, 0 * d:1 * d].reshape(m, H, dh), pos, c.rope_theta)
            k = rope(qkv[:, 1 * d:2 * d].reshape(m, H, dh), pos, c.rope_theta)
            v = qkv[:, 2 * d:3 * d].reshape(m, H, dh)
            cache.k[l][:, T:T + m, :] = k.transpose(1, 0, 2)
            cache.v[l][:, T:T + m, :] = v.transpose(1, 0, 2)
            keys = cache.k[l][:, :T + m, :]                             # [H, T+m, dh]
            vals = cache.v[l][:, :T + m, :]
            s = np.matmul(q.transpose(1, 0, 2), keys.transpose(0, 2, 1)) / np.sqrt(self.dtype(dh))
            # causal validity: row j (position T+j) sees cache rows 0..T+j only
            visible = np.arange(T + m)[None, :] <= pos[:, None]         # [m, T+m]
            s = np.where(visible[None, :, :], s, -np.inf)
            s = s - np.max(s, axis=-1, keepdims=True)
            p = np.exp(s)
            p = p / np.sum(p, axis=-1, keepdims=True)
            o = np.matmul(p, vals)                                      # [H, m, dh]
            h = h + o.transpose(1, 0, 2).reshape(m, d) @ w["wo"].T
            u = rmsnorm(h, w["norm2"], c.rms_eps)
            gu = u @ w["wgu"].T                                         # [m, 2F]
            a = silu(gu[:, :c.d_ffn]) * gu[:, c.d_ffn:]
            h = h + a @ w["wd"].T
        return rmsnorm(h, self.final_norm, c.rms_eps) @ self.lm_head.T


def argmax_tokens(logits: np.ndarray) -> np.ndarray:
    """Per-row arg max over the vocabulary on float32-rounded logits; lowest id on ties."""
    return np.argmax(logits.astype(np.float32), axis=-1).astype(np.int32)


def top2_gap(logits_row: np.ndarray) -> float:
    """Difference between the largest and second largest logit of one row."""
    part = np.partition(logits_row.astype(np.float64), -2)
    return float(part[-1] - part[-2])
