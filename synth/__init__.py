"""Seeded synthetic inputs (weights, token ids, references, KV fill).

This package serves BOTH the CPU oracle's tests and the GPU path's tests / bench, and
therefore contains none of the decoding method's arithmetic: no transformer math, no
n-gram matching, no accept logic.  It only draws pseudo-random numbers from a
counter-based generator (see gen.c) and arranges them into the shapes of the
workloads (model weights, prompts, reference documents with a chosen overlap
with a GIVEN output sequence).
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libsynthgen.so")


def build(force: bool = False) -> str:
    """Compile gen.c with gcc (host only) into libsynthgen.so next to it."""
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _SO, src, "-lm"])
    return _SO


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_SO)
        u64, dbl, sz = ctypes.c_uint64, ctypes.c_double, ctypes.c_size_t
        lib.synth_normal_f32.argtypes = [u64, u64, dbl, ctypes.c_void_p, sz]
        lib.synth_normal_bf16.argtypes = [u64, u64, dbl, ctypes.c_void_p, sz]
        lib.synth_uniform_i32.argtypes = [u64, u64, ctypes.c_int32, ctypes.c_void_p, sz]
        lib.synth_uniform_f64.argtypes = [u64, u64, ctypes.c_void_p, sz]
        for f in (lib.synth_normal_f32, lib.synth_normal_bf16, lib.synth_uniform_i32,
                  lib.synth_uniform_f64):
            f.restype = None
        _lib = lib
    return _lib


# ----------------------------------------------------------------------------- raw draws
def normal_f32(seed: int, stream: int, sigma: float, shape) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().synth_normal_f32(seed, stream, sigma, out.ctypes.data, out.size)
    return out


def normal_bf16(seed: int, stream: int, sigma: float, shape) -> np.ndarray:
    """bfloat16 bit patterns as uint16 (round-to-nearest-even of the float draw)."""
    out = np.empty(shape, dtype=np.uint16)
    _load().synth_normal_bf16(seed, stream, sigma, out.ctypes.data, out.size)
    return out


def uniform_tokens(seed: int, stream: int, n: int, vocab: int) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    _load().synth_uniform_i32(seed, stream, vocab, out.ctypes.data, out.size)
    return out


def uniform_f64(seed: int, stream: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.float64)
    _load().synth_uniform_f64(seed, stream, out.ctypes.data, out.size)
    return out


def bf16_to_f32(u16: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (u16.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16(f32: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 bit patterns (uint16), nearest-even (a format
    conversion for handing identical KV / activation fill to both sides)."""
    u = np.ascontiguousarray(f32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


# ----------------------------------------------------------------------------- model shapes
@dataclass(frozen=True)
class ModelCfg:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str            # "fp32" or "bf16": storage type of the matrices
    rms_eps: float = 1e-6
    rope_theta: float = 10000.0

    @property
    def streamed_params(self) -> int:
        """Matrix elements read once per decoding step (layers + LM head; the
        embedding table is only gathered)."""
        d, f = self.d_model, self.d_ffn
        per_layer = 3 * d * d + d * d + 2 * f * d + d * f
        return self.n_layers * per_layer + self.vocab * d


TINY = ModelCfg("tiny", 2, 128, 4, 32, 512, 512, "fp32")
SMALL = ModelCfg("small", 6, 512, 8, 64, 2048, 32000, "bf16")
LLAMA_7B = ModelCfg("7b", 32, 4096, 32, 128, 11008, 32000, "bf16")
LLAMA_13B = ModelCfg("13b", 40, 5120, 40, 128, 13824, 32000, "bf16")
MODEL_CFGS = {c.name: c for c in (TINY, SMALL, LLAMA_7B, LLAMA_13B)}

# stream ids (disjoint by construction)
_S_EMBED, _S_LMHEAD, _S_FNORM = 1, 2, 3
_S_PROMPT, _S_REF_STRUCT, _S_REF_NOISE, _S_KV, _S_MISC = 10, 11, 12, 13, 14
_S_LAYER0 = 1000          # layer l, matrix j -> _S_LAYER0 + 16*l + j


def _matrix(cfg: ModelCfg, seed: int, stream: int, shape, sigma=0.02) -> np.ndarray:
    if cfg.dtype == "bf16":
        return normal_bf16(seed, stream, sigma, shape)
    return normal_f32(seed, stream, sigma, shape)


def _gain(seed: int, stream: int, d: int, jitter: float) -> np.ndarray:
    g = np.ones(d, dtype=np.float32)
    if jitter:
        g += (jitter * (2.0 * uniform_f64(seed, stream, d) - 1.0)).astype(np.float32)
    return g


def make_weights(cfg: ModelCfg, seed: int, gain_jitter: float = 0.0, n_layers: int | None = None) -> dict:
    """All matrices ~ N(0, 0.02^2); norm gains 1.0 (optionally jittered for tests that
    need to see the gains).  Matrices are uint16 bf16 patterns for dtype "bf16", float32
    otherwise.  Row-major [out_features, in_features]:
      wqkv [3d, d] (q rows, then k rows, then v rows), wo [d, d],
      wgu [2F, d] (gate rows, then up rows), wd [d, F], embed [V, d], lm_head [V, d]."""
    d, f, v = cfg.d_model, cfg.d_ffn, cfg.vocab
    nl = cfg.n_layers if n_layers is None else n_layers
    w = {
        "embed": _matrix(cfg, seed, _S_EMBED, (v, d)),
        "lm_head": _matrix(cfg, seed, _S_LMHEAD, (v, d)),
        "final_norm": _gain(seed, _S_FNORM, d, gain_jitter),
        "layers": [],
    }
    for l in range(nl):
        s = _S_LAYER0 + 16 * l
        w["layers"].append({
            "wqkv": _matrix(cfg, seed, s + 0, (3 * d, d)),
            "wo": _matrix(cfg, seed, s + 1, (d, d)),
            "wgu": _matrix(cfg, seed, s + 2, (2 * f, d)),
            "wd": _matrix(cfg, seed, s + 3, (d, f)),
            "norm1": _gain(seed, s + 4, d, gain_jitter),
            "norm2": _gain(seed, s + 5, d, gain_jitter),
        })
    return w


def make_kv_fill(cfg: ModelCfg, seed: int, n_seqs: int, length: int, layer: int):
    """iid N(0,1) K and V entries for one layer, bf16 patterns, plain layout
    [n_seqs, n_heads, length, head_dim] (verify-step microbenchmark workload)."""
    shape = (n_seqs, cfg.n_heads, length, cfg.head_dim)
    k = normal_bf16(seed, _S_KV + 100 * (2 * layer), 1.0, shape)
    v = normal_bf16(seed, _S_KV + 100 * (2 * layer + 1), 1.0, shape)
    return k, v


# ----------------------------------------------------------------------------- references
def _geometric(u: float, mean: float) -> int:
    """Geometric on {1,2,...} with the given mean (inverse CDF)."""
    if mean <= 1.0:
        return 1
    p = 1.0 / mean
    return 1 + int(math.floor(math.log1p(-u) / math.log1p(-p)))


def make_ref(y: np.ndarray, overlap: float, mean_span: float, length: int, vocab: int,
             seed: int, spread: bool = True):
    """Build `length` reference token ids that share spans with the GIVEN output `y`.

    Walk y alternating copied spans (length ~ Geometric(mean_span)) and gaps
    (length ~ Geometric(mean_span*(1-overlap)/overlap)), so that a fraction `overlap`
    of y's positions is covered by copied spans.  A span [a,b) contributes y[a:b]; a gap
    contributes as many uniform-random ids.  The remaining length-len(walk) positions are
    uniform-random ids, placed at the end (spread=False) or split between the segments at
    seeded random points (spread=True), so spans land in different documents.
    Returns (ref int32[length], spans) with spans = [(ref_start, y_start, len), ...]."""
    y = np.asarray(y, dtype=np.int32)
    us = uniform_f64(seed, _S_REF_STRUCT, 4 * len(y) + 16)
    noise = uniform_tokens(seed, _S_REF_NOISE, length + len(y) + 16, vocab)
    ui = 0
    ni = 0
    segs = []                      # (kind, y_start, len)
    pos = 0
    gap_mean = mean_span * (1.0 - overlap) / overlap if overlap > 0 else float("inf")
    in_span = bool(us[ui] < overlap) if 0 < overlap < 1 else overlap >= 1
    ui += 1
    while pos < len(y):
        if in_span:
            ln = _geometric(us[ui], mean_span)
        else:
            ln = len(y) if math.isinf(gap_mean) else _geometric(us[ui], gap_mean)
        ui += 1
        ln = min(ln, len(y) - pos)
        segs.append(("span" if in_span else "gap", pos, ln))
        pos += ln
        if 0 < overlap < 1:
            in_span = not in_span
    walk_len = sum(s[2] for s in segs)
    pad = max(0, length - walk_len)
    # how the padding is split between the len(segs)+1 slots
    if spread and pad > 0:
        cuts = np.sort((us[ui:ui + len(segs)] * (pad + 1)).astype(np.int64))
        ui += len(segs)
        pads = np.diff(np.concatenate([[0], cuts, [pad]])).tolist()
    else:
        pads = [0] * len(segs) + [pad]
    out = []
    spans = []
    for i, (kind, ys, ln) in enumerate(segs):
        if pads[i]:
            out.append(noise[ni:ni + pads[i]]); ni += pads[i]
        start = sum(len(o) for o in out)
        if kind == "span":
            out.append(y[ys:ys + ln])
            spans.append((start, ys, ln))
        else:
            out.append(noise[ni:ni + ln]); ni += ln
    if pads[-1]:
        out.append(noise[ni:ni + pads[-1]]); ni += pads[-1]
    ref = np.concatenate(out).astype(np.int32) if out else np.zeros(0, np.int32)
    ref = ref[:length]
    spans = [(s, a, min(l, length - s)) for (s, a, l) in spans if s < length]
    return ref, spans


def replace_positions(y: np.ndarray, frac: float, vocab: int, seed: int) -> np.ndarray:
    """Copy of y with exactly round(frac*len(y)) distinct seeded positions replaced by
    uniform-random ids (tiny-config reference recipe)."""
    y = np.asarray(y, dtype=np.int32).copy()
    cnt = int(round(frac * len(y)))
    order = np.argsort(uniform_f64(seed, _S_REF_STRUCT + 1, len(y)), kind="stable")
    new = uniform_tokens(seed, _S_REF_NOISE + 1, len(y), vocab)
    for p in order[:cnt]:
        y[p] = new[p]
    return y


def split_docs(ref: np.ndarray, cuts) -> np.ndarray:
    """doc_offsets int32[n_docs+1] for a flat reference cut at the given positions."""
    return np.asarray([0, *cuts, len(ref)], dtype=np.int32)


# ----------------------------------------------------------------------------- workloads
@dataclass(frozen=True)
class Workload:
    """One of the five benchmark configurations (shapes only; y-dependent parts are built
    by `build_reference` once an output sequence is known)."""
    name: str
    model: ModelCfg
    prompt_len: int
    ref_len: int
    n: int
    k: int
    max_new: int
    overlap: float
    mean_span: float
    doc_cuts: tuple = ()
    seed: int = 20230410
    k_sweep: tuple = field(default_factory=tuple)
    n_similar: int = 0      # > 0: the reference is this many separate "similar answers", each built
                            #      from the output on its own (cache-assisted scenario), ref_len in total


WORKLOADS = {
    "tiny": Workload("tiny", TINY, 64, 48, n=1, k=4, max_new=32, overlap=0.8, mean_span=0.0),
    "small": Workload("small", SMALL, 512, 384, n=2, k=8, max_new=128, overlap=0.6, mean_span=12.0),
    "7b": Workload("7b", LLAMA_7B, 1536, 1472, n=1, k=8, max_new=256, overlap=0.5, mean_span=12.0,
                   doc_cuts=(491, 982), k_sweep=(1, 4, 8, 16)),
    "13b": Workload("13b", LLAMA_13B, 2048, 512, n=2, k=16, max_new=512, overlap=0.8, mean_span=12.0),
    # cache-assisted scenario (paper: Experiments, the cache-assisted setting): a short query, the
    # reference = 4 earlier answers to similar queries, held outside the prompt
    "cag_small": Workload("cag_small", SMALL, 16, 4 * 96, n=1, k=8, max_new=96, overlap=0.5, mean_span=10.0, n_similar=4),
    "cag7b": Workload("cag7b", LLAMA_7B, 16, 4 * 176, n=1, k=8, max_new=176, overlap=0.5, mean_span=12.0,
                      k_sweep=(4, 8, 16), n_similar=4),
}


def make_prompt(wl: Workload) -> np.ndarray:
    """Uniform-random prompt ids of the configured length.  The slot where the reference
    text would sit holds uniform filler: the reference itself is handed to the decoder as a
    separate argument (cache-assisted style), which keeps prompt/KV length exact and breaks
    the circular definition 'reference built from the output of a prompt containing it'."""
    return uniform_tokens(wl.seed, _S_PROMPT, wl.prompt_len, wl.model.vocab)


def build_reference(wl: Workload, y: np.ndarray):
    """Reference documents for workload `wl` given an output sequence y (len == max_new).
    Returns (ref int32[ref_len], doc_offsets int32[n_docs+1])."""
    if wl.name == "tiny":
        body = replace_positions(y, 1.0 - wl.overlap, wl.model.vocab, wl.seed)
        pad = uniform_tokens(wl.seed, _S_REF_NOISE + 2, wl.ref_len - len(body), wl.model.vocab)
        ref = np.concatenate([body, pad]).astype(np.int32)
    elif wl.n_similar > 0:
        # each "similar answer" copies its own random spans of the output (a different seed per
        # document), so a span missing from one document may be present in another
        per = wl.ref_len // wl.n_similar
        docs = [make_ref(y, wl.overlap, wl.mean_span, per, wl.model.vocab, wl.seed + 7919 * (i + 1))[0]
                for i in range(wl.n_similar)]
        ref = np.concatenate(docs).astype(np.int32)
        return ref, np.arange(0, wl.n_similar + 1, dtype=np.int32) * per
    else:
        ref, _ = make_ref(y, wl.overlap, wl.mean_span, wl.ref_len, wl.model.vocab, wl.seed)
    return ref, split_docs(ref, wl.doc_cuts)
