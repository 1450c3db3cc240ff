"""Pins for the oracle's transformer forward (CPU only).

The forward is checked against: closed forms (RMSNorm of a constant, one-key attention,
zeroed projections), invariants (RoPE is a rotation whose inner products depend on the
position difference only; cached multi-row forward == sequential single-row forwards;
dropping rejected rows == never having fed them), and an independent second opinion: the
same architecture written without a cache in PyTorch CPU float64 with library attention.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import OracleModel, CachedLLM, greedy_decode, llma_decode, infer_decoding_sequence
from oracle.model import rmsnorm, rope, silu, argmax_tokens, top2_gap

MINI = synth.ModelCfg("mini", 3, 64, 4, 16, 96, 97, "bf16")


def _model(cfg=MINI, seed=5, jitter=0.3, dtype=np.float64):
    return OracleModel(cfg, synth.make_weights(cfg, seed, gain_jitter=jitter), dtype)


# ------------------------------------------------------------------ primitives
def test_rmsnorm_constant_vector():
    x = np.full((2, 64), -3.0)
    out = rmsnorm(x, np.ones(64), 1e-6)
    assert np.allclose(out, -1.0, atol=1e-6)
    g = np.linspace(0.5, 2.0, 64)
    assert np.allclose(rmsnorm(x, g, 0.0), -g)


def test_silu_values():
    assert silu(np.array([0.0]))[0] == 0.0
    assert np.isclose(silu(np.array([1.0]))[0], 1.0 / (1.0 + np.exp(-1.0)))
    assert np.isclose(silu(np.array([-20.0]))[0], -20.0 * np.exp(-20.0), rtol=1e-6)


def test_rope_is_relative_rotation():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((1, 2, 32))
    k = rng.standard_normal((1, 2, 32))
    assert np.array_equal(rope(q, np.array([0]), 10000.0), q)                   # identity at 0
    for p in (1, 17, 900):
        assert np.allclose(np.linalg.norm(rope(q, np.array([p]), 10000.0), axis=-1),
                           np.linalg.norm(q, axis=-1))                          # norm preserved
    def ip(pq, pk):
        return np.sum(rope(q, np.array([pq]), 10000.0) * rope(k, np.array([pk]), 10000.0), axis=-1)
    assert np.allclose(ip(5, 2), ip(105, 102)) and np.allclose(ip(40, 40), ip(0, 0))
    assert not np.allclose(ip(5, 2), ip(5, 3))
    # explicit first pair, base frequency 1: (x0, x16) rotated by angle p
    x = np.zeros((1, 1, 32)); x[0, 0, 0] = 1.0
    r = rope(x, np.array([2]), 10000.0)
    assert np.isclose(r[0, 0, 0], np.cos(2.0)) and np.isclose(r[0, 0, 16], np.sin(2.0))
    # last pair: frequency theta^(-(d-2)/d)
    x = np.zeros((1, 1, 32)); x[0, 0, 15] = 1.0
    r = rope(x, np.array([3]), 10000.0)
    a = 3.0 * 10000.0 ** (-30.0 / 32.0)
    assert np.isclose(r[0, 0, 15], np.cos(a)) and np.isclose(r[0, 0, 31], np.sin(a))


# ------------------------------------------------------------------ closed forms of the whole forward
def test_zero_output_projections_closed_form():
    """With Wo = Wd = 0 every layer adds nothing: logits = RMSNorm(E[t]) Wlm^T."""
    w = synth.make_weights(MINI, 3, gain_jitter=0.3)
    for lw in w["layers"]:
        lw["wo"][:] = 0
        lw["wd"][:] = 0
    m = OracleModel(MINI, w)
    toks = [5, 9, 33]
    got = m.forward(toks, m.new_cache(8), 0)
    E = synth.bf16_to_f32(w["embed"]).astype(np.float64)
    Wl = synth.bf16_to_f32(w["lm_head"]).astype(np.float64)
    x = E[toks]
    want = (w["final_norm"] * x / np.sqrt((x ** 2).mean(-1, keepdims=True) + MINI.rms_eps)) @ Wl.T
    assert np.allclose(got, want, rtol=1e-12, atol=1e-14)


def test_single_position_attention_returns_value():
    """One token, empty cache: softmax over one key is 1, so attention output = v and
    h1 = h0 + Wo v, regardless of q, k and RoPE."""
    cfg = synth.ModelCfg("one", 1, 64, 4, 16, 96, 97, "bf16")
    w = synth.make_weights(cfg, 11, gain_jitter=0.3)
    lw = w["layers"][0]
    lw["wd"][:] = 0
    m = OracleModel(cfg, w)
    got = m.forward([7], m.new_cache(4), 0)
    f = lambda a: synth.bf16_to_f32(a).astype(np.float64)
    h0 = f(w["embed"])[7]
    u = lw["norm1"] * h0 / np.sqrt((h0 ** 2).mean() + cfg.rms_eps)
    v = f(lw["wqkv"])[2 * 64:3 * 64] @ u
    h1 = h0 + f(lw["wo"]) @ v
    want = (w["final_norm"] * h1 / np.sqrt((h1 ** 2).mean() + cfg.rms_eps)) @ f(w["lm_head"]).T
    assert np.allclose(got[0], want, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ cache / causality invariants
def test_multirow_equals_sequential_single_rows():
    m = _model()
    rng = np.random.default_rng(1)
    toks = rng.integers(0, MINI.vocab, 23).tolist()
    c1, c2 = m.new_cache(32), m.new_cache(32)
    seq = np.concatenate([m.forward([t], c1, i) for i, t in enumerate(toks)])
    a = m.forward(toks[:9], c2, 0)
    b = m.forward(toks[9:10], c2, 9)
    c = m.forward(toks[10:], c2, 10)
    assert np.allclose(np.concatenate([a, b, c]), seq, rtol=1e-9, atol=1e-11)
    for l in range(MINI.n_layers):
        assert np.allclose(c1.k[l][:, :23], c2.k[l][:, :23], atol=1e-12)
        assert np.allclose(c1.v[l][:, :23], c2.v[l][:, :23], atol=1e-12)


def test_later_rows_do_not_influence_earlier_rows():
    m = _model()
    toks = [1, 2, 3, 4, 5, 6]
    a = m.forward(toks, m.new_cache(8), 0)
    toks2 = toks[:3] + [90, 91, 92]
    b = m.forward(toks2, m.new_cache(8), 0)
    assert np.allclose(a[:3], b[:3], rtol=1e-11, atol=1e-13) and not np.allclose(a[3:], b[3:])


def test_truncation_equals_never_fed():
    """Feed 1+4 rows, keep only the first 2 (a = 1), then a plain step: logits equal those
    of a fresh cache that only ever saw the kept tokens."""
    m = _model()
    prompt = [4, 8, 15, 16, 23, 42]
    c = m.new_cache(32)
    m.forward(prompt, c, 0)
    m.forward([10, 11, 12, 13, 14], c, 6)              # rows 6..10; rows 8..10 are rejected
    after = m.forward([20], c, 8)
    c2 = m.new_cache(32)
    m.forward(prompt + [10, 11], c2, 0)
    fresh = m.forward([20], c2, 8)
    assert np.allclose(after, fresh, rtol=1e-11, atol=1e-13)    # BLAS blocking differs with row count


# ------------------------------------------------------------------ independent second opinion
def torch_reference_logits(cfg, w, tokens):
    """No cache, float64, library matmul / softmax-attention, HF-style rotate_half RoPE."""
    f = lambda a: torch.from_numpy(synth.bf16_to_f32(a) if a.dtype == np.uint16 else a).double()
    t = torch.tensor(tokens, dtype=torch.long)
    S, H, dh = len(tokens), cfg.n_heads, cfg.head_dim
    inv = 1.0 / (cfg.rope_theta ** (torch.arange(0, dh, 2, dtype=torch.float64) / dh))
    fr = torch.outer(torch.arange(S, dtype=torch.float64), inv)
    emb = torch.cat([fr, fr], dim=-1)
    cos, sin = emb.cos()[None], emb.sin()[None]           # [1,S,dh]

    def rot_half(x):
        return torch.cat([-x[..., dh // 2:], x[..., :dh // 2]], dim=-1)

    def norm(x, g):
        return f(g) * x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + cfg.rms_eps)

    h = f(w["embed"])[t]
    for lw in w["layers"]:
        u = norm(h, lw["norm1"])
        q, k, v = (u @ f(lw["wqkv"]).T).split(cfg.d_model, dim=-1)
        q = q.view(S, H, dh).transpose(0, 1)
        k = k.view(S, H, dh).transpose(0, 1)
        v = v.view(S, H, dh).transpose(0, 1)
        q = q * cos + rot_half(q) * sin
        k = k * cos + rot_half(k) * sin
        o = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        h = h + o.transpose(0, 1).reshape(S, cfg.d_model) @ f(lw["wo"]).T
        u = norm(h, lw["norm2"])
        g, up = (u @ f(lw["wgu"]).T).split(cfg.d_ffn, dim=-1)
        h = h + (torch.nn.functional.silu(g) * up) @ f(lw["wd"]).T
    return (norm(h, w["final_norm"]) @ f(w["lm_head"]).T).numpy()


@pytest.mark.parametrize("cfg", [MINI, synth.TINY], ids=["mini-bf16", "tiny-fp32"])
def test_against_uncached_torch_float64(cfg):
    w = synth.make_weights(cfg, 21, gain_jitter=0.25)
    toks = synth.uniform_tokens(3, 77, 40, cfg.vocab).tolist()
    m = OracleModel(cfg, w)
    c = m.new_cache(64)
    got = np.concatenate([m.forward(toks[:25], c, 0), m.forward(toks[25:], c, 25)])
    want = torch_reference_logits(cfg, w, toks)
    assert np.allclose(got, want, rtol=1e-9, atol=1e-11)


def test_small_config_two_layers_against_torch():
    """The 'small' benchmark shape (d_h = 64, vocab 32000), cut to 2 layers for speed."""
    cfg = synth.SMALL
    w = synth.make_weights(cfg, 2, n_layers=2)
    toks = synth.uniform_tokens(4, 78, 12, cfg.vocab).tolist()
    m = OracleModel(cfg, w)
    got = m.forward(toks, m.new_cache(16), 0)
    want = torch_reference_logits(cfg, w, toks)
    assert np.allclose(got, want, rtol=1e-9, atol=1e-11)


def test_float32_oracle_close_to_float64():
    w = synth.make_weights(MINI, 8)
    toks = list(range(1, 20))
    a = OracleModel(MINI, w, np.float64).forward(toks, OracleModel(MINI, w).new_cache(32), 0)
    m32 = OracleModel(MINI, w, np.float32)
    b = m32.forward(toks, m32.new_cache(32), 0)
    assert b.dtype == np.float32 and np.allclose(a, b, atol=2e-5)


# ------------------------------------------------------------------ the method on the real model
def test_llma_equals_greedy_on_transformer_and_trace_matches_prediction():
    cfg = synth.TINY
    w = synth.make_weights(cfg, 20230410)
    m = OracleModel(cfg, w)
    prompt = synth.uniform_tokens(1, 10, 24, cfg.vocab)
    N = 24
    y = greedy_decode(CachedLLM(m, prompt, 64), N)
    ref = synth.replace_positions(np.array(y), 0.2, cfg.vocab, 9)
    D = [ref.tolist(), synth.uniform_tokens(2, 12, 16, cfg.vocab).tolist()]
    for n, k in ((1, 4), (2, 3), (1, 16)):
        llm = CachedLLM(m, prompt, 64)
        y2, trace = llma_decode(llm, D, n, k, N)
        assert y2 == y
        assert trace == infer_decoding_sequence(y, D, n, k)
        assert sum(e for _, e, _, _ in trace) == N
        assert any(e > 1 for _, e, _, _ in trace)          # the reference really helps
        assert llm.rows_fed == len(prompt) - 1 + sum(r for r, _, _, _ in trace)


def test_argmax_lowest_index_on_ties():
    lg = np.array([[0.0, 3.0, 3.0, 1.0], [2.0, 2.0, 2.0, 2.0]])
    assert argmax_tokens(lg).tolist() == [1, 0]
    # a float64 difference below float32 resolution is a tie in the deciding precision
    lg = np.array([[1.0, 1.0 + 1e-12]])
    assert argmax_tokens(lg).tolist() == [0]


def test_top2_gap_hand_rows_and_sorted_definition():
    """top2_gap decides when a GPU / oracle token mismatch counts as a near-tie, so it is pinned
    on its own: hand rows (exact tie -> 0, the runner-up may sit before or after the maximum,
    negative rows, float32 input) and the definition via a full sort on random rows."""
    assert top2_gap(np.array([1.0, 5.0, 2.0, 4.5])) == 0.5
    assert top2_gap(np.array([4.5, 1.0, 5.0])) == 0.5
    assert top2_gap(np.array([3.0, 3.0, -1.0])) == 0.0
    assert top2_gap(np.array([7.0, 7.0])) == 0.0
    assert top2_gap(np.array([-9.0, -2.0, -2.25, -30.0])) == 0.25
    assert top2_gap(np.array([0.0, 1e-3], dtype=np.float32)) == pytest.approx(1e-3, rel=1e-6)
    assert top2_gap(np.array([1.0, 1.0 + 1e-12])) == pytest.approx(1e-12, rel=1e-3)    # no rounding to float32 here
    rng = np.random.default_rng(5)
    for n in (2, 3, 17, 32000):
        for _ in range(20):
            row = rng.standard_normal(n) * 1.3
            if n > 3:
                row[rng.integers(n)] = row.max() - rng.random() * 1e-3               # a close runner-up
            srt = np.sort(row)
            assert top2_gap(row) == pytest.approx(srt[-1] - srt[-2], abs=1e-15)
            assert top2_gap(row) >= 0.0


def test_layers_widened_on_demand_give_identical_logits():
    """lazy=True only moves the exact bf16 -> float conversion into forward()."""
    w = synth.make_weights(MINI, 31, gain_jitter=0.2)
    toks = list(range(3, 30))
    a, b = OracleModel(MINI, w, np.float32), OracleModel(MINI, w, np.float32, lazy=True)
    ca, cb = a.new_cache(40), b.new_cache(40)
    assert len(cb.k) == MINI.n_layers
    for T0, T1 in ((0, 20), (20, 27)):
        assert np.array_equal(a.forward(toks[T0:T1], ca, T0), b.forward(toks[T0:T1], cb, T0))
