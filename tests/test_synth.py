"""The seeded generators: determinism, distribution, and the reference builder's overlap."""
import numpy as np

import synth


def _mix64(x):
    m = (1 << 64) - 1
    x ^= x >> 30; x = (x * 0xBF58476D1CE4E5B9) & m
    x ^= x >> 27; x = (x * 0x94D049BB133111EB) & m
    x ^= x >> 31
    return x


def test_counter_based_words_match_python_reimplementation():
    seed, stream, V = 42, 10, 32000
    key = _mix64(seed ^ _mix64((stream + 0x632BE59BD9B4E019) & ((1 << 64) - 1)))
    want = [((_mix64((key + (i + 1) * 0x9E3779B97F4A7C15) & ((1 << 64) - 1)) >> 32) * V) >> 32 for i in range(50)]
    assert synth.uniform_tokens(seed, stream, 50, V).tolist() == want


def test_determinism_and_prefix_property():
    a = synth.normal_bf16(1, 2, 0.02, 1001)
    b = synth.normal_bf16(1, 2, 0.02, 5000)
    assert np.array_equal(a, b[:1001])                       # element i depends on (seed, stream, i) only
    assert not np.array_equal(a, synth.normal_bf16(1, 3, 0.02, 1001))
    assert not np.array_equal(a, synth.normal_bf16(2, 2, 0.02, 1001))


def test_gaussian_moments_and_bf16_rounding():
    x = synth.normal_f32(7, 1, 0.02, 400000).astype(np.float64)
    assert abs(x.mean()) < 2e-4 and abs(x.std() - 0.02) < 2e-4
    assert abs(np.mean(np.abs(x) > 0.04) - 0.0455) < 0.003  # two-sigma tail
    b = synth.bf16_to_f32(synth.normal_bf16(7, 1, 0.02, 400000)).astype(np.float64)
    assert np.all(np.abs(b - x) <= np.abs(x) * 2.0 ** -8)    # half ulp of an 8-bit significand
    assert np.array_equal(synth.f32_to_bf16(x.astype(np.float32)), synth.normal_bf16(7, 1, 0.02, 400000))


def test_weights_shapes_and_dtypes():
    w = synth.make_weights(synth.TINY, 1)
    assert w["embed"].dtype == np.float32 and w["embed"].shape == (512, 128)
    assert w["layers"][1]["wgu"].shape == (1024, 128) and w["layers"][0]["wd"].shape == (128, 512)
    assert np.all(w["final_norm"] == 1.0)
    w = synth.make_weights(synth.SMALL, 1, n_layers=1)
    assert w["layers"][0]["wqkv"].dtype == np.uint16 and w["layers"][0]["wqkv"].shape == (1536, 512)
    assert synth.LLAMA_7B.streamed_params == 6_607_077_376
    assert synth.LLAMA_13B.streamed_params == 12_851_609_600


def test_make_ref_overlap_and_spans():
    y = synth.uniform_tokens(5, 1, 4000, 32000)
    ref, spans = synth.make_ref(y, 0.5, 12.0, 6000, 32000, seed=3)
    assert len(ref) == 6000
    covered = sum(l for _, _, l in spans)
    assert 0.42 < covered / len(y) < 0.58
    assert 9 < covered / len(spans) < 15
    for rs, ys, l in spans:
        assert np.array_equal(ref[rs:rs + l], y[ys:ys + l])
    ref2, _ = synth.make_ref(y, 0.5, 12.0, 6000, 32000, seed=3)
    assert np.array_equal(ref, ref2)


def test_tiny_reference_recipe():
    wl = synth.WORKLOADS["tiny"]
    y = synth.uniform_tokens(9, 1, 32, 512)
    ref, offs = synth.build_reference(wl, y)
    assert len(ref) == 48 and offs.tolist() == [0, 48]
    assert int(np.sum(ref[:32] != y)) in (5, 6)               # 6 replaced (a replacement may repeat the old id)
    wl7 = synth.WORKLOADS["7b"]
    y = synth.uniform_tokens(9, 2, 256, 32000)
    ref, offs = synth.build_reference(wl7, y)
    assert len(ref) == 1472 and offs.tolist() == [0, 491, 982, 1472]


def test_cache_assisted_reference_recipe():
    """Four 'similar answers' of equal length outside the prompt, each with its own spans of the
    output; together they cover more of the output than one of them."""
    wl = synth.WORKLOADS["cag7b"]
    assert wl.prompt_len == 16 and wl.n_similar == 4
    y = synth.uniform_tokens(11, 3, wl.max_new, wl.model.vocab)
    ref, offs = synth.build_reference(wl, y)
    assert len(ref) == wl.ref_len and offs.tolist() == [0, 176, 352, 528, 704]
    docs = [ref[offs[i]:offs[i + 1]] for i in range(4)]
    assert all(not np.array_equal(docs[0], d) for d in docs[1:])
    def covered(ds):
        pos = set()
        yl = y.tolist()
        for d in ds:
            dl = d.tolist()
            for i in range(len(yl) - 3):           # output 4-grams that occur in the document
                g = yl[i:i + 4]
                if any(dl[j:j + 4] == g for j in range(len(dl) - 3)):
                    pos.update(range(i, i + 4))
        return len(pos) / len(yl)
    one, four = covered(docs[:1]), covered(docs)
    assert 0.15 < one < 0.75 and four > one
    ref2, offs2 = synth.build_reference(wl, y)
    assert np.array_equal(ref, ref2) and np.array_equal(offs, offs2)
