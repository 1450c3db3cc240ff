"""Pins for the oracle's trigger, LLMA loop and step-sequence predictor (CPU only).

Each pin checks oracle/decode.py against something other than itself: an exhaustive
search written a different way (byte-string find), closed forms for scripted targets,
the worked example from the paper's illustration, and the invariants the paper states
(identical output to greedy; 1..k+1 tokens per step; accepted + steps = output tokens).
"""
import itertools
import math
import os
import random

import pytest

from oracle import (ScriptedLLM, greedy_decode, match_ngrams, llma_decode, copy_length,
                    infer_decoding_sequence, get_matched_tokens)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ independent brute force
def brute_trigger(y, D, n):
    """All occurrences via bytes.find (library substring search), scored by reversing both
    sides and taking os.path.commonprefix (library common-prefix) -- no code shared with
    match_ngrams."""
    if n < 1 or len(y) < n:
        return (False, -1, -1)
    yb = bytes(y)
    tail = yb[-n:]
    cands = []
    for di, d in enumerate(D):
        db = bytes(d)
        start = 0
        while True:
            f = db.find(tail, start)
            if f < 0:
                break
            pos = f + n
            if pos < len(db):                       # something left to copy
                suf = len(os.path.commonprefix([db[:pos][::-1], yb[::-1]]))
                cands.append((-suf, di, pos))
            start = f + 1
    if not cands:
        return (False, -1, -1)
    _, di, pos = min(cands)
    return (True, di, pos)


def test_matcher_exhaustive_tiny():
    """Every y of length <= 5 and every single document of length <= 5 over 2 symbols,
    n in 1..3: 2^5*2^5*... small enough to enumerate."""
    checked = 0
    for ly in range(0, 6):
        for y in itertools.product(range(2), repeat=ly):
            for ld in range(0, 6):
                for d in itertools.product(range(2), repeat=ld):
                    for n in (1, 2, 3):
                        assert match_ngrams(list(y), [list(d)], n) == brute_trigger(list(y), [list(d)], n)
                        checked += 1
    assert checked > 10000


def test_matcher_random_multidoc():
    rng = random.Random(7)
    for _ in range(3000):
        V = rng.choice([2, 3, 4])
        y = [rng.randrange(V) for _ in range(rng.randrange(0, 13))]
        D = [[rng.randrange(V) for _ in range(rng.randrange(0, 13))] for _ in range(rng.randrange(0, 4))]
        n = rng.choice([1, 2, 3])
        assert match_ngrams(y, D, n) == brute_trigger(y, D, n)


def test_matcher_special_cases():
    assert match_ngrams([1, 2], [], 1) == (False, -1, -1)                 # empty D
    assert match_ngrams([1], [[1, 2, 3]], 2) == (False, -1, -1)           # n > len(y)
    assert match_ngrams([], [[1, 2, 3]], 1) == (False, -1, -1)            # nothing generated yet
    assert match_ngrams([3], [[1, 2, 3]], 1) == (False, -1, -1)           # match only at doc end
    assert match_ngrams([2, 3], [[1, 2], [3, 4]], 2) == (False, -1, -1)   # straddles two docs
    assert match_ngrams([2], [[1, 2, 3]], 1) == (True, 0, 2)
    # longest backward agreement wins over the earlier position
    assert match_ngrams([7, 8, 9], [[0, 9, 1, 7, 8, 9, 2]], 1) == (True, 0, 6)
    # tie in backward agreement -> smallest doc, then smallest pos
    assert match_ngrams([9], [[5, 9, 1, 6, 9, 2], [9, 3]], 1) == (True, 0, 2)
    assert match_ngrams([9], [[4], [5, 9, 1], [6, 9, 2]], 1) == (True, 1, 2)


def test_copy_length_rule():
    d = list(range(10))
    assert copy_length(4, d, 3, 100, 0) == 4
    assert copy_length(4, d, 8, 100, 0) == 2          # document end
    assert copy_length(4, d, 3, 10, 7) == 2           # budget: 10-7-1
    assert copy_length(4, d, 3, 10, 9) == 0           # last token: plain step


# ------------------------------------------------------------------ worked example (paper figure)
def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [int(v) for v in vals]
    return out


def test_fig2_worked_example():
    g = _read_golden("fig2_worked_example.txt")
    n, k = g["n"][0], g["k"][0]
    llm = ScriptedLLM(g["target"])
    N = 2 + g["expected_step3_emitted"][0]
    y, trace = llma_decode(llm, [g["doc"]], n, k, N + 2)
    assert y[:len(g["target"])] == g["target"]
    assert trace[0] == (1, 1, -1, -1) and trace[1] == (1, 1, -1, -1)
    assert trace[2] == (g["expected_step3_rows_in"][0], g["expected_step3_emitted"][0], 0,
                        g["expected_match_pos"][0])
    assert y[2:2 + 6] == g["expected_step3_tokens"]


# ------------------------------------------------------------------ closed forms with scripted targets
@pytest.mark.parametrize("N,k", [(32, 4), (33, 4), (17, 1), (64, 16), (5, 8), (40, 7)])
def test_reference_equals_target_closed_form(N, k):
    """D = [y*] with distinct tokens, n = 1: the first step is plain (nothing generated yet),
    then every step copies from the aligned position and accepts every draft, so
    #steps = 1 + ceil((N-1)/(k+1))."""
    target = list(range(100, 100 + N))
    llm = ScriptedLLM(target)
    y, trace = llma_decode(llm, [target], 1, k, N)
    assert y == target
    assert len(trace) == 1 + math.ceil((N - 1) / (k + 1))
    assert all(e == r for r, e, _, _ in trace)                 # every fed row yields a token
    # every copying step starts at the aligned position (pos == number of tokens so far)
    assert all(pos == sum(e for _, e, _, _ in trace[:i]) for i, (_, _, di, pos) in enumerate(trace) if di >= 0)


def test_disjoint_reference_is_plain_greedy():
    target = list(range(50))
    llm = ScriptedLLM(target)
    y, trace = llma_decode(llm, [[1000 + i for i in range(30)]], 1, 8, 50)
    assert y == target
    assert trace == [(1, 1, -1, -1)] * 50
    assert llm.calls == [(i, 0) for i in range(50)]


def test_k0_and_empty_reference_reduce_to_greedy_step_for_step():
    target = [3, 1, 4, 1, 5, 9, 2, 6, 5, 3, 5, 8, 9, 7, 9]
    for D, k in (([], 4), ([target], 0)):
        llm = ScriptedLLM(target)
        y, trace = llma_decode(llm, D, 1, k, len(target))
        assert y == target and trace == [(1, 1, -1, -1)] * len(target)
        assert llm.calls == [(i, 0) for i in range(len(target))]


def _random_case(rng):
    V = rng.choice([3, 5, 50])
    N = rng.randrange(1, 40)
    target = [rng.randrange(V) for _ in range(N)]
    docs = []
    for _ in range(rng.randrange(0, 4)):
        kind = rng.randrange(4)
        if kind == 0:
            d = [rng.randrange(V) for _ in range(rng.randrange(0, 30))]
        elif kind == 1:
            a = rng.randrange(0, N)
            d = target[a:a + rng.randrange(1, 20)]
        elif kind == 2:
            d = [target[0]] * rng.randrange(1, 10)
        else:
            d = [t if rng.random() < 0.8 else rng.randrange(V) for t in target]
        docs.append(d)
    return target, docs, rng.choice([1, 2, 3]), rng.choice([0, 1, 2, 4, 8, 16])


def test_lossless_bounds_and_identities_random():
    """For arbitrary references: output identical to greedy; each step emits 1..k+1 tokens
    and never more than rows fed; sum(accepted) + #steps = N; exactly N tokens; the trace
    equals the model-free prediction computed from the greedy output."""
    rng = random.Random(1234)
    for _ in range(1500):
        target, D, n, k = _random_case(rng)
        N = len(target)
        assert greedy_decode(ScriptedLLM(target), N) == target
        llm = ScriptedLLM(target)
        y, trace = llma_decode(llm, D, n, k, N)
        assert y == target                                  # lossless, and filler never leaks
        assert len(y) == N
        done = 0
        for rows_in, emitted, di, pos in trace:
            assert 1 <= emitted <= rows_in <= k + 1
            if di < 0:
                assert rows_in == 1
            else:                                       # the n-token tail really sits before pos
                assert D[di][pos - n:pos] == target[done - n:done] and pos < len(D[di])
            done += emitted
        assert sum(e - 1 for _, e, _, _ in trace) + len(trace) == N
        assert trace == infer_decoding_sequence(target, D, n, k)
        # model calls are exactly the trace's rows
        assert [1 + c[1] for c in llm.calls] == [r for r, _, _, _ in trace]


def test_adversarial_references_lossless():
    target = [5, 5, 5, 1, 2, 3, 5, 5, 1, 2, 9, 9, 9, 9, 4, 5, 5, 5, 1, 2, 3, 7]
    N = len(target)
    cases = {
        "identical": [target],
        "shift_by_one": [target[1:] + [0]],
        "single_token": [[5] * 40],
        "reversed": [target[::-1]],
        "many_small": [target[i:i + 3] for i in range(0, N, 2)],
    }
    for name, D in cases.items():
        for n in (1, 2, 3):
            for k in (1, 3, 8, 32):
                y, trace = llma_decode(ScriptedLLM(target), D, n, k, N)
                assert y == target, (name, n, k)
                assert trace == infer_decoding_sequence(target, D, n, k)


def test_get_matched_tokens():
    assert get_matched_tokens([1, 2, 3, 4], 1, [9, 2, 3, 5], 1) == 2
    assert get_matched_tokens([1, 2, 3], 1, [2, 3], 0) == 2        # runs off both ends
    assert get_matched_tokens([1, 2, 3], 3, [2, 3], 0) == 0


def test_plain_steps_independent_of_k():
    """The paper's decoding statistics show #steps - #triggers (the steps that copy nothing)
    constant in k for fixed n (44.17 - 38.66 = 33.76 - 28.25 in its retrieval-augmented series).
    Reason: whether position i has a candidate depends on y[:i], D and n only, and a position that
    an accepted copy skips always has one (the span being copied), so the candidate-free positions
    are all step starts, whatever k.  Pinned here against the independent brute-force matcher:
    #plain steps == number of positions without a candidate, for every k and n.  (The document
    ends in a token the target never contains and the target ends in tokens the document never
    contains, so neither the end-of-document nor the output-budget cap turns a trigger into a
    plain step.)"""
    rng = random.Random(99)
    for trial in range(20):
        target = [rng.randrange(6) for _ in range(60)] + [7, 8]
        D = [[t if rng.random() < 0.7 else rng.randrange(6) for t in target[:60]] + [9]]
        for n in (1, 2, 3):
            free = sum(1 for i in range(len(target)) if not brute_trigger(target[:i], D, n)[0])
            counts = set()
            for k in (1, 4, 8, 16, 18):
                y, trace = llma_decode(ScriptedLLM(target), D, n, k, len(target))
                assert y == target
                plain = sum(1 for t in trace if t[2] < 0)
                assert plain == free, (trial, n, k, plain, free)
                counts.add(len(trace) - sum(1 for t in trace if t[2] >= 0))
            assert len(counts) == 1
            # and more copies never need more steps
            steps = [len(llma_decode(ScriptedLLM(target), D, n, k, len(target))[1]) for k in (1, 4, 8, 16)]
            assert steps == sorted(steps, reverse=True) and steps[0] > steps[-1]


def test_docs_from_flat():
    from oracle import docs_from_flat
    import numpy as np
    ref = np.arange(10, 20, dtype=np.int32)
    assert docs_from_flat(ref, [0, 3, 3, 10]) == [[10, 11, 12], [], [13, 14, 15, 16, 17, 18, 19]]
    assert docs_from_flat(ref, [0, 10]) == [ref.tolist()]
    assert docs_from_flat(ref[:0], [0]) == []
    D = docs_from_flat(ref, np.asarray([0, 4, 9, 10], dtype=np.int32))
    assert [len(d) for d in D] == [4, 5, 1] and sum(D, []) == ref.tolist()
    assert all(isinstance(t, int) for d in D for t in d)
