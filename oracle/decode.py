"""CPU oracle: greedy decoding, the n-gram trigger, LLMA decoding and the model-free
step-sequence predictor.

TEST INFRASTRUCTURE ONLY (see model.py).  Every function follows the paper's own order of
steps and notation: x prompt, y output, D documents, n match length, k copy length, N
output budget.

An `llm` here is any callable  llm(y, drafts) -> (o_0, ..., o_len(drafts))  where o_j is
the greedy next token after the context  x + y + drafts[:j]  (Eq. 3; Eq. 2 when drafts is
empty).  `CachedLLM` backs it with the transformer oracle and a key/value cache;
`ScriptedLLM` replays a fixed target, which is the paper's target-guided trick.
"""
from __future__ import annotations

import numpy as np

from .model import OracleModel, argmax_tokens


# --------------------------------------------------------------------------- the model as LLM(.)
class CachedLLM:
    """LLM(x, y, d_pos..d_pos+k-1) on the transformer oracle with a KV cache.

    The cache always holds the first len(x)+len(y)-1 context tokens when a call starts; the
    call feeds the last context token plus the drafts.  Rows written for drafts that are
    later rejected lie beyond the next call's start position and are overwritten, which is
    the cache truncation the method needs."""

    def __init__(self, model: OracleModel, x, capacity: int):
        self.model = model
        self.x = [int(t) for t in x]
        self.cache = model.new_cache(capacity)
        self.last_logits = None
        self.rows_fed = 0
        if len(self.x) > 1:
            model.forward(self.x[:-1], self.cache, 0)
            self.rows_fed += len(self.x) - 1

    def __call__(self, y, drafts):
        ctx_len = len(self.x) + len(y)
        last = y[-1] if len(y) else self.x[-1]
        rows = [int(last)] + [int(t) for t in drafts]
        self.last_logits = self.model.forward(rows, self.cache, ctx_len - 1)
        self.rows_fed += len(rows)
        return argmax_tokens(self.last_logits).tolist()


class ScriptedLLM:
    """A fake model whose greedy continuation of the empty output is exactly `target`
    (extended with `filler` beyond its end).  After any prefix that deviates from the
    target it answers with `filler`, so outputs computed from wrong drafts are visibly
    wrong if they were ever emitted."""

    def __init__(self, target, filler: int = -7):
        self.target = [int(t) for t in target]
        self.filler = filler
        self.calls = []                      # (len(y), len(drafts)) per call

    def _next(self, prefix):
        i = len(prefix)
        if i < len(self.target) and prefix == self.target[:i]:
            return self.target[i]
        return self.filler

    def __call__(self, y, drafts):
        self.calls.append((len(y), len(drafts)))
        y = [int(t) for t in y]
        drafts = [int(t) for t in drafts]
        return [self._next(y + drafts[:j]) for j in range(len(drafts) + 1)]


# --------------------------------------------------------------------------- Eq. 2
def greedy_decode(llm, N: int):
    """Stepwise decoding: y_i = argmax P(. | x, y_<i), one token per model call."""
    y = []
    while len(y) < N:
        y.append(llm(y, [])[0])
    return y


# --------------------------------------------------------------------------- trigger
def match_ngrams(y, D, n: int):
    """Does the n-token tail of y occur in some document?  (Method, second paragraph.)

    Candidates are all (doc, pos) with n <= pos < len(d) and d[pos-n:pos] == y[-n:], so
    that at least one token d[pos] is left to copy and the span lies inside one document.
    Among several, the one whose preceding text agrees longest with the end of y wins
    (length of the common suffix of d[:pos] and y); remaining ties go to the smallest doc
    index, then the smallest pos (the paper breaks them at random; any choice gives the
    same tokens).  Only generated tokens are matched, never the prompt.
    Returns (matched, doc, pos)."""
    i = len(y)
    if n < 1 or i < n:
        return False, -1, -1
    best = None
    for di, d in enumerate(D):
        for pos in range(n, len(d)):
            if list(d[pos - n:pos]) != list(y[i - n:i]):
                continue
            score = 0
            while score < pos and score < i and d[pos - 1 - score] == y[i - 1 - score]:
                score += 1
            if best is None or score > best[0]:
                best = (score, di, pos)
    if best is None:
        return False, -1, -1
    return True, best[1], best[2]


def copy_length(k: int, d, pos: int, N: int, i: int) -> int:
    """Number of draft tokens actually copied: at most k, never past the document's end,
    and never more than would overshoot the output budget (a step emits up to drafts+1)."""
    return max(0, min(k, len(d) - pos, N - i - 1))


# --------------------------------------------------------------------------- Algorithm 1
def llma_decode(llm, D, n: int, k: int, N: int):
    """LLMA decoding.  Returns (y, trace); trace rows are (rows_in, emitted, doc, pos) with
    doc = pos = -1 for steps that copied nothing."""
    y = []
    trace = []
    while len(y) < N:
        matched, di, pos = match_ngrams(y, D, n)
        ke = copy_length(k, D[di], pos, N, len(y)) if matched else 0
        if ke == 0:
            o = llm(y, [])
            y.append(o[0])
            trace.append((1, 1, -1, -1))
            continue
        drafts = [int(t) for t in D[di][pos:pos + ke]]
        o = llm(y, drafts)
        y.append(o[0])
        emitted = 1
        for j in range(ke):
            if o[j] != drafts[j]:
                break
            y.append(o[j + 1])
            emitted += 1
        trace.append((1 + ke, emitted, di, pos))
    return y, trace


# --------------------------------------------------------------------------- Algorithm 2
def get_matched_tokens(d, pos: int, y, step: int) -> int:
    """Length of the common prefix of d[pos:] and y[step:]."""
    c = 0
    while pos + c < len(d) and step + c < len(y) and d[pos + c] == y[step + c]:
        c += 1
    return c


def infer_decoding_sequence(y, D, n: int, k: int):
    """Predict LLMA's step sequence from a known greedy output y without any model
    (the target-guided simulation's Algorithm).  Uses the same trigger and the same
    copy-length rule as llma_decode with N = len(y); rows are (rows_in, emitted, doc, pos)."""
    step = 0
    s = []
    N = len(y)
    while step < N:
        matched, di, pos = match_ngrams(y[:step], D, n)
        ke = copy_length(k, D[di], pos, N, step) if matched else 0
        if ke == 0:
            step += 1
            s.append((1, 1, -1, -1))
            continue
        num_valid = min(ke, get_matched_tokens(D[di], pos, y, step))
        s.append((1 + ke, num_valid + 1, di, pos))
        step += num_valid + 1
    return s


def docs_from_flat(ref, doc_offsets):
    """Split a flat reference array into the list of documents D."""
    ref = np.asarray(ref)
    return [ref[doc_offsets[j]:doc_offsets[j + 1]].tolist() for j in range(len(doc_offsets) - 1)]
