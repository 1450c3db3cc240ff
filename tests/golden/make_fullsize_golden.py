#!/usr/bin/env python3
"""Writes the stored oracle results for the two full-size configurations whose CPU oracle run
takes minutes (LLaMA-7B shape, 32 layers) to tens of minutes (13B shape, 40 layers):

    python tests/golden/make_fullsize_golden.py 7b     -> tests/golden/oracle_7b_rag_prompt1536.npz
    python tests/golden/make_fullsize_golden.py 13b    -> tests/golden/oracle_13b_multiturn_prompt2048.npz

Imports only oracle/ (the CPU implementation written from the paper) and synth/ (the seeded
input generators); nothing here touches the GPU library.  The GPU parity tests load the
files with numpy.load (no pickling) and compare the library's logits / tokens / step traces
with them; the step traces themselves are recomputed in the tests from the stored tokens with
the oracle's model-free step predictor (Algorithm 2), which takes milliseconds.

What is stored, per generated position i of stepwise greedy decoding (Eq. 2) on the
configuration's own seeded prompt and weights, float32 arithmetic (float64 copies of the
weights do not fit in host memory at these sizes):
    y[i]                 the oracle's greedy token
    top_ids/top_vals[i]  its four largest logits (ids, values) -- top_vals[i,0] - top_vals[i,1]
                         is the top-2 gap that decides whether a token mismatch is a near-tie
    col_vals[i]          the logits of `cols`, 128 seeded vocabulary columns, for the logit tolerance
13b additionally stores one verification step (Eq. 3) at the end of the 2048-token prompt whose
16 drafts are the first nine greedy tokens followed by seven uniform ids (`vs_*` arrays, one row per
fed row), so accepted count and corrected token at full depth have an oracle value.
13b generates only the first N_13B tokens: every oracle forward widens the 40 layers from bf16 again.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import synth                                                        # noqa: E402
from oracle import OracleModel, CachedLLM                           # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
N_COLS, COL_STREAM = 128, 900
N_13B = 32
FILES = {"7b": "oracle_7b_rag_prompt1536.npz", "13b": "oracle_13b_multiturn_prompt2048.npz"}


def sample_cols(wl):
    return np.unique(synth.uniform_tokens(wl.seed, COL_STREAM, N_COLS, wl.model.vocab)).astype(np.int32)


def record(lg_row, cols):
    lg = lg_row.astype(np.float32)
    order = np.argsort(-lg, kind="stable")[:4]                      # ties: lowest id first
    return order.astype(np.int32), lg[order], lg[cols]


def run(name):
    wl = synth.WORKLOADS[name]
    cfg = wl.model
    t0 = time.time()
    w = synth.make_weights(cfg, wl.seed)
    lazy = name == "13b"
    om = OracleModel(cfg, w, dtype=np.float32, lazy=lazy)
    if not lazy:
        del w
    print(f"[{name}] weights ready in {time.time() - t0:.0f}s", flush=True)
    prompt = synth.make_prompt(wl)
    n_new = N_13B if name == "13b" else wl.max_new
    cols = sample_cols(wl)
    t0 = time.time()
    llm = CachedLLM(om, prompt, wl.prompt_len + n_new + 32)
    print(f"[{name}] prompt of {len(prompt)} tokens processed in {time.time() - t0:.0f}s", flush=True)
    y, ids, vals, cv = [], [], [], []
    t0 = time.time()
    for i in range(n_new):
        o = llm(y, [])
        a, b, c = record(llm.last_logits[0], cols)
        assert int(a[0]) == int(o[0])
        y.append(int(o[0])); ids.append(a); vals.append(b); cv.append(c)
        if i % 8 == 7:
            print(f"[{name}] {i + 1}/{n_new} tokens, {time.time() - t0:.0f}s", flush=True)
    out = {"y": np.asarray(y, np.int32), "top_ids": np.stack(ids), "top_vals": np.stack(vals),
           "cols": cols, "col_vals": np.stack(cv), "seed": np.int64(wl.seed), "prompt_len": np.int32(len(prompt))}
    if name == "13b":
        junk = synth.uniform_tokens(wl.seed, COL_STREAM + 1, 7, cfg.vocab).tolist()
        drafts = y[:9] + junk
        T = len(prompt) - 1
        lg = om.forward([int(prompt[-1])] + drafts, llm.cache, T)   # overwrites rows T.. (the greedy run is over)
        rec = [record(lg[j], cols) for j in range(len(drafts) + 1)]
        out.update({"vs_draft": np.asarray(drafts, np.int32), "vs_top_ids": np.stack([r[0] for r in rec]),
                    "vs_top_vals": np.stack([r[1] for r in rec]), "vs_col_vals": np.stack([r[2] for r in rec])})
    path = os.path.join(HERE, FILES[name])
    np.savez_compressed(path, **out)
    print(f"[{name}] wrote {path} ({os.path.getsize(path)} bytes)", flush=True)


if __name__ == "__main__":
    for nm in sys.argv[1:] or ["7b", "13b"]:
        run(nm)
