"""CPU oracle for LLMA decoding (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It never imports the GPU package and shares no code with it.
"""
from .model import OracleModel, KVCache, argmax_tokens, top2_gap, rmsnorm, rope, silu  # noqa: F401
from .decode import (CachedLLM, ScriptedLLM, greedy_decode, match_ngrams, copy_length,  # noqa: F401
                     llma_decode, get_matched_tokens, infer_decoding_sequence, docs_from_flat)
