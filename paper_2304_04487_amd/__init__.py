"""Python binding of libllma.so (include/llma.h): argument marshalling only.

Every step of the decoding path runs inside the HIP library; PyTorch is used here only to
hold device memory (weights handed to llma_create, logits dump buffers) and to name the
stream.  There is no CPU fallback: if the shared library has not been built, importing the
functions works but the first call raises LlmaError.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_double, c_float, c_int32, c_int64, c_void_p

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libllma.so")

LLMA_OK, LLMA_E_INVAL, LLMA_E_RANGE, LLMA_E_NOMEM, LLMA_E_HIP, LLMA_E_STATE = 0, -1, -2, -3, -4, -5
LLMA_DTYPE_F32, LLMA_DTYPE_BF16 = 0, 1
LLMA_OPT_ACT_SPLIT, LLMA_OPT_KERNEL_TIMING, LLMA_OPT_USE_GRAPH = 1, 2, 3

EXPORTS = [
    "llma_create", "llma_destroy", "llma_last_error", "llma_reset", "llma_prefill", "llma_get_state",
    "llma_set_pending", "llma_kv_import", "llma_find_trigger", "llma_verify_step",
    "llma_verify_step_batch", "llma_generate", "llma_generate_batch", "llma_set_logits_dump", "llma_set_option",
    "llma_get_kernel_timing", "llma_time_ffn_gemm", "llma_time_step_gemm", "llma_device_bytes", "llma_find_trigger_static", "llma_truncate",
    "llma_describe",
]
LLMA_TRIGGER_STATIC_MAX_REF = 1 << 20


class LlmaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"llma error {code}: {msg}")
        self.code = code


class ModelCfgC(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab",
                                       "max_seq", "max_batch", "max_k", "dtype", "kv_split")] + \
               [("rms_eps", c_float), ("rope_theta", c_float)]


class WeightsC(ctypes.Structure):
    _fields_ = [("embed", c_void_p), ("lm_head", c_void_p), ("final_norm", c_void_p),
                ("wqkv", POINTER(c_void_p)), ("wo", POINTER(c_void_p)), ("wgu", POINTER(c_void_p)),
                ("wdown", POINTER(c_void_p)), ("norm1", POINTER(c_void_p)), ("norm2", POINTER(c_void_p))]


class StepRec(ctypes.Structure):
    _fields_ = [("rows_in", c_int32), ("emitted", c_int32), ("doc", c_int32), ("pos", c_int32)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads the in-tree libllma.so; raises LlmaError when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise LlmaError(LLMA_E_INVAL, f"{LIB_PATH} is missing: run `python -m paper_2304_04487_amd.build` "
                                      "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    i32p, vp = POINTER(c_int32), c_void_p
    lib.llma_create.argtypes = [POINTER(ModelCfgC), POINTER(WeightsC), vp, POINTER(vp)]
    lib.llma_destroy.argtypes = [vp]
    lib.llma_last_error.argtypes = [vp]
    lib.llma_last_error.restype = c_char_p
    lib.llma_reset.argtypes = [vp, c_int32]
    lib.llma_prefill.argtypes = [vp, c_int32, i32p, c_int32]
    lib.llma_get_state.argtypes = [vp, c_int32, i32p, i32p]
    lib.llma_set_pending.argtypes = [vp, c_int32, c_int32]
    lib.llma_truncate.argtypes = [vp, c_int32, c_int32]
    lib.llma_kv_import.argtypes = [vp, c_int32, c_int32, vp, vp, c_int32]
    lib.llma_find_trigger.argtypes = [i32p, c_int32, i32p, i32p, c_int32, c_int32, i32p, i32p]
    lib.llma_find_trigger_static.argtypes = [vp, c_int32, vp, c_int32, vp, c_int32, c_int32, vp, vp]
    lib.llma_verify_step.argtypes = [vp, c_int32, i32p, c_int32, i32p, i32p, i32p]
    lib.llma_verify_step_batch.argtypes = [vp, c_int32, i32p, i32p, c_int32, i32p, i32p, i32p]
    lib.llma_generate.argtypes = [vp, c_int32, i32p, c_int32, i32p, i32p, c_int32, c_int32, c_int32, c_int32,
                                  i32p, i32p, POINTER(StepRec), i32p]
    lib.llma_generate_batch.argtypes = [vp, c_int32, i32p, i32p, i32p, i32p, i32p, i32p, c_int32, c_int32, c_int32,
                                        i32p, i32p, POINTER(StepRec), i32p]
    lib.llma_set_logits_dump.argtypes = [vp, vp, c_int32]
    lib.llma_set_option.argtypes = [vp, c_int32, c_int32]
    lib.llma_get_kernel_timing.argtypes = [vp, POINTER(c_int64), POINTER(c_double)]
    lib.llma_time_ffn_gemm.argtypes = [vp, c_int32, c_int32, POINTER(c_double)]
    lib.llma_time_step_gemm.argtypes = [vp, c_int32, c_int32, c_int32, POINTER(c_double)]
    lib.llma_describe.argtypes = [vp, c_char_p, c_int32]
    lib.llma_device_bytes.argtypes = [vp]
    lib.llma_device_bytes.restype = c_int64
    _lib = lib
    return lib


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32).reshape(-1))


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(POINTER(c_int32))


def _check(rc: int, ctx=None) -> int:
    if rc < 0:
        raise LlmaError(rc, load_library().llma_last_error(ctx).decode())
    return rc


def llma_find_trigger(y, ref, doc_offsets, n: int):
    """Returns (matched, doc, pos); see llma_find_trigger in llma.h."""
    lib = load_library()
    y, ref, offs = _i32(y), _i32(ref), _i32(doc_offsets)
    doc, pos = c_int32(-1), c_int32(-1)
    rc = _check(lib.llma_find_trigger(_ptr(y), len(y), _ptr(ref), _ptr(offs), len(offs) - 1, n, byref(doc), byref(pos)))
    return bool(rc), doc.value, pos.value


def llma_find_trigger_static(y_dev, ref_dev, doc_offsets_dev, n: int, result_dev, stream=None):
    """The allocation-free trigger scan on DEVICE int32 tensors (anything with data_ptr() and
    numel()); result_dev: 3 device ints (matched, doc, pos).  Enqueues on `stream` (an object with
    .cuda_stream, or None for the default stream) and returns without synchronising."""
    lib = load_library()
    n_docs = max(int(doc_offsets_dev.numel()) - 1, 0)
    st = c_void_p(stream.cuda_stream) if stream is not None else None
    _check(lib.llma_find_trigger_static(c_void_p(y_dev.data_ptr()), int(y_dev.numel()), c_void_p(ref_dev.data_ptr()),
                                        int(ref_dev.numel()), c_void_p(doc_offsets_dev.data_ptr()), n_docs, n,
                                        c_void_p(result_dev.data_ptr()), st))


class Context:
    """Owns one llma_ctx.  `cfg` is any object with n_layers, d_model, n_heads, head_dim, d_ffn,
    vocab, dtype ("fp32" | "bf16"), rms_eps, rope_theta; `weights` the dict of numpy arrays
    (bf16 as uint16 bit patterns) laid out as llma.h describes."""

    def __init__(self, cfg, weights: dict, max_seq: int, max_batch: int = 1, max_k: int = 16, device="cuda:0",
                 kv_split: bool = True):
        import torch
        self._torch = torch
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        self.max_seq, self.max_batch, self.max_k = max_seq, max_batch, max_k
        self._h = c_void_p()
        torch.cuda.set_device(self.device)
        stream = torch.cuda.current_stream(self.device)
        L = len(weights["layers"])
        c = ModelCfgC(L, cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab, max_seq, max_batch, max_k,
                      LLMA_DTYPE_BF16 if cfg.dtype == "bf16" else LLMA_DTYPE_F32, int(bool(kv_split)),
                      cfg.rms_eps, cfg.rope_theta)

        def dev(a):
            return torch.from_numpy(np.ascontiguousarray(a)).to(self.device)

        # upload layer by layer and let llma_create copy; the temporaries are freed afterwards
        keep = {"embed": dev(weights["embed"]), "lm_head": dev(weights["lm_head"]), "final_norm": dev(weights["final_norm"])}
        names = ("wqkv", "wo", "wgu", "wd", "norm1", "norm2")
        per = {n: [dev(lw[n]) for lw in weights["layers"]] for n in names}
        arr = {n: (c_void_p * L)(*[t.data_ptr() for t in per[n]]) for n in names}
        w = WeightsC(keep["embed"].data_ptr(), keep["lm_head"].data_ptr(), keep["final_norm"].data_ptr(),
                     arr["wqkv"], arr["wo"], arr["wgu"], arr["wd"], arr["norm1"], arr["norm2"])
        torch.cuda.synchronize(self.device)
        _check(self.lib.llma_create(byref(c), byref(w), c_void_p(stream.cuda_stream), byref(self._h)))
        del keep, per
        self._dump = None

    # -- lifetime
    def close(self):
        if self._h:
            self.lib.llma_destroy(self._h)
            self._h = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ck(self, rc):
        return _check(rc, self._h)

    # -- state
    def reset(self, seq: int = 0):
        self._ck(self.lib.llma_reset(self._h, seq))

    def prefill(self, prompt, seq: int = 0):
        p = _i32(prompt)
        self._ck(self.lib.llma_prefill(self._h, seq, _ptr(p), len(p)))

    def get_state(self, seq: int = 0):
        t, p = c_int32(), c_int32()
        self._ck(self.lib.llma_get_state(self._h, seq, byref(t), byref(p)))
        return t.value, p.value

    def truncate(self, new_len: int, seq: int = 0):
        self._ck(self.lib.llma_truncate(self._h, seq, int(new_len)))

    def set_pending(self, token: int, seq: int = 0):
        self._ck(self.lib.llma_set_pending(self._h, seq, int(token)))

    def kv_import(self, seq: int, layer: int, k_dev, v_dev, length: int):
        """k_dev, v_dev: torch device tensors, plain [n_heads, length, head_dim] in the model dtype
        (bf16 tensors or uint16 bit patterns for bf16 models)."""
        self._ck(self.lib.llma_kv_import(self._h, seq, layer, c_void_p(k_dev.data_ptr()), c_void_p(v_dev.data_ptr()), length))

    # -- the method
    def verify_step(self, draft, seq: int = 0):
        """Returns (n_accepted, next_token, emitted list)."""
        d = _i32(draft)
        k = len(d)
        na, nt = c_int32(), c_int32()
        em = np.zeros(k + 1, dtype=np.int32)
        self._ck(self.lib.llma_verify_step(self._h, seq, _ptr(d), k, byref(na), byref(nt), _ptr(em)))
        return na.value, nt.value, em[:na.value + 1].tolist()

    def verify_step_batch(self, seqs, drafts):
        """drafts: [n_seqs, k].  Returns (n_accepted[n_seqs], next_token[n_seqs], emitted[n_seqs][...])."""
        s = _i32(seqs)
        d2 = np.asarray(drafts, dtype=np.int32).reshape(len(s), -1)
        k = d2.shape[1]
        d = _i32(d2)
        na, nt = np.zeros(len(s), np.int32), np.zeros(len(s), np.int32)
        em = np.zeros(len(s) * (k + 1), np.int32)
        self._ck(self.lib.llma_verify_step_batch(self._h, len(s), _ptr(s), _ptr(d), k, _ptr(na), _ptr(nt), _ptr(em)))
        em = em.reshape(len(s), k + 1)
        return na, nt, [em[b, :na[b] + 1].tolist() for b in range(len(s))]

    def generate(self, prompt, ref, doc_offsets, n: int, k: int, max_new: int, seq: int = 0):
        """Returns (tokens int32[max_new], trace list of (rows_in, emitted, doc, pos))."""
        p = _i32(prompt)
        r = _i32(ref if ref is not None else [])
        offs = _i32(doc_offsets if doc_offsets is not None else [0])
        out = np.zeros(max_new, np.int32)
        n_out, n_steps = c_int32(), c_int32()
        tr = (StepRec * max_new)()
        self._ck(self.lib.llma_generate(self._h, seq, _ptr(p), len(p), _ptr(r), _ptr(offs), len(offs) - 1, n, k, max_new,
                                        _ptr(out), byref(n_out), tr, byref(n_steps)))
        trace = [(t.rows_in, t.emitted, t.doc, t.pos) for t in tr[:n_steps.value]]
        return out[:n_out.value], trace

    def generate_batch(self, prompts, refs, n: int, k: int, max_new: int, seqs=None):
        """One LLMA decoding per sequence, all sequences in the same steps.  prompts: list of id
        arrays; refs: list of (ref, doc_offsets) or None per sequence.  Returns a list of
        (tokens int32[max_new], trace) per sequence."""
        B = len(prompts)
        s = _i32(seqs if seqs is not None else list(range(B)))
        ps = [_i32(p) for p in prompts]
        poff = _i32(np.concatenate([[0], np.cumsum([len(p) for p in ps])]))
        pcat = _i32(np.concatenate(ps))
        rs, offs, nd = [], [], []
        for r in refs:
            if r is None:
                rs.append(np.zeros(0, np.int32)); offs.append(np.zeros(1, np.int32)); nd.append(0)
            else:
                rs.append(_i32(r[0])); offs.append(_i32(r[1])); nd.append(len(offs[-1]) - 1)
        rcat, ocat, ndv = _i32(np.concatenate(rs)), _i32(np.concatenate(offs)), _i32(nd)
        out = np.zeros(B * max_new, np.int32)
        n_out, n_steps = np.zeros(B, np.int32), np.zeros(B, np.int32)
        tr = (StepRec * (B * max_new))()
        self._ck(self.lib.llma_generate_batch(self._h, B, _ptr(s), _ptr(pcat), _ptr(poff), _ptr(rcat), _ptr(ocat), _ptr(ndv),
                                              n, k, max_new, _ptr(out), _ptr(n_out), tr, _ptr(n_steps)))
        res = []
        for b in range(B):
            trace = [(t.rows_in, t.emitted, t.doc, t.pos) for t in tr[b * max_new:b * max_new + int(n_steps[b])]]
            res.append((out[b * max_new:b * max_new + int(n_out[b])].copy(), trace))
        return res

    # -- inspection
    def enable_logits_dump(self, rows: int):
        """Allocates a device buffer [rows, vocab] fp32 that every later forward fills."""
        self._dump = self._torch.zeros((rows, self.cfg.vocab), dtype=self._torch.float32, device=self.device)
        self._ck(self.lib.llma_set_logits_dump(self._h, c_void_p(self._dump.data_ptr()), rows))

    def disable_logits_dump(self):
        self._ck(self.lib.llma_set_logits_dump(self._h, None, 0))
        self._dump = None

    def logits(self, rows: int) -> np.ndarray:
        self._torch.cuda.synchronize(self.device)
        return self._dump[:rows].cpu().numpy()

    def set_option(self, option: int, value: int):
        self._ck(self.lib.llma_set_option(self._h, option, value))

    def kernel_timing(self):
        n, ms = c_int64(), c_double()
        self._ck(self.lib.llma_get_kernel_timing(self._h, byref(n), byref(ms)))
        return n.value, ms.value

    def time_ffn_gemm(self, rows: int, reps: int) -> float:
        us = c_double()
        self._ck(self.lib.llma_time_ffn_gemm(self._h, rows, reps, byref(us)))
        return us.value

    def time_step_gemm(self, which: int, rows: int, reps: int) -> float:
        us = c_double()
        self._ck(self.lib.llma_time_step_gemm(self._h, which, rows, reps, byref(us)))
        return us.value

    def describe(self) -> str:
        buf = ctypes.create_string_buffer(512)
        self._ck(self.lib.llma_describe(self._h, buf, 512))
        return buf.value.decode()

    def device_bytes(self) -> int:
        return int(self.lib.llma_device_bytes(self._h))
