"""Python binding of libngg (argument marshalling only; every step of the verify
path runs in the library's HIP kernels).  PyTorch is used for device memory and
the stream.  Function names mirror include/ngg.h.

The library is built in-tree by ``__graft_entry__.build()``; importing this
package never compiles anything, and using it without the built library raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libngg.so")

NGG_OK, NGG_EINVAL, NGG_ECAPACITY, NGG_ESTATE, NGG_EHIP, NGG_ENOMEM = 0, -1, -2, -3, -4, -5
NGG_F32, NGG_BF16 = 0, 1
PROF_CLASSES = ("gemm_qkv", "gemm_o", "gemm_gateup", "gemm_down", "gemm_unembed", "attention", "norm", "drafts",
                "accept_commit", "other")

EXPORTS = ("ngg_create", "ngg_destroy", "ngg_prefill", "ngg_build_drafts", "ngg_verify_step", "ngg_commit",
           "ngg_greedy_decode", "ngg_get_tokens", "ngg_last_error", "ngg_profile_enable", "ngg_profile_reset",
           "ngg_profile_read", "ngg_debug_peek", "ngg_bigram_table_build", "ngg_bigram_source", "ngg_profile_bracket_overhead", "ngg_unigram_build", "ngg_decode_more", "ngg_profile_sample",
           "ngg_context_drafts_static", "ngg_allocation", "ngg_profile_read_bandwidth", "ngg_step_graphs")
NGG_STATIC_MAX_TOKENS = 32768


class ngg_model_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab",
                                         "dtype")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("max_seq", "max_k", "max_w")]


class ngg_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")]


class ngg_weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("unemb", C.c_void_p), ("final_norm", C.c_void_p),
                ("layers", C.POINTER(ngg_layer_weights))]


class ngg_draft_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("k", "w", "k_ctx_max", "q_min", "q_max")]


class ngg_verify_out(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("k", "w", "winner", "n_accept", "n_new")] + \
               [("greedy", C.POINTER(C.c_int32)), ("accept_len", C.POINTER(C.c_int32)),
                ("new_tokens", C.POINTER(C.c_int32)), ("logits", C.POINTER(C.c_float))]


class ngg_stats(C.Structure):
    _fields_ = [("calls", C.c_int64), ("tokens", C.c_int64), ("new_hist", C.c_int64 * 34),
                ("winner_src", C.c_int64 * 2), ("ctx_rows", C.c_int64),
                ("ms_prefill", C.c_double), ("ms_drafts", C.c_double), ("ms_verify", C.c_double),
                ("ms_commit", C.c_double), ("accept_hist", (C.c_int64 * 34) * 2), ("rank_hist", (C.c_int64 * 32) * 2),
                ("alloc_hist", C.c_int64 * 33)]


_lib = None


def load_library():
    """Loads csrc/libngg.so and declares the C ABI.  Raises if it was not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` (hipcc, gfx950) first; "
                           "there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, i32p, i8p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int8)
    lib.ngg_create.argtypes = [C.POINTER(ngg_model_desc), C.POINTER(ngg_weights), vp, C.POINTER(vp)]
    lib.ngg_destroy.argtypes = [vp]
    lib.ngg_prefill.argtypes = [vp, i32p, C.c_int32]
    lib.ngg_build_drafts.argtypes = [vp, C.POINTER(ngg_draft_cfg), i32p, i8p, i32p]
    lib.ngg_verify_step.argtypes = [vp, i32p, C.c_int32, C.c_int32, C.POINTER(ngg_verify_out)]
    lib.ngg_commit.argtypes = [vp, C.c_int32, i32p]
    lib.ngg_greedy_decode.argtypes = [vp, i32p, C.c_int32, C.c_int32, C.POINTER(ngg_draft_cfg), i32p,
                                      C.POINTER(ngg_stats)]
    lib.ngg_get_tokens.argtypes = [vp, i32p, C.c_int32, i32p]
    lib.ngg_decode_more.argtypes = [vp, C.c_int32, C.c_int32, C.POINTER(ngg_draft_cfg), i32p, i32p, C.POINTER(ngg_stats)]
    lib.ngg_last_error.argtypes = [vp]
    lib.ngg_last_error.restype = C.c_char_p
    lib.ngg_profile_enable.argtypes = [vp, C.c_int32]
    lib.ngg_profile_reset.argtypes = [vp]
    lib.ngg_profile_sample.argtypes = [vp, C.c_int32]
    lib.ngg_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.ngg_debug_peek.argtypes = [vp, C.c_char_p, vp, C.c_int64, C.POINTER(C.c_int64), i32p]
    lib.ngg_bigram_table_build.argtypes = [vp, C.c_int32]
    lib.ngg_unigram_build.argtypes = [vp, C.c_int32]
    lib.ngg_profile_bracket_overhead.argtypes = [vp, C.POINTER(C.c_double)]
    lib.ngg_bigram_source.argtypes = [vp, C.c_int32]
    lib.ngg_allocation.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32]
    lib.ngg_step_graphs.argtypes = [vp, C.c_int32]
    lib.ngg_profile_read_bandwidth.argtypes = [vp, C.POINTER(C.c_double)]
    lib.ngg_context_drafts_static.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, vp, vp]
    for name in EXPORTS:
        if name != "ngg_last_error":
            getattr(lib, name).restype = C.c_int32
    _lib = lib
    return lib


class NggError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"ngg status {status}: {message}")
        self.status = status


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a, ctype=C.c_int32):
    return a.ctypes.data_as(C.POINTER(ctype))


def upload_weights(desc: dict, weights: dict, device="cuda"):
    """Host fp32 arrays (bf16-representable for a bf16 model) -> device tensors of the
    model's storage type.  Values are copied bit-exactly."""
    import torch
    dt = torch.bfloat16 if desc["dtype"] == "bf16" else torch.float32

    def up(a):
        if isinstance(a, torch.Tensor):
            return a.to(device=device, dtype=dt).contiguous()
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device=device, dtype=dt).contiguous()

    out = dict(tok_emb=up(weights["tok_emb"]), unemb=up(weights["unemb"]), final_norm=up(weights["final_norm"]),
               layers=[{k: up(v) for k, v in lw.items()} for lw in weights["layers"]])
    return out


class Context:
    """Owns an ngg_ctx.  `weights` is either host arrays (uploaded here) or the dict of
    device tensors returned by upload_weights (kept alive here: the library borrows them)."""

    def __init__(self, desc: dict, weights: dict, max_seq: int, max_k: int, max_w: int, stream=None):
        import torch
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("ngg needs a GPU: there is no CPU fallback")
        first = weights["tok_emb"]
        self.dev_weights = weights if (isinstance(first, torch.Tensor) and first.is_cuda) else upload_weights(desc, weights)
        self.desc = dict(desc)
        d = ngg_model_desc(desc["n_layers"], desc["d_model"], desc["n_heads"], desc["n_kv_heads"], desc["head_dim"],
                           desc["d_ffn"], desc["vocab"], NGG_BF16 if desc["dtype"] == "bf16" else NGG_F32,
                           desc["rms_eps"], desc["rope_theta"], max_seq, max_k, max_w)
        self.max_k, self.max_w = max_k, max_w
        L = desc["n_layers"]
        self._layers = (ngg_layer_weights * L)()
        for i, lw in enumerate(self.dev_weights["layers"]):
            for name, _ in ngg_layer_weights._fields_:
                setattr(self._layers[i], name, lw[name].data_ptr())
        w = ngg_weights(self.dev_weights["tok_emb"].data_ptr(), self.dev_weights["unemb"].data_ptr(),
                        self.dev_weights["final_norm"].data_ptr(), self._layers)
        self._stream = stream if stream is not None else torch.cuda.current_stream()
        torch.cuda.synchronize()                       # uploads done before the library reads them on its stream
        self.h = C.c_void_p()
        st = self.lib.ngg_create(C.byref(d), C.byref(w), C.c_void_p(self._stream.cuda_stream), C.byref(self.h))
        if st != NGG_OK:
            raise NggError(st, self.lib.ngg_last_error(None).decode())

    def _check(self, st):
        if st != NGG_OK:
            raise NggError(st, self.lib.ngg_last_error(self.h).decode())

    def close(self):
        if self.h:
            self.lib.ngg_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the C entry points, same names -----------------------------------------------------
    def prefill(self, prompt):
        p = _i32(prompt)
        self._check(self.lib.ngg_prefill(self.h, _ptr(p), len(p)))

    def build_drafts(self, cfg: dict, fetch=True):
        c = ngg_draft_cfg(cfg["k"], cfg["w"], cfg["k_ctx_max"], cfg["q_min"], cfg["q_max"])
        if not fetch:
            self._check(self.lib.ngg_build_drafts(self.h, C.byref(c), None, None, None))
            return None
        drafts = np.zeros((cfg["k"], cfg["w"]), dtype=np.int32)
        src = np.zeros(cfg["k"], dtype=np.int8)
        n_ctx = C.c_int32(0)
        self._check(self.lib.ngg_build_drafts(self.h, C.byref(c), _ptr(drafts), _ptr(src, C.c_int8), C.byref(n_ctx)))
        return drafts, src, n_ctx.value

    def verify_step(self, drafts, k=None, w=None, want_logits=False, fetch=True):
        if drafts is not None:
            drafts = _i32(drafts)
            k, w = drafts.shape
        out = ngg_verify_out()
        res = {}
        if fetch:
            res["greedy"] = np.zeros((k, w + 1), dtype=np.int32)
            res["accept_len"] = np.zeros(k, dtype=np.int32)
            res["new_tokens"] = np.zeros(w + 1, dtype=np.int32)
            out.greedy, out.accept_len, out.new_tokens = _ptr(res["greedy"]), _ptr(res["accept_len"]), _ptr(res["new_tokens"])
        if want_logits:
            res["logits"] = np.zeros((k, w + 1, self.desc["vocab"]), dtype=np.float32)
            out.logits = _ptr(res["logits"], C.c_float)
        self._check(self.lib.ngg_verify_step(self.h, _ptr(drafts) if drafts is not None else None, k, w, C.byref(out)))
        res.update(winner=out.winner, n_accept=out.n_accept, n_new=out.n_new)
        if fetch:
            res["new_tokens"] = res["new_tokens"][:out.n_new]
        return res

    def commit(self, max_new=1 << 30):
        n = C.c_int32(0)
        self._check(self.lib.ngg_commit(self.h, max_new, C.byref(n)))
        return n.value

    @staticmethod
    def _stats(st):
        return dict(calls=st.calls, tokens=st.tokens, new_hist=list(st.new_hist), winner_src=list(st.winner_src),
                    ctx_rows=st.ctx_rows, ms_prefill=st.ms_prefill, ms_drafts=st.ms_drafts, ms_verify=st.ms_verify,
                    ms_commit=st.ms_commit, accept_hist=[list(r) for r in st.accept_hist],
                    rank_hist=[list(r) for r in st.rank_hist], alloc_hist=list(st.alloc_hist))

    def greedy_decode(self, prompt, n_gen, cfg: dict | None):
        p = _i32(prompt)
        out = np.zeros(n_gen, dtype=np.int32)
        st = ngg_stats()
        c = None if cfg is None else ngg_draft_cfg(cfg["k"], cfg["w"], cfg["k_ctx_max"], cfg["q_min"], cfg["q_max"])
        self._check(self.lib.ngg_greedy_decode(self.h, _ptr(p), len(p), n_gen, C.byref(c) if c is not None else None,
                                               _ptr(out), C.byref(st)))
        return out, self._stats(st)

    def decode_more(self, n_gen, max_calls, cfg: dict | None):
        out = np.zeros(n_gen, dtype=np.int32)
        n_out = C.c_int32(0)
        st = ngg_stats()
        c = None if cfg is None else ngg_draft_cfg(cfg["k"], cfg["w"], cfg["k_ctx_max"], cfg["q_min"], cfg["q_max"])
        self._check(self.lib.ngg_decode_more(self.h, n_gen, max_calls, C.byref(c) if c is not None else None, _ptr(out),
                                             C.byref(n_out), C.byref(st)))
        return out[:n_out.value], self._stats(st)

    def profile_read_bandwidth(self):
        g = C.c_double(0.0)
        self._check(self.lib.ngg_profile_read_bandwidth(self.h, C.byref(g)))
        return g.value

    def profile_bracket_overhead(self):
        us = C.c_double(0.0)
        self._check(self.lib.ngg_profile_bracket_overhead(self.h, C.byref(us)))
        return us.value

    def bigram_table_build(self, top_k):
        self._check(self.lib.ngg_bigram_table_build(self.h, top_k))

    def unigram_build(self, top_k):
        self._check(self.lib.ngg_unigram_build(self.h, top_k))

    def allocation(self, mode, coverage_percent=90, warmup_wins=8):
        self._check(self.lib.ngg_allocation(self.h, int(mode), int(coverage_percent), int(warmup_wins)))

    def step_graphs(self, mode):
        self._check(self.lib.ngg_step_graphs(self.h, int(mode)))

    def bigram_source(self, source):
        """0 = direct sweep per step (default), 1 = the precomputed full-model table, 2 = the unigram."""
        self._check(self.lib.ngg_bigram_source(self.h, source))

    def get_tokens(self):
        n = C.c_int32(0)
        self._check(self.lib.ngg_get_tokens(self.h, None, 0, C.byref(n)))
        out = np.zeros(n.value, dtype=np.int32)
        self._check(self.lib.ngg_get_tokens(self.h, _ptr(out), n.value, C.byref(n)))
        return out

    def debug_peek(self, name, dtype, count=None):
        """Internal device buffer `name` as a flat numpy array of `dtype` (test aid)."""
        nbytes, stride = C.c_int64(0), C.c_int32(0)
        self._check(self.lib.ngg_debug_peek(self.h, name.encode(), None, 0, C.byref(nbytes), C.byref(stride)))
        item = np.dtype(dtype).itemsize
        n = nbytes.value // item if count is None else min(count, nbytes.value // item)
        out = np.zeros(n, dtype=dtype)
        self._check(self.lib.ngg_debug_peek(self.h, name.encode(), out.ctypes.data_as(C.c_void_p), n * item,
                                            C.byref(nbytes), C.byref(stride)))
        return out, stride.value

    def profile_enable(self, class_mask=-1):
        self._check(self.lib.ngg_profile_enable(self.h, int(class_mask)))

    def profile_sample(self, every=1):
        self._check(self.lib.ngg_profile_sample(self.h, int(every)))

    def profile_reset(self):
        self._check(self.lib.ngg_profile_reset(self.h))

    def profile_read(self):
        n = len(PROF_CLASSES)
        ms = (C.c_double * n)()
        cnt = (C.c_int64 * n)()
        self._check(self.lib.ngg_profile_read(self.h, ms, cnt))
        return {name: (ms[i], cnt[i]) for i, name in enumerate(PROF_CLASSES)}


def context_drafts_static(tokens, w, k_ctx_max, q_min, q_max, rows, n_rows, stream=None, n=None):
    """ngg_context_drafts_static: the context N-gram rows for `tokens` (int32 DEVICE tensor, the whole
    context) into `rows` (int32 DEVICE tensor [k_ctx_max][w]) and `n_rows` (int32 DEVICE tensor [1]),
    queued on `stream` (a torch stream, default: the current one) without synchronising.  Allocates
    nothing.  `n` overrides the token count (for testing the argument checks)."""
    import torch
    lib = load_library()
    for t in (tokens, rows, n_rows):
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
            raise TypeError("context_drafts_static takes contiguous int32 device tensors")
    if rows.numel() < k_ctx_max * w or n_rows.numel() < 1:
        raise ValueError("rows must hold k_ctx_max * w entries and n_rows one")
    s = stream if stream is not None else torch.cuda.current_stream()
    st = lib.ngg_context_drafts_static(tokens.data_ptr(), int(tokens.numel() if n is None else n), int(w), int(k_ctx_max),
                                       int(q_min), int(q_max), rows.data_ptr(), n_rows.data_ptr(), s.cuda_stream)
    if st != NGG_OK:
        raise NggError(st, lib.ngg_last_error(None).decode())
