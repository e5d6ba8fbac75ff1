"""ctypes binding of libcsd.so: same names as the C ABI, torch tensors in, torch tensors out.

Only marshalling happens here; every step of the verify path runs in the HIP kernels.
`import torch` must come before the library is loaded so that the library binds to the HIP
runtime PyTorch already brought into the process (one runtime, shared streams and pointers).
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcsd.so")

EXPORTS = ["csd_version", "csd_last_hip_error", "csd_model_create", "csd_model_destroy", "csd_kv_bytes",
           "csd_kv_write", "csd_kv_read", "csd_cross_kv_init", "csd_bigram_fit", "csd_bigram_draft", "csd_maxgram_draft", "csd_verify_block",
           "csd_accept", "csd_verify_accept", "csd_verify_accept_static", "csd_review_ctx", "csd_bigram_draft_append", "csd_cascade_gate", "csd_verify_tree", "csd_tree_accept", "csd_tree_commit", "csd_debug_set_trace", "csd_debug_path", "csd_debug_gemm_plan", "csd_debug_copy", "csd_debug_read", "csd_debug_mfma",
           "csd_prof_enable", "csd_prof_read"]

_STATUS = {-1: "CSD_EINVAL", -2: "CSD_ESHAPE", -3: "CSD_ENULL", -4: "CSD_EHIP", -5: "CSD_EUNSUPPORTED"}


class CsdError(RuntimeError):
    def __init__(self, what, status, hip=0):
        super().__init__(f"{what}: {_STATUS.get(status, status)}" + (f" (hipError {hip})" if status == -4 else ""))
        self.status = status


class Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("arch", "dtype", "n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab",
                 "max_batch", "max_seq", "max_block", "enc_len")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class Review(C.Structure):
    """csd_review: device pointers of one review with device-resident control."""
    _fields_ = [("ctx", C.c_void_p), ("ctx_stride", C.c_int32), ("ctx_len", C.c_void_p), ("cache_len", C.c_void_p),
                ("prefix_len", C.c_void_p), ("q_tab", C.c_void_p), ("q_onehot_tab", C.c_void_p), ("q_base", C.c_void_p),
                ("q_stride", C.c_int32), ("u_acc_tab", C.c_void_p), ("u_samp_tab", C.c_void_p), ("out_q_tab", C.c_void_p),
                ("out_onehot_tab", C.c_void_p), ("out_base", C.c_void_p), ("out_stride", C.c_int32),
                ("lower_cache_len", C.c_void_p * 4), ("n_lower", C.c_int32), ("n_accepted", C.c_void_p),
                ("next_token", C.c_void_p), ("status", C.c_void_p), ("ext_rows", C.c_void_p)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded library; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(_LIB_PATH)
        L.csd_version.restype = C.c_char_p
        L.csd_kv_bytes.restype = C.c_size_t
        L.csd_kv_bytes.argtypes = [C.c_void_p]
        for n in EXPORTS:
            if n not in ("csd_version", "csd_kv_bytes"):
                getattr(L, n).restype = C.c_int32
        _lib = L
    return _lib


def _chk(rc, what):
    if rc != 0:
        raise CsdError(what, rc, lib().csd_last_hip_error())


def _ptr(t, dtype=None):
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda:
        raise ValueError("device tensor required")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor required")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Model:
    """csd_model plus the KV cache tensor the caller owns."""

    def __init__(self, shape, weights, max_batch=1, max_seq=2048, max_block=16):
        dtype = 1 if shape.dtype == "bf16" else 0
        self.shape = shape
        self.cfg = Cfg(shape.arch, dtype, shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim,
                       shape.d_ffn, shape.vocab, max_batch, max_seq, max_block, getattr(shape, "enc_len", 0),
                       shape.rms_eps, shape.rope_theta)
        want = torch.bfloat16 if dtype == 1 else torch.float32
        ptrs = []
        for i, w in enumerate(weights):
            bias_table = shape.arch == 1 and i == len(weights) - 1       # relative-position bias: always fp32
            ptrs.append(_ptr(w, want if (w.ndim == 2 and not bias_table) else torch.float32).value)
        arr = (C.c_void_p * len(ptrs))(*ptrs)
        self._h = C.c_void_p()
        _chk(lib().csd_model_create(C.byref(self.cfg), arr, len(ptrs), _stream(), C.byref(self._h)), "csd_model_create")
        torch.cuda.current_stream().synchronize()     # the caller's weights may now be freed
        self.kv = torch.zeros(lib().csd_kv_bytes(self._h), dtype=torch.uint8, device="cuda")
        self.max_batch, self.max_seq, self.max_block = max_batch, max_seq, max_block

    def close(self):
        if getattr(self, "_h", None):
            torch.cuda.synchronize()
            lib().csd_model_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def cross_kv_init(self, enc_out):
        """arch 1: enc_out [B][enc_len][d] fp32 on the device -> cross-attention keys/values in the cache."""
        _chk(lib().csd_cross_kv_init(self._h, _ptr(self.kv), _ptr(enc_out, torch.float32), enc_out.shape[0], _stream()),
             "csd_cross_kv_init")

    def kv_write(self, layer, b, pos0, K, V):
        n = K.shape[0]
        _chk(lib().csd_kv_write(self._h, _ptr(self.kv), layer, b, pos0, n, _ptr(K, torch.float32),
                                _ptr(V, torch.float32), _stream()), "csd_kv_write")

    def kv_read(self, layer, b, pos0, n):
        hd = self.shape.n_heads * self.shape.head_dim
        K = torch.empty((n, hd), dtype=torch.float32, device="cuda")
        V = torch.empty((n, hd), dtype=torch.float32, device="cuda")
        _chk(lib().csd_kv_read(self._h, _ptr(self.kv), layer, b, pos0, n, _ptr(K), _ptr(V), _stream()), "csd_kv_read")
        return K, V

    def verify_block(self, tokens, cache_len, temperature=1.0, want_probs=False, logits=None, probs=None):
        """tokens [B][m] int32, cache_len [B] int32 (device) -> logits [B][m][V] (and probs)."""
        B, m = tokens.shape
        V = self.shape.vocab
        if logits is None:
            logits = torch.empty((B, m, V), dtype=torch.float32, device="cuda")
        if want_probs and probs is None:
            probs = torch.empty((B, m, V), dtype=torch.float32, device="cuda")
        _chk(lib().csd_verify_block(self._h, _ptr(self.kv), _ptr(tokens, torch.int32), _ptr(cache_len, torch.int32),
                                    B, m, C.c_float(temperature), _ptr(logits), _ptr(probs), _stream()),
             "csd_verify_block")
        return (logits, probs) if want_probs else logits

    def verify_accept(self, tokens, cache_len, u_acc, u_samp, q=None, q_onehot=None, temperature=1.0,
                      lenience=1.0, mode=0, logits=None, probs=None, n_accepted=None, next_token=None, static=False):
        """static=True: csd_verify_accept_static (scratch in the library's static device array)."""
        B, m = tokens.shape
        if n_accepted is None:
            n_accepted = torch.empty(B, dtype=torch.int32, device="cuda")
        if next_token is None:
            next_token = torch.empty(B, dtype=torch.int32, device="cuda")
        fn = lib().csd_verify_accept_static if static else lib().csd_verify_accept
        _chk(fn(self._h, _ptr(self.kv), _ptr(tokens, torch.int32), _ptr(cache_len, torch.int32),
                B, m, C.c_float(temperature), _ptr(q), _ptr(q_onehot), _ptr(u_acc), _ptr(u_samp),
                C.c_float(lenience), mode, _ptr(logits), _ptr(probs), _ptr(n_accepted),
                _ptr(next_token), _stream()), "csd_verify_accept_static" if static else "csd_verify_accept")
        return n_accepted, next_token

    def verify_tree(self, tokens, parent, cache_len, temperature=1.0, want_probs=False, logits=None, probs=None):
        """csd_verify_tree: tokens, parent [B][m] int32 (device) -> logits [B][m][V] (and probs)."""
        B, m = tokens.shape
        V = self.shape.vocab
        if logits is None:
            logits = torch.empty((B, m, V), dtype=torch.float32, device="cuda")
        if want_probs and probs is None:
            probs = torch.empty((B, m, V), dtype=torch.float32, device="cuda")
        _chk(lib().csd_verify_tree(self._h, _ptr(self.kv), _ptr(tokens, torch.int32), _ptr(parent, torch.int32),
                                   _ptr(cache_len, torch.int32), B, m, C.c_float(temperature), _ptr(logits), _ptr(probs),
                                   _stream()), "csd_verify_tree")
        return (logits, probs) if want_probs else logits

    def tree_commit(self, cache_len, path, n_accepted):
        """csd_tree_commit: the kept rows' K/V move to where a plain block would have stored them."""
        B, m = path.shape
        _chk(lib().csd_tree_commit(self._h, _ptr(self.kv), _ptr(cache_len, torch.int32), _ptr(path, torch.int32),
                                   _ptr(n_accepted, torch.int32), B, m, _stream()), "csd_tree_commit")

    def review_ctx(self, ctx, ctx_len, cache_len, prefix_len, m_max, status, q_tab=None, q_onehot_tab=None, q_base=None,
                   u_acc_tab=None, u_samp_tab=None, out_q_tab=None, out_onehot_tab=None, out_base=None, lower=(),
                   n_accepted=None, next_token=None, ext_rows=None, temperature=1.0, lenience=1.0, mode=0):
        """csd_review_ctx: one review with device-resident control (every tensor stays on the device)."""
        def dp(t):
            return None if t is None else t.data_ptr()
        r = Review()
        r.ctx, r.ctx_stride, r.ctx_len, r.cache_len, r.prefix_len = dp(ctx), ctx.shape[1], dp(ctx_len), dp(cache_len), dp(prefix_len)
        r.q_tab, r.q_onehot_tab, r.q_base = dp(q_tab), dp(q_onehot_tab), dp(q_base)
        r.q_stride = (q_onehot_tab if q_onehot_tab is not None else q_tab).shape[1] if (q_tab is not None or q_onehot_tab is not None) else 0
        r.u_acc_tab, r.u_samp_tab = dp(u_acc_tab), dp(u_samp_tab)
        r.out_q_tab, r.out_onehot_tab, r.out_base = dp(out_q_tab), dp(out_onehot_tab), dp(out_base)
        r.out_stride = (out_onehot_tab if out_onehot_tab is not None else out_q_tab).shape[1] if (out_q_tab is not None or out_onehot_tab is not None) else 0
        for i, t in enumerate(lower):
            r.lower_cache_len[i] = t.data_ptr()
        r.n_lower = len(lower)
        r.n_accepted, r.next_token, r.status, r.ext_rows = dp(n_accepted), dp(next_token), dp(status), dp(ext_rows)
        _chk(lib().csd_review_ctx(self._h, _ptr(self.kv), C.byref(r), ctx.shape[0], m_max, C.c_float(temperature),
                                  C.c_float(lenience), mode, _stream()), "csd_review_ctx")

    def set_trace(self, trace):
        _chk(lib().csd_debug_set_trace(self._h, _ptr(trace)), "csd_debug_set_trace")

    def path(self, B, m):
        return int(lib().csd_debug_path(self._h, B, m))

    def prof_enable(self, on=True):
        _chk(lib().csd_prof_enable(self._h, 1 if on else 0), "csd_prof_enable")

    def prof_read(self, kernel_class, reset=False):
        ms, n = C.c_double(), C.c_int64()
        _chk(lib().csd_prof_read(self._h, kernel_class, C.byref(ms), C.byref(n), 1 if reset else 0), "csd_prof_read")
        return ms.value, n.value


def debug_copy(dst, src):
    """Streaming copy of src into dst (same byte size, a multiple of 16): counter calibration."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("debug_copy: size mismatch")
    _chk(lib().csd_debug_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), C.c_size_t(nbytes), _stream()),
         "csd_debug_copy")


def debug_read(src, sink):
    """Streaming read of src (byte size a multiple of 16); sink: uint32/int32 device tensor of >= 2048 words."""
    nbytes = src.numel() * src.element_size()
    _chk(lib().csd_debug_read(C.c_void_p(src.data_ptr()), C.c_size_t(nbytes), C.c_void_p(sink.data_ptr()), _stream()),
         "csd_debug_read")


def debug_mfma(iters, sink):
    """4096 waves x iters x 8 matrix instructions (16x16x32 bf16) on registers; returns the flops issued."""
    _chk(lib().csd_debug_mfma(C.c_int64(iters), C.c_void_p(sink.data_ptr()), _stream()), "csd_debug_mfma")
    return 4096 * iters * 8 * 16384


def bigram_fit(tokens, vocab, next_table):
    """In-place fit of next_table [vocab] int32 (pre-filled with the default successors)."""
    _chk(lib().csd_bigram_fit(_ptr(tokens, torch.int32), tokens.shape[0], vocab, _ptr(next_table, torch.int32),
                              _stream()), "csd_bigram_fit")
    return next_table


def bigram_draft(ctx, ctx_len, next_table, k, max_match=0, want_match_len=True, out=None):
    if ctx.ndim == 1:
        ctx = ctx[None, :]
    B, stride = ctx.shape
    if out is None:
        out = torch.empty((B, k), dtype=torch.int32, device="cuda")
    elif tuple(out.shape) != (B, k):
        raise ValueError("out must be [B][k]")
    mlen = torch.empty(B, dtype=torch.int32, device="cuda") if want_match_len else None
    _chk(lib().csd_bigram_draft(_ptr(ctx, torch.int32), _ptr(ctx_len, torch.int32), B, stride,
                                _ptr(next_table, torch.int32), next_table.shape[0], k, max_match, _ptr(out),
                                _ptr(mlen), _stream()), "csd_bigram_draft")
    return (out, mlen) if want_match_len else out


def maxgram_draft(haystack, haystack_len, needle, needle_len, next_table, k, max_match=0):
    """Max-Gram with a haystack of its own: returns (tokens [B][k], match_len [B], n_copied [B])."""
    B, hs = haystack.shape
    out = torch.empty((B, k), dtype=torch.int32, device="cuda")
    mlen = torch.empty(B, dtype=torch.int32, device="cuda")
    ncp = torch.empty(B, dtype=torch.int32, device="cuda")
    _chk(lib().csd_maxgram_draft(_ptr(haystack, torch.int32), _ptr(haystack_len, torch.int32), hs, _ptr(needle, torch.int32),
                                 _ptr(needle_len, torch.int32), needle.shape[1], B, _ptr(next_table, torch.int32),
                                 next_table.shape[0], k, max_match, _ptr(out), _ptr(mlen), _ptr(ncp), _stream()),
         "csd_maxgram_draft")
    return out, mlen, ncp


def tree_accept(p, tokens, parent, u=None, mode=0):
    """csd_tree_accept: p [B][m][V] -> (n_accepted [B], path [B][m], next_token [B])."""
    B, m, V = p.shape
    n_acc = torch.empty(B, dtype=torch.int32, device="cuda")
    path = torch.full((B, m), -1, dtype=torch.int32, device="cuda")
    nxt = torch.empty(B, dtype=torch.int32, device="cuda")
    _chk(lib().csd_tree_accept(_ptr(p, torch.float32), _ptr(tokens, torch.int32), _ptr(parent, torch.int32), _ptr(u), B, m, V,
                               mode, _ptr(n_acc), _ptr(path), _ptr(nxt), _stream()), "csd_tree_accept")
    return n_acc, path, nxt


def bigram_draft_append(ctx, ctx_len, next_table, k, max_match=0, gate=None, q_onehot_tab=None, q_base=None):
    """csd_bigram_draft_append: Max-Gram drafts written at the end of the device-side sequences."""
    _chk(lib().csd_bigram_draft_append(_ptr(ctx, torch.int32), ctx.shape[1], _ptr(ctx_len, torch.int32), ctx.shape[0],
                                       _ptr(next_table, torch.int32), next_table.shape[0], k, max_match, _ptr(gate),
                                       _ptr(q_onehot_tab), _ptr(q_base), q_onehot_tab.shape[1] if q_onehot_tab is not None else 0,
                                       _stream()), "csd_bigram_draft_append")


def cascade_gate(ctx_len, gate_out, loop_start=None, need=0, parent_gate=None):
    """csd_cascade_gate: the loop condition of Algorithm 1 evaluated on the device."""
    _chk(lib().csd_cascade_gate(_ptr(ctx_len, torch.int32), _ptr(loop_start), need, _ptr(parent_gate), ctx_len.shape[0],
                                _ptr(gate_out, torch.int32), _stream()), "csd_cascade_gate")


def accept(p, q, draft, u_acc, u_samp, lenience=1.0, mode=0, q_onehot=None):
    B, k1, V = p.shape
    k = k1 - 1
    n_acc = torch.empty(B, dtype=torch.int32, device="cuda")
    nxt = torch.empty(B, dtype=torch.int32, device="cuda")
    _chk(lib().csd_accept(_ptr(p, torch.float32), _ptr(q), _ptr(q_onehot), _ptr(draft), _ptr(u_acc), _ptr(u_samp),
                          B, k, V, C.c_float(lenience), mode, _ptr(n_acc), _ptr(nxt), _stream()), "csd_accept")
    return n_acc, nxt
