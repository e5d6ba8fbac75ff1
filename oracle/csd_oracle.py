"""ctypes front end of the CPU oracle (oracle/csd_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  The HIP library and its Python binding never import this module and
this module never imports them.  Arrays are numpy, on the host.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csd_oracle.c")
_LIB = os.path.join(_HERE, "libcsd_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  FP contraction is off so every fp32 step of the accept
    rule is one IEEE operation."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("arch", "dtype", "n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab",
                 "max_batch", "max_seq", "max_block", "enc_len")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.csdo_kv_bytes.restype = C.c_size_t
        _lib.csdo_threads.restype = C.c_int32
        for name in ("csdo_model_create", "csdo_model_destroy", "csdo_kv_write", "csdo_kv_read",
                     "csdo_verify_block", "csdo_bigram_fit", "csdo_bigram_draft", "csdo_accept",
                     "csdo_cross_kv_init", "csdo_rel_bucket"):
            getattr(_lib, name).restype = C.c_int32
        for name in ("csdo_set_trace", "csdo_rmsnorm", "csdo_rope", "csdo_softmax", "csdo_probs_f32"):
            getattr(_lib, name).restype = None
    return _lib


def threads() -> int:
    return int(lib().csdo_threads())


def _p(a, ctype=None):
    if a is None:
        return None
    return a.ctypes.data_as(C.c_void_p)


def _chk(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what} failed with status {rc}")


def _as_host(w):
    """numpy view of a weight: fp32 array, or uint16 array holding bf16 bit patterns."""
    if isinstance(w, np.ndarray):
        return np.ascontiguousarray(w)
    import torch  # weights usually arrive as CPU torch tensors from the input generator
    t = w.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


class Model:
    """Borrowed-weight oracle model with its own fp64 KV cache."""

    def __init__(self, shape, weights, max_batch=1, max_seq=64, max_block=32):
        dtype = 1 if shape.dtype == "bf16" else 0
        self.shape = shape
        self.cfg = Cfg(shape.arch, dtype, shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim,
                       shape.d_ffn, shape.vocab, max_batch, max_seq, max_block, getattr(shape, "enc_len", 0),
                       shape.rms_eps, shape.rope_theta)
        self._w = [_as_host(w) for w in weights]
        for i, a in enumerate(self._w):
            bias_table = shape.arch == 1 and i == len(self._w) - 1      # relative-position bias stays fp32
            want = np.uint16 if (dtype == 1 and a.ndim == 2 and not bias_table) else np.float32
            if a.dtype != want:
                raise TypeError(f"weight dtype {a.dtype}, expected {want}")
        arr = (C.c_void_p * len(self._w))(*[a.ctypes.data for a in self._w])
        self._h = C.c_void_p()
        _chk(lib().csdo_model_create(C.byref(self.cfg), arr, len(self._w), C.byref(self._h)), "model_create")
        n = lib().csdo_kv_bytes(self._h) // 8
        self.kv = np.zeros(n, dtype=np.float64)
        self._trace = None

    def __del__(self):
        try:
            if getattr(self, "_h", None):
                lib().csdo_model_destroy(self._h)
                self._h = None
        except Exception:      # interpreter shutdown
            pass

    def reset_cache(self):
        self.kv[:] = 0.0

    def kv_write(self, layer, b, pos0, K, V):
        K = np.ascontiguousarray(K, dtype=np.float32)
        V = np.ascontiguousarray(V, dtype=np.float32)
        _chk(lib().csdo_kv_write(self._h, _p(self.kv), layer, b, pos0, K.shape[0], _p(K), _p(V)), "kv_write")

    def kv_read(self, layer, b, pos0, n):
        hd = self.shape.n_heads * self.shape.head_dim
        K = np.empty((n, hd), dtype=np.float64)
        V = np.empty((n, hd), dtype=np.float64)
        _chk(lib().csdo_kv_read(self._h, _p(self.kv), layer, b, pos0, n, _p(K), _p(V)), "kv_read")
        return K, V

    def cross_kv_init(self, enc_out):
        """arch 1: enc_out [B][enc_len][d] -> cross-attention keys/values of every layer, in the cache."""
        x = np.ascontiguousarray(enc_out, dtype=np.float32)
        _chk(lib().csdo_cross_kv_init(self._h, _p(self.kv), _p(x), x.shape[0]), "cross_kv_init")

    def verify_tree(self, tokens, parent, cache_len, temperature=1.0, want_probs=False):
        """Tree block (Section 5.1, Appendix B): tokens, parent [B][m] int32 (parent[b][0] = -1, parent[b][i] < i)
        -> logits [B][m][V] fp64 (and probs); row i is stored at cache row cache_len + i."""
        return self.verify_block(tokens, cache_len, temperature, want_probs, parent=parent)

    def tree_commit(self, b, cache_len, path):
        """Move the K/V of the kept rows path (increasing, below row 0) to cache rows cache_len + 1 ..."""
        path = np.ascontiguousarray(path, dtype=np.int32)
        _chk(lib().csdo_tree_commit(self._h, _p(self.kv), b, int(cache_len), _p(path), len(path)), "tree_commit")

    def verify_block(self, tokens, cache_len, temperature=1.0, want_probs=False, trace=False, parent=None):
        """tokens [B][m] int32, cache_len [B] -> logits [B][m][V] fp64 (and probs)."""
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        cache_len = np.ascontiguousarray(cache_len, dtype=np.int32)
        B, m = tokens.shape
        V = self.shape.vocab
        logits = np.empty((B, m, V), dtype=np.float64)
        probs = np.empty((B, m, V), dtype=np.float64) if want_probs else None
        tr = None
        if trace:
            tr = np.zeros((self.shape.n_layers + 1, m, self.shape.d_model), dtype=np.float64)
            lib().csdo_set_trace(self._h, _p(tr))
        if parent is not None:
            parent = np.ascontiguousarray(parent, dtype=np.int32).reshape(B, m)
            rc = lib().csdo_verify_tree(self._h, _p(self.kv), _p(tokens), _p(parent), _p(cache_len), B, m,
                                        C.c_double(temperature), _p(logits), _p(probs))
        else:
            rc = lib().csdo_verify_block(self._h, _p(self.kv), _p(tokens), _p(cache_len), B, m,
                                         C.c_double(temperature), _p(logits), _p(probs))
        if trace:
            lib().csdo_set_trace(self._h, None)
        _chk(rc, "verify_block")
        out = [logits]
        if want_probs:
            out.append(probs)
        if trace:
            out.append(tr)
        return out[0] if len(out) == 1 else tuple(out)


def probs_f32(logits, temperature=1.0):
    logits = np.ascontiguousarray(logits, dtype=np.float64)
    V = logits.shape[-1]
    rows = logits.size // V
    p = np.empty(logits.shape, dtype=np.float32)
    lib().csdo_probs_f32(_p(logits), rows, V, C.c_double(temperature), _p(p))
    return p


def bigram_fit(tokens, vocab, next_table):
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    table = np.array(next_table, dtype=np.int32, copy=True)
    _chk(lib().csdo_bigram_fit(_p(tokens), tokens.shape[0], vocab, _p(table)), "bigram_fit")
    return table


def bigram_draft(ctx, ctx_len, next_table, k, max_match=0):
    ctx = np.ascontiguousarray(ctx, dtype=np.int32)
    if ctx.ndim == 1:
        ctx = ctx[None, :]
    ctx_len = np.ascontiguousarray(ctx_len, dtype=np.int32).reshape(-1)
    table = np.ascontiguousarray(next_table, dtype=np.int32)
    B, stride = ctx.shape
    out = np.empty((B, k), dtype=np.int32)
    mlen = np.empty(B, dtype=np.int32)
    _chk(lib().csdo_bigram_draft(_p(ctx), _p(ctx_len), B, stride, _p(table), table.shape[0], k,
                                 max_match, _p(out), _p(mlen)), "bigram_draft")
    return out, mlen


def maxgram_draft(haystack, haystack_len, needle, needle_len, next_table, k, max_match=0):
    """Max-Gram with a separate haystack -> (tokens [B][k], match_len [B], n_copied [B])."""
    hay = np.ascontiguousarray(haystack, dtype=np.int32)
    ned = np.ascontiguousarray(needle, dtype=np.int32)
    if hay.ndim == 1:
        hay = hay[None, :]
    if ned.ndim == 1:
        ned = ned[None, :]
    hl = np.ascontiguousarray(haystack_len, dtype=np.int32).reshape(-1)
    nl = np.ascontiguousarray(needle_len, dtype=np.int32).reshape(-1)
    table = np.ascontiguousarray(next_table, dtype=np.int32)
    B = ned.shape[0]
    out = np.empty((B, k), dtype=np.int32)
    mlen = np.empty(B, dtype=np.int32)
    ncp = np.empty(B, dtype=np.int32)
    _chk(lib().csdo_maxgram_draft(_p(hay), _p(hl), hay.shape[1], _p(ned), _p(nl), ned.shape[1], B, _p(table),
                                  table.shape[0], k, max_match, _p(out), _p(mlen), _p(ncp)), "maxgram_draft")
    return out, mlen, ncp


def accept(p, q, draft, u_acc, u_samp, lenience=1.0, mode=0, q_onehot=None):
    """p [B][k+1][V] fp32, q [B][k][V] fp32 or None, draft [B][k] -> (n_accepted [B], next_token [B])."""
    p = np.ascontiguousarray(p, dtype=np.float32)
    B, k1, V = p.shape
    k = k1 - 1
    q = None if q is None else np.ascontiguousarray(q, dtype=np.float32)
    draft = np.ascontiguousarray(draft, dtype=np.int32).reshape(B, k)
    u_acc = np.ascontiguousarray(u_acc, dtype=np.float32).reshape(B, k)
    u_samp = np.ascontiguousarray(u_samp, dtype=np.float32).reshape(B)
    oh = None if q_onehot is None else np.ascontiguousarray(q_onehot, dtype=np.uint8)
    n_acc = np.empty(B, dtype=np.int32)
    nxt = np.empty(B, dtype=np.int32)
    _chk(lib().csdo_accept(_p(p), _p(q), _p(oh), _p(draft), _p(u_acc), _p(u_samp), B, k, V,
                           C.c_float(lenience), mode, _p(n_acc), _p(nxt)), "accept")
    return n_acc, nxt


def tree_accept(p, tokens, parent, u, mode=0):
    """p [B][m][V] fp32, tokens, parent [B][m], u [B][m] -> (n_accepted [B], path [B][m], next_token [B])."""
    p = np.ascontiguousarray(p, dtype=np.float32)
    B, m, V = p.shape
    tokens = np.ascontiguousarray(tokens, dtype=np.int32).reshape(B, m)
    parent = np.ascontiguousarray(parent, dtype=np.int32).reshape(B, m)
    u = np.ascontiguousarray(u, dtype=np.float32).reshape(B, m)
    n_acc = np.empty(B, dtype=np.int32)
    path = np.full((B, m), -1, dtype=np.int32)
    nxt = np.empty(B, dtype=np.int32)
    _chk(lib().csdo_tree_accept(_p(p), _p(tokens), _p(parent), _p(u), B, m, V, mode, _p(n_acc), _p(path), _p(nxt)),
         "tree_accept")
    return n_acc, path, nxt


def rel_bucket(n):
    """Bucket of the arch-1 relative-position bias for the distance n = query position - key position."""
    return int(lib().csdo_rel_bucket(int(n)))


def rmsnorm(x, g, eps):
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = np.ascontiguousarray(g, dtype=np.float32)
    y = np.empty_like(x)
    lib().csdo_rmsnorm(_p(x), _p(g), x.shape[0], C.c_double(eps), _p(y))
    return y


def rope(x, pos, theta=10000.0):
    y = np.array(x, dtype=np.float64, copy=True)
    lib().csdo_rope(_p(y), y.shape[0], int(pos), C.c_double(theta))
    return y


def softmax(logits, temperature=1.0):
    x = np.ascontiguousarray(logits, dtype=np.float64)
    p = np.empty_like(x)
    lib().csdo_softmax(_p(x), x.shape[0], C.c_double(1.0 / temperature), _p(p))
    return p


def accept_margins(p, q, draft, u_acc, u_samp, lenience=1.0, mode=0, q_onehot=None):
    """How far each decision of accept() on sequence 0 is from flipping (plain Python over the same rule,
    Section 2 / 3.1), for comparisons between implementations whose probabilities differ within a tolerance:
      tests: list of (accepted, |u q(x) - l p(x)| / (l p(x))) for every acceptance test that was evaluated;
      draw:  distance of the draw's threshold to the nearest boundary of the chosen token's CDF interval, as a
             fraction of the total weight (sampling), or the gap between the two largest entries of the row (greedy).
    Returns (n_accepted, next_token, tests, draw)."""
    p = np.asarray(p, dtype=np.float32)
    _, k1, V = p.shape
    k = k1 - 1
    lf = np.float32(lenience)
    tests = []
    n = 0
    if mode == 1:
        for i in range(k):
            top2 = np.sort(p[0, i])[-2:]
            ok = int(draft[0][i]) == int(np.argmax(p[0, i]))
            tests.append((ok, float(top2[1] - top2[0])))
            if not ok:
                break
            n += 1
        row = p[0, n]
        top2 = np.sort(row)[-2:]
        return n, int(np.argmax(row)), tests, float(top2[1] - top2[0])
    for i in range(k):
        x = int(draft[0][i])
        dense = q is not None and not (q_onehot is not None and q_onehot[i])
        qx = np.float32(q[0, i, x]) if dense else np.float32(1.0)
        lhs = np.float32(np.float32(u_acc[0][i]) * qx)
        rhs = np.float32(lf * p[0, i, x])
        ok = bool(lhs < rhs)
        tests.append((ok, float(abs(float(lhs) - float(rhs)) / max(float(rhs), 1e-30))))
        if not ok:
            break
        n += 1
    row = p[0, n].astype(np.float32)
    if n < k:
        x = int(draft[0][n])
        dense = q is not None and not (q_onehot is not None and q_onehot[n])
        qrow = q[0, n].astype(np.float32) if dense else np.eye(V, dtype=np.float32)[x]
        r = np.maximum(np.float32(0), (lf * row).astype(np.float32) - qrow).astype(np.float32)
        if not (r > 0).any():
            r = row
    else:
        r = row
    w = np.floor(r.astype(np.float64) * 2.0 ** 40)
    Z = w.sum()
    T = np.floor(np.floor(float(u_samp[0]) * 2.0 ** 24) * Z / 2.0 ** 24)
    cum = np.cumsum(w)
    tok = int(np.searchsorted(cum, T, side="right"))
    lo = cum[tok - 1] if tok > 0 else 0.0
    return n, tok, tests, float(min(T - lo, cum[tok] - T) / Z)
