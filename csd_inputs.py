"""Seeded synthetic inputs for the Cascade-Speculative-Drafting verify path.

This module only *generates inputs* (model shapes, weights, token ids, uniforms,
cache contents).  It holds none of the method's arithmetic and is the one module
that both the CPU oracle's tests and the HIP path's tests / bench may import.

Everything is produced by a counter-based generator (the splitmix64 sequence,
evaluated element-wise with integer tensor ops), so the same bits come out on a
CPU and on a GPU, in any chunking.  "Normal" values are a variance-matched
Irwin-Hall sum of the four 16-bit fields of one 64-bit draw (support +-3.46 sigma):
integer-exact up to one final fp32 multiply, hence reproducible bit for bit.

The paper runs trained Vicuna-7B / vicuna-68m / FLAN-T5 checkpoints on GSM8K and
MMLU prompts (Section 5.1, Implementation Details); none of those exist here, so
random-init models of the same shapes and synthetic token streams stand in.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, asdict

import torch

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(x: int) -> int:
    """uint64 bit pattern -> the signed python int torch.int64 wants."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def splitmix64_scalar(state: int) -> int:
    """One output of the splitmix64 generator for the (already advanced) state."""
    z = state & _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def stream_base(seed: int, stream: int) -> int:
    """Start state of the sub-stream `stream` of `seed`."""
    return splitmix64_scalar((seed * 0x100000001B3 + stream * _GOLDEN + 0x1234567) & _M64)


def raw_bits(n: int, seed: int, stream: int, device="cpu", offset: int = 0) -> torch.Tensor:
    """n consecutive splitmix64 outputs (as int64 bit patterns) of a sub-stream."""
    base = stream_base(seed, stream)
    out = torch.empty(n, dtype=torch.int64, device=device)
    chunk = 1 << 24
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        i = torch.arange(lo + offset + 1, hi + offset + 1, dtype=torch.int64, device=device)
        out[lo:hi] = _mix(i * _s64(_GOLDEN) + _s64(base))
    return out


_IH_STD = math.sqrt(4.0 * ((1 << 32) - 1) / 12.0)


def normal(shape, std: float, seed: int, stream: int, device="cpu") -> torch.Tensor:
    """fp32 tensor of approximately N(0, std^2) values (Irwin-Hall of 4x16 bit)."""
    n = 1
    for s in shape:
        n *= s
    out = torch.empty(n, dtype=torch.float32, device=device)
    scale = torch.tensor(std / _IH_STD, dtype=torch.float32, device=device)
    chunk = 1 << 24
    base = stream_base(seed, stream)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        i = torch.arange(lo + 1, hi + 1, dtype=torch.int64, device=device)
        r = _mix(i * _s64(_GOLDEN) + _s64(base))
        s = (r & 0xFFFF) + (_lsr(r, 16) & 0xFFFF) + (_lsr(r, 32) & 0xFFFF) + _lsr(r, 48)
        out[lo:hi] = (s - 131070).to(torch.float32) * scale
    return out.reshape(shape)


def token_ids(n: int, vocab: int, seed: int, stream: int, device="cpu") -> torch.Tensor:
    """n ids uniform over [0, vocab) as int32."""
    r = raw_bits(n, seed, stream, device)
    return (_lsr(r, 33) % vocab).to(torch.int32)


def uniforms(n: int, seed: int, stream: int, device="cpu") -> torch.Tensor:
    """n fp32 uniforms in [0,1), each exactly j * 2^-24."""
    r = raw_bits(n, seed, stream, device)
    return _lsr(r, 40).to(torch.float32) * (2.0 ** -24)


def repeat_stream(n: int, vocab: int, seed: int, stream: int,
                  p_copy: float = 0.3, mean_span: float = 6.0, zipf_a: float = 1.1) -> torch.Tensor:
    """Token stream with planted repeats (CPU, int32).

    Section 3.3's premise is that phrases of the prompt recur in the generation;
    uniform ids almost never repeat at vocab 32000, so this stream draws Zipf-like
    unigrams and, with probability p_copy at a position, starts copying a span
    (geometric length, mean mean_span) from a uniformly chosen earlier offset.
    """
    r = raw_bits(3 * n, seed, stream).tolist()
    u = [((x >> 11) & ((1 << 53) - 1)) / float(1 << 53) for x in r]
    # Zipf-like ranks by inverse transform of a Pareto tail, clipped to the vocab
    out = []
    i = 0
    while len(out) < n:
        u0, u1, u2 = u[3 * i], u[3 * i + 1], u[3 * i + 2]
        i += 1
        if len(out) >= 4 and u0 < p_copy:
            src = int(u1 * (len(out) - 1))
            span = 1 + int(math.log(max(u2, 1e-12)) / math.log(1.0 - 1.0 / mean_span))
            for j in range(span):
                if len(out) >= n:
                    break
                out.append(out[src + j] if src + j < len(out) else out[-1])
        else:
            rank = int((1.0 - u1) ** (-1.0 / zipf_a)) - 1
            out.append(rank % vocab)
        if i >= n:
            break
    while len(out) < n:
        out.append(out[len(out) % max(1, len(out) // 2)])
    return torch.tensor(out[:n], dtype=torch.int32)


def default_next_table(vocab: int, seed: int, device="cpu") -> torch.Tensor:
    """Default bigram successor table: next[v] = hash(seed, v) mod vocab (int32)."""
    return token_ids(vocab, vocab, seed, 0xB16A, device)


# --------------------------------------------------------------------------- models

@dataclass
class ModelShape:
    name: str
    arch: int          # 0: LLaMA-style (RMSNorm, RoPE, SwiGLU); 1: T5-style decoder (relative bias, cross-attention, gated GELU)
    dtype: str         # "fp32" | "bf16"  (weights and KV cache)
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    enc_len: int = 0   # arch 1: rows of the encoder output the decoder cross-attends

    def n_weights(self) -> int:
        return 3 + 9 * self.n_layers if self.arch == 0 else 4 + 14 * self.n_layers

    def streamed_params(self) -> int:
        """Matrix elements one review forward reads (the embedding is gathered, not streamed; the
        cross-attention key/value projections run once per prompt, not per step)."""
        d, f, v, L = self.d_model, self.d_ffn, self.vocab, self.n_layers
        hd = self.n_heads * self.head_dim
        if self.arch == 0:
            return L * (4 * d * hd + 3 * d * f) + d * v
        return L * (6 * d * hd + 3 * d * f) + d * v

    def as_dict(self):
        return asdict(self)


TINY = ModelShape("tiny", 0, "fp32", 2, 64, 4, 16, 256, 512)
DRAFT_160M = ModelShape("draft160m", 0, "bf16", 12, 768, 12, 64, 3072, 32000)
TARGET_7B = ModelShape("target7b", 0, "bf16", 32, 4096, 32, 128, 11008, 32000)
T5_TINY = ModelShape("t5tiny", 1, "fp32", 2, 64, 4, 16, 128, 512, rms_eps=1e-6, enc_len=24)
T5XXL_DEC = ModelShape("t5xxl_dec", 1, "bf16", 24, 4096, 64, 64, 10240, 32128, rms_eps=1e-6, enc_len=512)

# Workloads named after the benchmark configurations: batch, cached prefix, drafted tokens.
WORKLOADS = {
    "tiny":        dict(shape=TINY, B=1, prefix=32, k=4, seed=0xC5D00001),
    "draft160m":   dict(shape=DRAFT_160M, B=1, prefix=512, k=8, seed=0xC5D00002),
    "target7b":    dict(shape=TARGET_7B, B=1, prefix=1024, k=5, seed=0xC5D00003),
    # drafts of this configuration are sampled from the reviewer's own distributions perturbed by seeded
    # noise so that a draft is accepted with probability about 0.6 (bench.py builds them at setup)
    "target7b_b8": dict(shape=TARGET_7B, B=8, prefix=2048, k=16, seed=0xC5D00003, draft="target_mix", acceptance=0.6),
    "t5xxl":       dict(shape=T5XXL_DEC, B=1, prefix=256, k=4, seed=0xC5D00004),
}


REL_BUCKETS = 32     # rows of the relative-position bias table of an arch-1 model


def weight_names(shape: ModelShape):
    names = ["embed"]
    per_layer = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down") if shape.arch == 0 else \
                ("self_norm", "wq", "wk", "wv", "wo", "cross_norm", "cq", "ck", "cv", "co", "ffn_norm", "w0", "w1", "w_out")
    for l in range(shape.n_layers):
        names += [f"l{l}.{w}" for w in per_layer]
    names += ["final_norm", "lm_head"]
    if shape.arch == 1:
        names.append("rel_bias")
    return names


def weight_shapes(shape: ModelShape):
    d, f, v = shape.d_model, shape.d_ffn, shape.vocab
    hd = shape.n_heads * shape.head_dim
    if shape.arch == 0:
        per_layer = [(d,), (d, hd), (d, hd), (d, hd), (hd, d), (d,), (d, f), (d, f), (f, d)]
        return [(v, d)] + per_layer * shape.n_layers + [(d,), (d, v)]
    per_layer = [(d,), (d, hd), (d, hd), (d, hd), (hd, d), (d,), (d, hd), (d, hd), (d, hd), (hd, d),
                 (d,), (d, f), (d, f), (f, d)]
    return [(v, d)] + per_layer * shape.n_layers + [(d,), (d, v), (REL_BUCKETS, shape.n_heads)]


def make_weights(shape: ModelShape, seed: int, device="cpu", std: float = 0.02):
    """Canonical-order weight list.  Matrices are row-major [in][out] in the model
    dtype (bf16 = round-to-nearest-even of the fp32 draw); norm gains are fp32 ones."""
    out = []
    names = weight_names(shape)
    for idx, shp in enumerate(weight_shapes(shape)):
        if len(shp) == 1:
            out.append(torch.ones(shp, dtype=torch.float32, device=device))
            continue
        s_w = std
        if shape.arch == 1 and names[idx].endswith((".wq", ".cq")):
            # T5 attention has no 1/sqrt(head_dim) factor: the family folds it into the initialisation of the
            # query projections.  Without it a random-init model's softmaxes are near one-hot and rounding
            # differences double per layer, so no finite-precision forward could be compared at full depth.
            s_w = std / float(shape.head_dim) ** 0.5
        w = normal(shp, s_w, seed, 0x1000 + idx, device)
        if shape.dtype == "bf16" and names[idx] != "rel_bias":     # the small bias table stays fp32
            w = w.to(torch.bfloat16)
        out.append(w.contiguous())
    return out


def encoder_output(shape: ModelShape, B: int, seed: int, device="cpu", std: float = 1.0):
    """Seeded stand-in for the encoder's final hidden states [B][enc_len][d] of an arch-1 model (fp32
    holding values exact in the model dtype)."""
    x = normal((B, shape.enc_len, shape.d_model), std, seed, 0x300000, device)
    if shape.dtype == "bf16":
        x = x.to(torch.bfloat16).to(torch.float32)
    return x.contiguous()


def synthetic_kv(shape: ModelShape, n_rows: int, seed: int, layer: int, b: int, device="cpu",
                 std: float = 1.0):
    """Seeded stand-in K and V rows [n_rows][H*dh] (fp32 holding values exact in the
    cache dtype) for filling a cache at sizes where a real prefill is too slow."""
    hd = shape.n_heads * shape.head_dim
    k = normal((n_rows, hd), std, seed, 0x200000 + (layer * 64 + b) * 2, device)
    v = normal((n_rows, hd), std, seed, 0x200000 + (layer * 64 + b) * 2 + 1, device)
    if shape.dtype == "bf16":
        k = k.to(torch.bfloat16).to(torch.float32)
        v = v.to(torch.bfloat16).to(torch.float32)
    return k, v
