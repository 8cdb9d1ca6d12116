"""Counter-based seeded generators for model weights and prompts.

Every number is a pure function of (seed, tensor id, element index), so any
tensor (or any slice of one) can be regenerated independently, on any device,
with bit-identical results: the hash uses only wrapping 64-bit integer
arithmetic, and the Gaussian transform is a sum of eight 16-bit uniforms
(Irwin-Hall) scaled by one float32 multiplication - no libm call anywhere.

The shapes, seeds and value distributions are those of the five synthetic
workloads that stand in for the paper's trained 1.3B / 7B models and HELM
prompts (Section 5.2 and Appendix B of the paper use trained weights and text,
neither of which is available): uniform-random token ids and Gaussian weights
whose head scale spreads max-softmax confidences over (0, 1).

This file contains no transformer arithmetic.  Both the CPU oracle's tests and
the HIP library's tests / benchmark draw their inputs from here.
"""
from __future__ import annotations

import enum
import math
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import torch

_M64 = (1 << 64) - 1


def _s64(c: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 holds for it."""
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes (torch's >> is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    """A 64-bit finalizer (xor-shift-multiply, three rounds); bijective."""
    x = (x ^ _lsr(x, 30)) * _s64(0xBF58476D1CE4E5B9)
    x = (x ^ _lsr(x, 27)) * _s64(0x94D049BB133111EB)
    return x ^ _lsr(x, 31)


def _mix64_int(x: int) -> int:
    x &= _M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M64
    return x ^ (x >> 31)


def _stream_base(seed: int, tid: int) -> int:
    """Start counter of the stream for (seed, tensor id)."""
    return _mix64_int(_mix64_int(seed * 0x9E3779B97F4A7C15 + 0x1234567) + tid * 0xD1B54A32D192ED03)


_IH_STD = math.sqrt(8.0 * (65536.0 ** 2 - 1.0) / 12.0)  # std of the sum of eight uniform{0..65535}
_CHUNK = 1 << 24


def _hash_chunk(base: int, start: int, n: int, device) -> Tuple[torch.Tensor, torch.Tensor]:
    idx = torch.arange(start, start + n, dtype=torch.int64, device=device)
    k = idx + _s64(base)
    h1 = _mix64(k)
    h2 = _mix64(k ^ _s64(0xA5A5A5A5DEADBEEF))
    return h1, h2


def gaussian_tensor(seed: int, tid: int, numel: int, sigma: float, mean: float = 0.0,
                    device="cpu", start: int = 0) -> torch.Tensor:
    """float32[numel]: element i = mean + sigma * z_i, z_i approximately N(0,1).

    z_i = (u_0 + ... + u_7 - 4*65535) / std, the u_j being the eight 16-bit
    fields of two 64-bit hashes of (seed, tid, start + i).  |z| <= 4.9.
    """
    base = _stream_base(seed, tid)
    out = torch.empty(numel, dtype=torch.float32, device=device)
    scale = torch.tensor(sigma / _IH_STD, dtype=torch.float32, device=device)
    for c0 in range(0, numel, _CHUNK):
        n = min(_CHUNK, numel - c0)
        h1, h2 = _hash_chunk(base, start + c0, n, device)
        s = torch.zeros(n, dtype=torch.int64, device=device)
        for h in (h1, h2):
            for sh in (0, 16, 32, 48):
                s += _lsr(h, sh) & 0xFFFF
        s -= 4 * 65535
        v = s.to(torch.float32) * scale          # one exact-rounded fp32 multiply
        if mean != 0.0:
            v = v + torch.tensor(mean, dtype=torch.float32, device=device)
        out[c0:c0 + n] = v
    return out


def to_numpy(t: torch.Tensor):
    """float32 -> float32 array; bfloat16 -> uint16 array of the same bit patterns (numpy has no bfloat16)."""
    import numpy as np

    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def uniform_ints(seed: int, tid: int, numel: int, lo: int, hi: int, device="cpu") -> torch.Tensor:
    """int64[numel], uniform in [lo, hi) (modulo bias < 2^-40, irrelevant here)."""
    base = _stream_base(seed, tid)
    h1, _ = _hash_chunk(base, 0, numel, device)
    return lo + (_lsr(h1, 8) % (hi - lo))


class TensorKind(enum.IntEnum):
    EMBED = 0        # [vocab][d]
    ATTN_NORM = 1    # [d]      per layer, RMSNorm gain before attention
    WQ = 2           # [d][d]   per layer, y = W x  (row = output feature)
    WK = 3
    WV = 4
    WO = 5
    MLP_NORM = 6     # [d]
    WG = 7           # [d_ff][d]
    WU = 8           # [d_ff][d]
    WD = 9           # [d][d_ff]
    EXIT_NORM = 10   # [d]      per exit
    EXIT_HEAD = 11   # [vocab][d] per exit
    FINAL_NORM = 12  # [d]
    FINAL_HEAD = 13  # [vocab][d]
    EXIT_MLP_NORM = 14  # [d]        per exit, only with an MLP in the exit (gain of the norm in front of it)
    EXIT_WG = 15        # [d_ff][d]  per exit
    EXIT_WU = 16        # [d_ff][d]
    EXIT_WD = 17        # [d][d_ff]
    # a complete Transformer layer in the exit: the four kinds above are its MLP half, these its attention half
    EXIT_ATTN_NORM = 18  # [d]     per exit
    EXIT_WQ = 19         # [d][d]  per exit
    EXIT_WK = 20
    EXIT_WV = 21
    EXIT_WO = 22


_NORMS = (TensorKind.ATTN_NORM, TensorKind.MLP_NORM, TensorKind.EXIT_NORM, TensorKind.FINAL_NORM, TensorKind.EXIT_MLP_NORM,
          TensorKind.EXIT_ATTN_NORM)
_HEADS = (TensorKind.EXIT_HEAD, TensorKind.FINAL_HEAD)


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    exit_layers: Tuple[int, ...]          # 1-based "after layer e", ascending, < n_layers
    dtype: str = "bf16"                   # "f32" | "bf16" (storage of matrices / embedding)
    sigma: float = 0.02                   # std of embedding and layer matrices
    head_sigma: float = 0.3               # std of exit / final heads
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    # structure of the exits (Section 2: an output embedding matrix, an optional normalisation in front of it,
    # optionally an MLP before that; input and output embeddings tied or untied)
    exit_norm: bool = True                # RMSNorm in front of each exit's output embedding
    tie_embeddings: bool = False          # every exit and the final head use the input embedding matrix
    exit_mlp: bool = False                # each exit starts with an MLP block of its own (same form as a layer's)
    exit_layer: bool = False              # each exit starts with a complete Transformer layer of its own (not with exit_mlp)
    exit_head_sigma: Tuple[float, ...] = ()  # std of each exit's own head, where it differs from head_sigma (untied heads)

    @property
    def exit_flags(self) -> int:
        return ((0 if self.exit_norm else 1) | (2 if self.tie_embeddings else 0) | (4 if self.exit_mlp else 0)
                | (8 if self.exit_layer else 0))

    def tensor_shape(self, kind: TensorKind) -> Tuple[int, ...]:
        d, f, v = self.d_model, self.d_ff, self.vocab
        return {
            TensorKind.EMBED: (v, d), TensorKind.ATTN_NORM: (d,), TensorKind.WQ: (d, d),
            TensorKind.WK: (d, d), TensorKind.WV: (d, d), TensorKind.WO: (d, d),
            TensorKind.MLP_NORM: (d,), TensorKind.WG: (f, d), TensorKind.WU: (f, d),
            TensorKind.WD: (d, f), TensorKind.EXIT_NORM: (d,), TensorKind.EXIT_HEAD: (v, d),
            TensorKind.FINAL_NORM: (d,), TensorKind.FINAL_HEAD: (v, d),
            TensorKind.EXIT_MLP_NORM: (d,), TensorKind.EXIT_WG: (f, d), TensorKind.EXIT_WU: (f, d),
            TensorKind.EXIT_WD: (d, f), TensorKind.EXIT_ATTN_NORM: (d,), TensorKind.EXIT_WQ: (d, d),
            TensorKind.EXIT_WK: (d, d), TensorKind.EXIT_WV: (d, d), TensorKind.EXIT_WO: (d, d),
        }[TensorKind(kind)]

    def n_params(self) -> int:
        n = 0
        for kind, _ in model_tensor_list(self):
            n += math.prod(self.tensor_shape(kind))
        return n


def _head_sigma(d: int) -> float:
    return 0.3 / math.sqrt(d / 128.0)


@dataclass(frozen=True)
class Workload:
    shape: ModelShape
    batch: int
    prompt_len: Tuple[int, int]           # (lo, hi) inclusive; lo == hi for fixed length
    new_tokens: int
    thresholds: Tuple[float, ...]
    weight_seed: int = 0
    prompt_seed: int = 1
    length_seed: int = 2
    note: str = ""


CONFIGS: Dict[str, Workload] = {
    "C1": Workload(ModelShape(4, 128, 4, 32, 352, 1024, (1, 2), "f32", 0.02, 0.3),
                   1, (16, 16), 32, (0.0, 0.5, 0.8, 1.0), note="tiny fp32"),
    "C2": Workload(ModelShape(24, 2048, 16, 128, 5504, 50304, (6, 12), "bf16", 0.02, _head_sigma(2048)),
                   1, (512, 512), 256, (0.8, 1.0), note="1.3B-shaped"),
    "C3": Workload(ModelShape(32, 4096, 32, 128, 11008, 50304, (8, 16), "bf16", 0.02, _head_sigma(4096)),
                   1, (1024, 1024), 256, (0.2, 0.4, 0.6, 0.8, 1.0), note="7B-shaped"),
    "C4": Workload(ModelShape(32, 4096, 32, 128, 11008, 50304, (8, 16), "bf16", 0.02, _head_sigma(4096)),
                   16, (256, 2048), 256, (0.6,), note="7B-shaped, ragged batch 16"),
    "C5": Workload(ModelShape(60, 6656, 52, 128, 17920, 50304, (15, 30), "bf16", 0.02, _head_sigma(6656)),
                   4, (2048, 2048), 512, (0.5, 0.8, 1.0), note="30B-shaped"),
}


# Multipliers of the exit heads' std (first exit, second exit) of the 7B-shaped model under which, at threshold 0.8, the
# seeded model leaves about 7 of 18 tokens at the first exit, 1 of the remaining 11 at the second and sends the rest
# to full depth: the exit mix of the one generation the paper tabulates token by token (Table 4).  Found by a sweep
# of the multiplier on the GPU (fraction of head evaluations with confidence >= 0.8: 0.41 at 3.0, 0.09 at 1.5).
TABLE4_EXIT_HEAD_SCALE = (3.0, 1.5)


def model_tensor_list(shape: ModelShape) -> List[Tuple[TensorKind, int]]:
    """(kind, index) of every tensor of a model, in canonical order."""
    out: List[Tuple[TensorKind, int]] = [(TensorKind.EMBED, 0)]
    for l in range(shape.n_layers):
        for k in (TensorKind.ATTN_NORM, TensorKind.WQ, TensorKind.WK, TensorKind.WV, TensorKind.WO,
                  TensorKind.MLP_NORM, TensorKind.WG, TensorKind.WU, TensorKind.WD):
            out.append((k, l))
    for i in range(len(shape.exit_layers)):
        if shape.exit_layer:
            for k in (TensorKind.EXIT_ATTN_NORM, TensorKind.EXIT_WQ, TensorKind.EXIT_WK, TensorKind.EXIT_WV, TensorKind.EXIT_WO):
                out.append((k, i))
        if shape.exit_mlp or shape.exit_layer:
            for k in (TensorKind.EXIT_MLP_NORM, TensorKind.EXIT_WG, TensorKind.EXIT_WU, TensorKind.EXIT_WD):
                out.append((k, i))
        if shape.exit_norm:
            out.append((TensorKind.EXIT_NORM, i))
        if not shape.tie_embeddings:
            out.append((TensorKind.EXIT_HEAD, i))
    out.append((TensorKind.FINAL_NORM, 0))
    if not shape.tie_embeddings:
        out.append((TensorKind.FINAL_HEAD, 0))
    return out


def model_tensor(shape: ModelShape, kind: TensorKind, index: int, seed: int = 0, device="cpu",
                 gain_jitter: float = 0.0) -> torch.Tensor:
    """One tensor of the seeded model.

    Matrices and the embedding come back in the model's storage dtype (for
    "bf16": the round-to-nearest-even bf16 of the generated fp32 value); norm
    gains are always fp32 and equal 1 unless ``gain_jitter`` > 0 (then
    1 + gain_jitter * z, used by tests so that a misplaced gain is visible).
    """
    kind = TensorKind(kind)
    dims = shape.tensor_shape(kind)
    numel = math.prod(dims)
    if kind < TensorKind.EXIT_MLP_NORM:
        tid = int(kind) + 16 * index
    elif kind < TensorKind.EXIT_ATTN_NORM:
        tid = 100000 + (int(kind) - 14) + 4 * index
    else:
        tid = 200000 + (int(kind) - 18) + 8 * index
    if kind in _NORMS:
        if gain_jitter == 0.0:
            return torch.ones(dims, dtype=torch.float32, device=device)
        return gaussian_tensor(seed, tid, numel, gain_jitter, 1.0, device).reshape(dims)
    sigma = shape.head_sigma if kind in _HEADS or (kind == TensorKind.EMBED and shape.tie_embeddings) else shape.sigma
    if kind == TensorKind.EXIT_HEAD and shape.exit_head_sigma:
        sigma = shape.exit_head_sigma[index]
    t = gaussian_tensor(seed, tid, numel, sigma, 0.0, device).reshape(dims)
    if shape.dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t


def prompt_tokens(vocab: int, n: int, seed: int = 1, device="cpu") -> torch.Tensor:
    """int32[n] token ids uniform in [0, vocab)."""
    return uniform_ints(seed, 1000, n, 0, vocab, device).to(torch.int32)


def prompt_lengths(n_seqs: int, lo: int, hi: int, seed: int = 2) -> List[int]:
    """Prompt lengths uniform in [lo, hi] (inclusive)."""
    return [int(v) for v in uniform_ints(seed, 1001, n_seqs, lo, hi + 1)]


def write_weight_file(path: str, shape: ModelShape, seed: int = 0, max_positions: int = 4096,
                      gain_jitter: float = 0.0) -> None:
    """Writes the seeded model in the library's weight-file format: the 8 bytes "EEWT0001", the config
    (19 little-endian 32-bit fields: n_layers, d_model, n_heads, head_dim, d_ff, vocab, n_exits,
    exit_layers[8], dtype, max_positions, rms_eps, rope_base), then every tensor in canonical order as
    raw elements (matrices in the storage dtype, gains fp32).  A model whose exits are not the default
    structure is written as "EEWT0002": the same with a 20th field, exit_flags, after rope_base.  Per exit the
    canonical order is: the attention half of its Transformer layer (if any), its MLP (if any, alone or as the
    layer's second half), its norm (if any), its output embedding (unless tied)."""
    import struct

    ex = list(shape.exit_layers) + [0] * (8 - len(shape.exit_layers))
    hdr = struct.pack("<7i8i2i2f", shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ff,
                      shape.vocab, len(shape.exit_layers), *ex, 1 if shape.dtype == "bf16" else 0, max_positions,
                      shape.rms_eps, shape.rope_base)
    with open(path, "wb") as f:
        if shape.exit_flags:
            f.write(b"EEWT0002")
            hdr += struct.pack("<i", shape.exit_flags)
        else:
            f.write(b"EEWT0001")
        f.write(hdr)
        for kind, idx in model_tensor_list(shape):
            t = model_tensor(shape, kind, idx, seed, "cpu", gain_jitter).contiguous()
            if t.dtype == torch.bfloat16:
                t = t.view(torch.int16)
            f.write(t.numpy().tobytes())
