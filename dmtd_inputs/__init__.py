"""Seeded synthetic inputs for the DMTD decode path: model shapes, weight blobs, prompts.

This module only *draws numbers*.  It contains none of the method's arithmetic (no
norm, attention, projection or scheduling code), so the CPU oracle and the HIP path
can both be fed from it without sharing any computation.

Generator: a counter-based SplitMix64.  Element ``i`` of stream ``(seed, stream_id)``
is ``mix(base + (i + 1) * GOLDEN)`` with ``base = mix(mix(seed) ^ stream_id * ODD)``,
so any slice of any tensor can be produced independently and in parallel and the
result does not depend on chunking or on a library's RNG.  Normal deviates use
Box-Muller on consecutive counter pairs (element 2j gets the cosine branch, 2j+1 the
sine branch), computed in float64 and rounded once to float32, then (for bf16 models)
once more to bfloat16 with round-to-nearest-even.

The paper's speed test uses prompts sampled uniformly from the vocabulary and a
fine-tuned Qwen3-4B (Sec. 3.4, Table 3); here random-init weights N(0, 0.02) of the
same shapes stand in for the fine-tuned model, and prompts are uniform over the
vocabulary.
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_ODD = np.uint64(0xD6E8FEB86659FD93)
_MASK64 = (1 << 64) - 1


def _mix_scalar(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def stream_base(seed: int, stream_id: int) -> int:
    return _mix_scalar(_mix_scalar(seed + 0x9E3779B97F4A7C15) ^ ((stream_id * 0xD6E8FEB86659FD93) & _MASK64))


def raw_u64(seed: int, stream_id: int, start: int, count: int) -> np.ndarray:
    """Counter values ``start .. start+count-1`` of a stream as uint64."""
    base = np.uint64(stream_base(seed, stream_id))
    idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix(base + idx * _GOLDEN)


def uniform_ints(seed: int, stream_id: int, count: int, modulus: int, start: int = 0) -> np.ndarray:
    """``count`` integers in ``[0, modulus)`` (int32).  Plain modulo of the 64-bit draw."""
    return (raw_u64(seed, stream_id, start, count) % np.uint64(modulus)).astype(np.int32)


def _normal_chunk(seed: int, stream_id: int, start: int, count: int) -> np.ndarray:
    """Standard normal float64 values for elements ``start..start+count-1`` (start even)."""
    assert start % 2 == 0
    npair = (count + 1) // 2
    z = raw_u64(seed, stream_id, start, 2 * npair)
    two53 = float(1 << 53)
    u1 = ((z[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) / two53  # (0, 1]
    u2 = (z[1::2] >> np.uint64(11)).astype(np.float64) / two53  # [0, 1)
    r = np.sqrt(-2.0 * np.log(u1))
    ang = (2.0 * np.pi) * u2
    out = np.empty(2 * npair, dtype=np.float64)
    out[0::2] = r * np.cos(ang)
    out[1::2] = r * np.sin(ang)
    return out[:count]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Shape of a Qwen3-style decoder-only model (shapes only; no arithmetic)."""

    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    intermediate: int
    vocab: int
    dtype: str = "bf16"  # storage type of the weight blob: "fp32" or "bf16"
    rms_eps: float = 1e-6
    rope_theta: float = 1e6
    tied_embeddings: bool = True

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    batch: int
    prompt_len: int
    gen_len: int
    tau: int
    n_late: int


_TINY = ModelShape(4, 256, 4, 2, 64, 768, 1024, dtype="fp32")
_Q06B = ModelShape(28, 1024, 16, 8, 128, 3072, 151936)
_Q4B = ModelShape(36, 2560, 32, 8, 128, 9728, 151936)

WORKLOADS = {
    "C1": Workload("C1 tiny fp32, B=1, P=32, G=16, tau=2, n_late=1", _TINY, 1, 32, 16, 2, 1),
    "C2": Workload("C2 Qwen3-0.6B-shaped bf16, B=1, P=256, G=128, tau=2, n_late=4", _Q06B, 1, 256, 128, 2, 4),
    "C3": Workload("C3 Qwen3-4B-shaped bf16, B=1, P=1024, G=512, tau=3, n_late=8", _Q4B, 1, 1024, 512, 3, 8),
    "C4": Workload("C4 Qwen3-4B-shaped bf16, B=32, P=2048, G=256, tau=4, n_late=12", _Q4B, 32, 2048, 256, 4, 12),
    "C5": Workload("C5 Qwen3-4B-shaped bf16, B=8, P=16384, G=256, tau=3, n_late=8", _Q4B, 8, 16384, 256, 3, 8),
}


def tensor_specs(shape: ModelShape):
    """Ordered ``(name, dims, kind)`` of the weight blob; kind is "matrix" or "gain".

    Order: token table; per layer attn_norm, q, k, v, q_norm, k_norm, o, mlp_norm, gate, up,
    down; final_norm; lm_head only if the table is not tied.  Matrices are row-major
    ``[out, in]``.
    """
    s = shape
    specs = [("embed", (s.vocab, s.hidden), "matrix")]
    for l in range(s.n_layers):
        p = f"layers.{l}."
        specs += [
            (p + "attn_norm", (s.hidden,), "gain"),
            (p + "q", (s.n_q_heads * s.head_dim, s.hidden), "matrix"),
            (p + "k", (s.n_kv_heads * s.head_dim, s.hidden), "matrix"),
            (p + "v", (s.n_kv_heads * s.head_dim, s.hidden), "matrix"),
            (p + "q_norm", (s.head_dim,), "gain"),
            (p + "k_norm", (s.head_dim,), "gain"),
            (p + "o", (s.hidden, s.n_q_heads * s.head_dim), "matrix"),
            (p + "mlp_norm", (s.hidden,), "gain"),
            (p + "gate", (s.intermediate, s.hidden), "matrix"),
            (p + "up", (s.intermediate, s.hidden), "matrix"),
            (p + "down", (s.hidden, s.intermediate), "matrix"),
        ]
    specs.append(("final_norm", (s.hidden,), "gain"))
    if not s.tied_embeddings:
        specs.append(("lm_head", (s.vocab, s.hidden), "matrix"))
    return specs


def blob_elems(shape: ModelShape) -> int:
    return sum(int(np.prod(d)) for _, d, _ in tensor_specs(shape))


_CHUNK = 1 << 21


def make_weight_blob(shape: ModelShape, seed: int = 0, std: float = 0.02, gain_sigma: float = 0.0,
                     threads: int | None = None) -> np.ndarray:
    """The model's weights as one flat array (float32, or uint16 holding bfloat16 bits).

    Matrices are ``std * N(0,1)``; gains are ``1 + gain_sigma * N(0,1)`` (``gain_sigma=0``
    gives the unit gains the benchmark configurations name; tests use a non-zero value so
    that a mis-indexed gain cannot hide).  Tensor number ``t`` in :func:`tensor_specs`
    order draws from stream ``t``.
    """
    specs = tensor_specs(shape)
    total = sum(int(np.prod(d)) for _, d, _ in specs)
    bf16 = shape.dtype == "bf16"
    out = np.empty(total, dtype=np.uint16 if bf16 else np.float32)
    jobs = []
    off = 0
    for t, (_, dims, kind) in enumerate(specs):
        n = int(np.prod(dims))
        for c0 in range(0, n, _CHUNK):
            jobs.append((t, kind, off, c0, min(_CHUNK, n - c0)))
        off += n

    def run(job):
        t, kind, toff, c0, cnt = job
        g = _normal_chunk(seed, t, c0, cnt)
        if kind == "gain":
            v = (1.0 + gain_sigma * g).astype(np.float32) if gain_sigma else np.ones(cnt, np.float32)
        else:
            v = (std * g).astype(np.float32)
        out[toff + c0: toff + c0 + cnt] = f32_to_bf16_bits(v) if bf16 else v

    if threads is None:
        threads = min(16, os.cpu_count() or 1)
    if threads <= 1 or len(jobs) < 4:
        for j in jobs:
            run(j)
    else:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(run, jobs))
    return out


def make_prompts(vocab: int, batch: int, prompt_len: int, seed: int = 1) -> np.ndarray:
    """``[batch, prompt_len]`` int32 prompts, uniform over the vocabulary; sequence ``b`` uses seed ``seed + b``."""
    return np.stack([uniform_ints(seed + b, 0x70726F6D, prompt_len, vocab) for b in range(batch)])


def make_continuation(vocab: int, batch: int, length: int, seed: int = 1001) -> np.ndarray:
    """``[batch, length]`` int32 random tokens used as a teacher-forced continuation in parity runs."""
    return np.stack([uniform_ints(seed + b, 0x636F6E74, length, vocab) for b in range(batch)])
