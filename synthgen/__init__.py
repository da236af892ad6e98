"""Seeded synthetic inputs (token ids, random-init weights, model shapes).

Shared by the CPU oracle's tests, the GPU parity tests and the benchmark so that
both sides see bit-identical inputs.  Holds no arithmetic of the decoding method:
only shapes, seeds and the integer-hash generators of ``gen.c``.

Value recipe (see gen.c): token ids are ``hash mod vocab`` (uniform over the
vocabulary); weights are a centred 8-lane Irwin-Hall sum scaled to the requested
standard deviation (bell-shaped stand-in for N(0, std), tails clipped near 4.9
sigma), optionally rounded to bf16.  RMSNorm gains are the constant 1.0.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, replace
from typing import Iterator, NamedTuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libsynthgen.so")
_lib = None

WEIGHT_SEED = 20231108
PROMPT_SEED = 1
BUFFER_SEED = 2


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, src])
    return _SO


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, sz, i32, f32 = ctypes.c_uint64, ctypes.c_size_t, ctypes.c_int32, ctypes.c_float
        lib.synth_sigma_sum.restype = ctypes.c_double
        lib.synth_tokens.argtypes = [ctypes.c_void_p, sz, u64, u64, i32]
        lib.synth_normal_f32.argtypes = [ctypes.c_void_p, sz, u64, u64, f32, ctypes.c_int]
        lib.synth_normal_bf16.argtypes = [ctypes.c_void_p, sz, u64, u64, f32]
        for f in (lib.synth_tokens, lib.synth_normal_f32, lib.synth_normal_bf16):
            f.restype = None
        _lib = lib
    return _lib


def scale_for(std: float) -> np.float32:
    """fp32 multiplier that gives the centred lane sum the standard deviation ``std``."""
    return np.float32(std / _load().synth_sigma_sum())


def tokens(count: int, seed: int, stream: int, vocab: int) -> np.ndarray:
    out = np.empty(count, dtype=np.int32)
    _load().synth_tokens(out.ctypes.data, count, seed, stream, vocab)
    return out


def normal_f32(shape, seed: int, stream: int, std: float, round_bf16: bool) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().synth_normal_f32(out.ctypes.data, out.size, seed, stream, scale_for(std), int(round_bf16))
    return out


def normal_bf16(shape, seed: int, stream: int, std: float) -> np.ndarray:
    """bf16 bit patterns as uint16."""
    out = np.empty(shape, dtype=np.uint16)
    _load().synth_normal_bf16(out.ctypes.data, out.size, seed, stream, scale_for(std))
    return out


def normal_into(ptr: int, count: int, seed: int, stream: int, std: float, kind: str) -> None:
    """Fill caller memory at host address ``ptr``: kind 'f32', 'f32_bf16r' or 'bf16'."""
    lib = _load()
    if kind == "bf16":
        lib.synth_normal_bf16(ptr, count, seed, stream, scale_for(std))
    else:
        lib.synth_normal_f32(ptr, count, seed, stream, scale_for(std), int(kind == "f32_bf16r"))


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


# ----------------------------------------------------------------------------
# model shapes (the Llama-style decoders the benchmark configurations name)
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_base: float = 1e4
    dtype: str = "bf16"          # "f32" or "bf16": storage type of the weights
    init_std: float = 0.02

    @property
    def q_dim(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def n_params_streamed(self) -> int:
        """Weights read once per forward (embedding table excluded)."""
        per_layer = (self.d_model * (self.q_dim + 2 * self.kv_dim) + self.q_dim * self.d_model
                     + 3 * self.d_model * self.d_ffn)
        return self.n_layers * per_layer + self.d_model * self.vocab


SHAPES = {
    "tiny": ModelShape(2, 256, 4, 4, 64, 688, 1024, dtype="f32"),
    "7b": ModelShape(32, 4096, 32, 32, 128, 11008, 32000),
    "13b": ModelShape(40, 5120, 40, 40, 128, 13824, 32000),
    "70b": ModelShape(80, 8192, 64, 8, 128, 28672, 32000),
}


def small_variant(shape: ModelShape, **kw) -> ModelShape:
    return replace(shape, **kw)


class TensorSpec(NamedTuple):
    name: str        # 'emb','wlm' or per-layer 'wq','wk','wv','wo','wg','wu','wd'
    layer: int       # -1 for global tensors
    rows: int        # canonical layout is row-major [rows, cols] = [in, out]; emb is [vocab, d]
    cols: int
    stream: int


_KINDS = {"wq": 1, "wk": 2, "wv": 3, "wo": 4, "wg": 5, "wu": 6, "wd": 7}


def weight_tensors(s: ModelShape) -> Iterator[TensorSpec]:
    yield TensorSpec("emb", -1, s.vocab, s.d_model, 0xFFFF0001)
    for l in range(s.n_layers):
        dims = {"wq": (s.d_model, s.q_dim), "wk": (s.d_model, s.kv_dim), "wv": (s.d_model, s.kv_dim),
                "wo": (s.q_dim, s.d_model), "wg": (s.d_model, s.d_ffn), "wu": (s.d_model, s.d_ffn),
                "wd": (s.d_ffn, s.d_model)}
        for name, (r, c) in dims.items():
            yield TensorSpec(name, l, r, c, l * 16 + _KINDS[name])
    yield TensorSpec("wlm", -1, s.d_model, s.vocab, 0xFFFF0002)


def weight_array(s: ModelShape, spec: TensorSpec, seed: int = WEIGHT_SEED, as_bf16_bits: bool = False):
    """One weight tensor in canonical [in, out] layout (fp32, or bf16 bit patterns)."""
    if as_bf16_bits:
        assert s.dtype == "bf16"
        return normal_bf16((spec.rows, spec.cols), seed, spec.stream, s.init_std)
    return normal_f32((spec.rows, spec.cols), seed, spec.stream, s.init_std, s.dtype == "bf16")


def prompts(batch: int, length: int, vocab: int, seed: int = PROMPT_SEED) -> np.ndarray:
    return tokens(batch * length, seed, 0x50, vocab).reshape(batch, length)


def buffer_init(batch: int, buf_len: int, vocab: int, seed: int = BUFFER_SEED) -> np.ndarray:
    return tokens(batch * buf_len, seed, 0x51, vocab).reshape(batch, buf_len)
