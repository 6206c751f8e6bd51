"""Seeded synthetic inputs for the DEER draft-verify path: model shapes, weights, prompts, KV fill.

This module is the only code shared by the CPU oracle's tests and the HIP path's tests/bench.
It holds none of the method's arithmetic: it only names shapes and draws seeded random
numbers.  The paper (Sec. 4, "Models") evaluates on released Qwen checkpoints and a trained
0.5B dLLM drafter; none of those exist here, so every tensor is i.i.d. N(0, 0.02^2) from a
per-tensor seed, prompts are uniform token ids, and only the shapes stand in for the paper's
workloads.

Every tensor is defined chunk by chunk so that it can be produced in parallel or streamed:
  chunk c of tensor (model_seed, name, layer, expert) =
      PCG64(SeedSequence([model_seed, tensor_code(name), layer+1, expert+1, c]))
          .standard_normal(CHUNK, float32) * 0.02
flattened in row-major order of the canonical shape ([in][out] for every projection, so that
y = x @ W; [vocab][d] for the embedding table).
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np

CHUNK = 1 << 22  # elements per independently seeded chunk
WEIGHT_STD = 0.02

TENSOR_CODES = {
    "embed": 1, "lm_head": 2, "wq": 3, "wk": 4, "wv": 5, "wo": 6,
    "wg": 7, "wu": 8, "wd": 9, "router": 10, "kv_k": 11, "kv_v": 12,
}


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Decoder shape.  n_experts == 0 means a dense SwiGLU FFN of width d_ff."""
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    n_experts: int = 0
    top_k: int = 0
    d_ff_expert: int = 0
    rope_base: float = 10000.0
    rms_eps: float = 1e-6

    def tensor_shape(self, name: str):
        d, hq, hkv, hd = self.d_model, self.n_q_heads, self.n_kv_heads, self.head_dim
        f = self.d_ff_expert if self.n_experts else self.d_ff
        return {
            "embed": (self.vocab, d), "lm_head": (d, self.vocab),
            "wq": (d, hq * hd), "wk": (d, hkv * hd), "wv": (d, hkv * hd), "wo": (hq * hd, d),
            "wg": (d, f), "wu": (d, f), "wd": (f, d), "router": (d, self.n_experts),
        }[name]

    def layer_tensor_names(self):
        names = ["wq", "wk", "wv", "wo"]
        if self.n_experts:
            names.append("router")
        return names

    def n_params(self) -> int:
        d = self.d_model
        attn = d * (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim + self.n_q_heads * self.head_dim * d
        if self.n_experts:
            ffn = self.n_experts * 3 * d * self.d_ff_expert + d * self.n_experts
        else:
            ffn = 3 * d * self.d_ff
        return self.n_layers * (attn + ffn) + 2 * self.vocab * d


DRAFTER_05B = ModelShape(24, 896, 14, 2, 64, 4864, 151936, rope_base=1e6)

# The five workloads: (target, drafter, batch, prefix length j, block size k, temperature T).
CONFIGS = {
    "tiny": dict(
        target=ModelShape(2, 128, 4, 2, 32, 512, 1024, rope_base=10000.0),
        drafter=ModelShape(1, 128, 4, 2, 32, 512, 1024, rope_base=10000.0),
        batch=1, prefix=64, k=8, T=(0.0, 1.0), weight_dtype="f32"),
    "qwen3_4b": dict(
        target=ModelShape(36, 2560, 32, 8, 128, 9728, 151936, rope_base=1e6),
        drafter=DRAFTER_05B, batch=1, prefix=1024, k=16, T=(0.0,), weight_dtype="bf16"),
    "qwen3_8b": dict(
        target=ModelShape(36, 4096, 32, 8, 128, 12288, 151936, rope_base=1e6),
        drafter=DRAFTER_05B, batch=1, prefix=4096, k=32, T=(0.0,), weight_dtype="bf16"),
    "qwen3_30b_a3b": dict(
        target=ModelShape(48, 2048, 32, 4, 128, 0, 151936, n_experts=128, top_k=8,
                          d_ff_expert=768, rope_base=1e6),
        drafter=DRAFTER_05B, batch=1, prefix=2048, k=32, T=(0.0,), weight_dtype="bf16"),
    "qwen3_8b_long_batch": dict(
        target=ModelShape(36, 4096, 32, 8, 128, 12288, 151936, rope_base=1e6),
        drafter=DRAFTER_05B, batch=16, prefix=32768, k=32, T=(1.0,), weight_dtype="bf16"),
}

TARGET_SEED, DRAFTER_SEED, PROMPT_SEED, SAMPLING_SEED, KV_SEED = 1, 2, 3, 4, 5


def scaled(shape: ModelShape, **kw) -> ModelShape:
    """Same architecture with some fields replaced (e.g. fewer layers for a bounded test)."""
    return dataclasses.replace(shape, **kw)


# ---------------------------------------------------------------------------------------------
# bf16 <-> fp32 bit plumbing (storage format only)
# ---------------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------------------------------------
# seeded draws
# ---------------------------------------------------------------------------------------------
def _normal_chunk(key, n):
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence(key)))
    return g.standard_normal(n, dtype=np.float32)


def seeded_normal(key_prefix, n_elems: int, threads: int = 8) -> np.ndarray:
    """Flat fp32 N(0,1) vector of n_elems, defined chunk-wise by key_prefix + [chunk]."""
    out = np.empty(n_elems, dtype=np.float32)
    n_chunks = (n_elems + CHUNK - 1) // CHUNK

    def fill(c):
        lo = c * CHUNK
        hi = min(n_elems, lo + CHUNK)
        out[lo:hi] = _normal_chunk(list(key_prefix) + [c], hi - lo)

    if n_chunks == 1 or threads <= 1:
        for c in range(n_chunks):
            fill(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out


def weight_f32(shape: ModelShape, model_seed: int, name: str, layer: int = -1, expert: int = -1,
               threads: int = 8) -> np.ndarray:
    """Canonical fp32 tensor, N(0, 0.02^2)."""
    dims = shape.tensor_shape(name)
    n = int(np.prod(dims))
    v = seeded_normal([model_seed, TENSOR_CODES[name], layer + 1, expert + 1], n, threads)
    v *= np.float32(WEIGHT_STD)
    return v.reshape(dims)


def weight_bf16_bits(shape, model_seed, name, layer=-1, expert=-1, threads=8) -> np.ndarray:
    """The same tensor rounded once to bf16; these uint16 bit patterns are the model."""
    return f32_to_bf16_bits(weight_f32(shape, model_seed, name, layer, expert, threads))


def weight_as_f32(shape, model_seed, name, layer=-1, expert=-1, weight_dtype="bf16", threads=8):
    """What a consumer computing in fp32/fp64 should use: exact fp32 values of the stored model."""
    w = weight_f32(shape, model_seed, name, layer, expert, threads)
    if weight_dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(w))
    return w


def prompt_ids(vocab: int, length: int, seq: int = 0, seed: int = PROMPT_SEED) -> np.ndarray:
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, seq, length])))
    return g.integers(0, vocab, size=length, dtype=np.int64).astype(np.int32)


def kv_fill_bits(shape: ModelShape, which: str, layer: int, seq: int, n_slots: int,
                 seed: int = KV_SEED, std: float = 1.0, threads: int = 8) -> np.ndarray:
    """Seeded stand-in cache contents [n_slots][n_kv_heads][head_dim] as bf16 bits.

    Used where running a real prefill is too costly (32k-token prefixes): both sides load the
    same bytes.  The values have the scale of a random-init model's K/V rows."""
    n = n_slots * shape.n_kv_heads * shape.head_dim
    v = seeded_normal([seed, TENSOR_CODES["kv_" + which], layer + 1, seq + 1], n, threads)
    v *= np.float32(std)
    return f32_to_bf16_bits(v).reshape(n_slots, shape.n_kv_heads, shape.head_dim)


def mask_token_id(vocab: int) -> int:
    """The drafter's [MASK] id: the last vocabulary entry."""
    return vocab - 1
