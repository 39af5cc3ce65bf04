"""Seeded synthetic inputs for a Llama-style decode step (weights, KV prefill, token ids).

This module is the ONLY code shared by the HIP path's tests/bench and the CPU oracle's tests.
It holds none of the decoder's arithmetic: it turns (seed, tensor name, element index) into a
value with a counter-based integer hash, so any slab of any tensor can be regenerated anywhere
(CPU or GPU tensor) with identical bits.  Only integer ops, one int->fp32 conversion, one fp32
multiply and one fp32->bf16 round-to-nearest-even are used, all of which are exactly specified
on both devices.

Shapes follow the Llama-3.1 rows of the paper's model-configuration table (Section 2.1) and the
configs of this repository's benchmark description.  The values stand in for the real
checkpoints, GPTQ-quantised checkpoints and prompts the paper measured with.

Value recipes
  * bf16 weights / embedding / LM head: approx N(0, 0.02)  (sum of four 16-bit uniforms)
  * RMSNorm gains: 1 + N(0, 0.02), rounded to bf16
  * KV-cache prefill: approx N(0, 1), rounded to bf16 (taken as already rotated keys)
  * int8 per-output-channel: codes uniform in [-127, 127]; fp16 scale s = 0.02/73.6*(1+u/4)
  * int4 group-128: codes uniform in [0, 15]; fp16 zero = integer uniform in [0, 15];
    fp16 scale s = 0.02/6.5*(1+u/4); canonical packing: low nibble = even k
  * token ids: uniform in [0, vocab)
"""
from __future__ import annotations

import dataclasses
import zlib

import torch

_M32 = 0xFFFFFFFF
# std of the sum of four independent uniform integers on [0, 65535]
_IH4_STD = 37837.22


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Decoder dimensions (paper Section 2.1, model-configuration table)."""

    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def params_per_layer(self) -> int:
        d, f = self.d_model, self.d_ffn
        return (self.q_dim + 2 * self.kv_dim) * d + d * self.q_dim + 3 * f * d

    def replace(self, **kw) -> "ModelShape":
        return dataclasses.replace(self, **kw)


TINY = ModelShape("tiny", 4, 512, 8, 2, 64, 1376, 4096, 1e-5, 10000.0)
LLAMA_8B = ModelShape("llama3-8b", 32, 4096, 32, 8, 128, 14336, 128256, 1e-5, 500000.0)
LLAMA_70B = ModelShape("llama3-70b", 80, 8192, 64, 8, 128, 28672, 128256, 1e-5, 500000.0)
SHAPES = {s.name: s for s in (TINY, LLAMA_8B, LLAMA_70B)}

WDTYPE_BF16, WDTYPE_INT8, WDTYPE_INT4 = 0, 1, 2
INT4_GROUP = 128


def _tensor_key(seed: int, name: str) -> int:
    return (seed * 0x9E3779B1 + zlib.crc32(name.encode())) & _M32


def _mix(x: torch.Tensor) -> torch.Tensor:
    """32-bit avalanche finaliser on int64 tensors holding values in [0, 2^32)."""
    x = x ^ (x >> 16)
    x = (x * 0x7FEB352D) & _M32
    x = x ^ (x >> 15)
    x = (x * 0x846CA68B) & _M32
    x = x ^ (x >> 16)
    return x


def hash_u32(seed: int, name: str, start: int, count: int, device, stream: int = 0) -> torch.Tensor:
    """uint32 hash (as int64 tensor) of element indices [start, start+count) of tensor `name`."""
    key = _tensor_key(seed, name) ^ ((stream * 0x85EBCA6B) & _M32)
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    lo = idx & _M32
    hi = idx >> 32
    return _mix((_mix(lo ^ key) + hi * 0x27D4EB2F + 0x165667B1) & _M32)


_CHUNK = 1 << 24


def _chunks(n: int):
    for s in range(0, n, _CHUNK):
        yield s, min(_CHUNK, n - s)


def normal_bf16(seed: int, name: str, shape, std: float, device, mean: float = 0.0) -> torch.Tensor:
    """approx N(mean, std) rounded to bf16; element i depends only on (seed, name, i)."""
    n = 1
    for s in shape:
        n *= s
    out = torch.empty(n, dtype=torch.bfloat16, device=device)
    scale = float(std) / _IH4_STD
    for s0, cnt in _chunks(n):
        h1 = hash_u32(seed, name, s0, cnt, device, 0)
        h2 = hash_u32(seed, name, s0, cnt, device, 1)
        s = (h1 & 0xFFFF) + (h1 >> 16) + (h2 & 0xFFFF) + (h2 >> 16) - 131070
        v = s.to(torch.float32) * scale
        if mean != 0.0:
            v = v + mean
        out[s0:s0 + cnt] = v.to(torch.bfloat16)
    return out.view(*shape)


def uniform_int(seed: int, name: str, shape, lo: int, hi: int, device, dtype=torch.int32) -> torch.Tensor:
    """integers uniform on [lo, hi] inclusive."""
    n = 1
    for s in shape:
        n *= s
    out = torch.empty(n, dtype=dtype, device=device)
    span = hi - lo + 1
    for s0, cnt in _chunks(n):
        h = hash_u32(seed, name, s0, cnt, device, 2)
        out[s0:s0 + cnt] = (((h * span) >> 32) + lo).to(dtype)
    return out.view(*shape)


def unit_fp32(seed: int, name: str, shape, device) -> torch.Tensor:
    """u in [0, 1) with 16 bits of resolution, fp32 (exact)."""
    n = 1
    for s in shape:
        n *= s
    h = hash_u32(seed, name, 0, n, device, 3)
    return ((h >> 16).to(torch.float32) * (1.0 / 65536.0)).view(*shape)


# --------------------------------------------------------------------------------------------
# model tensors
# --------------------------------------------------------------------------------------------
LAYER_MATS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def mat_shape(shape: ModelShape, which: str):
    d, f = shape.d_model, shape.d_ffn
    return {
        "wq": (shape.q_dim, d), "wk": (shape.kv_dim, d), "wv": (shape.kv_dim, d),
        "wo": (d, shape.q_dim), "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
        "lm_head": (shape.vocab, d), "embed": (shape.vocab, d),
    }[which]


def make_matrix(shape: ModelShape, seed: int, name: str, which: str, wdtype: int, device) -> dict:
    """One projection matrix in canonical layout: row-major [out, in].

    Returns a dict with key 'w' (bf16 [N,K] | int8 [N,K] | uint8 [N,K/2]) and, for the
    quantised types, 's' (fp16 [N] | [N,K/128]) and 'z' (fp16 [N,K/128], int4 only).
    """
    n, k = mat_shape(shape, which)
    if wdtype == WDTYPE_BF16:
        return {"w": normal_bf16(seed, name, (n, k), 0.02, device)}
    if wdtype == WDTYPE_INT8:
        q = uniform_int(seed, name, (n, k), -127, 127, device, torch.int8)
        u = unit_fp32(seed, name + ".s", (n,), device)
        s = ((0.02 / 73.6) * (1.0 + 0.25 * u)).to(torch.float16)
        return {"w": q, "s": s}
    if wdtype == WDTYPE_INT4:
        assert k % INT4_GROUP == 0
        codes = uniform_int(seed, name, (n, k), 0, 15, device, torch.uint8)
        packed = (codes[:, 0::2] | (codes[:, 1::2] << 4)).contiguous()
        g = k // INT4_GROUP
        u = unit_fp32(seed, name + ".s", (n, g), device)
        s = ((0.02 / 6.5) * (1.0 + 0.25 * u)).to(torch.float16)
        z = uniform_int(seed, name + ".z", (n, g), 0, 15, device, torch.int32).to(torch.float16)
        return {"w": packed, "s": s, "z": z}
    raise ValueError(f"unknown wdtype {wdtype}")


def make_layer(shape: ModelShape, seed: int, layer: int, wdtype: int, device) -> dict:
    """All tensors of decoder layer `layer` (canonical layouts)."""
    out = {
        "attn_norm": normal_bf16(seed, f"l{layer}.attn_norm", (shape.d_model,), 0.02, device, mean=1.0),
        "ffn_norm": normal_bf16(seed, f"l{layer}.ffn_norm", (shape.d_model,), 0.02, device, mean=1.0),
    }
    for which in LAYER_MATS:
        out[which] = make_matrix(shape, seed, f"l{layer}.{which}", which, wdtype, device)
    return out


def make_head(shape: ModelShape, seed: int, wdtype: int, device, quant_lm_head: bool = True) -> dict:
    """Embedding table (always bf16), final norm gain, LM head."""
    return {
        "embed": normal_bf16(seed, "embed", (shape.vocab, shape.d_model), 0.02, device),
        "final_norm": normal_bf16(seed, "final_norm", (shape.d_model,), 0.02, device, mean=1.0),
        "lm_head": make_matrix(shape, seed, "lm_head", "lm_head",
                               wdtype if quant_lm_head else WDTYPE_BF16, device),
    }


def make_kv_prefill(shape: ModelShape, seed: int, layer: int, seq: int, n_ctx: int, device):
    """Prefilled cache rows for one (layer, sequence): K, V bf16 [n_ctx, n_kv_heads, head_dim]."""
    k = normal_bf16(seed, f"kv.l{layer}.s{seq}.k", (n_ctx, shape.n_kv_heads, shape.head_dim), 1.0, device)
    v = normal_bf16(seed, f"kv.l{layer}.s{seq}.v", (n_ctx, shape.n_kv_heads, shape.head_dim), 1.0, device)
    return k, v


def make_tokens(shape: ModelShape, seed: int, n_steps: int, batch: int, device="cpu") -> torch.Tensor:
    """Teacher-forced token ids, int32 [n_steps, batch]."""
    return uniform_int(seed, "tokens", (n_steps, batch), 0, shape.vocab - 1, device, torch.int32)


def weight_bytes_per_step(shape: ModelShape, wdtype: int, quant_lm_head: bool = True) -> int:
    """Bytes of parameters one decode step must read (every weight once, norm gains, scales)."""
    def mat_bytes(n, k, wd):
        if wd == WDTYPE_BF16:
            return n * k * 2
        if wd == WDTYPE_INT8:
            return n * k + n * 2
        return n * k // 2 + 2 * (n * (k // INT4_GROUP)) * 2

    total = 0
    for which in LAYER_MATS:
        n, k = mat_shape(shape, which)
        total += mat_bytes(n, k, wdtype)
    total += 2 * shape.d_model * 2
    total *= shape.n_layers
    total += shape.d_model * 2
    n, k = mat_shape(shape, "lm_head")
    total += mat_bytes(n, k, wdtype if quant_lm_head else WDTYPE_BF16)
    return total


def kv_bytes_per_step(shape: ModelShape, batch: int, n_ctx: int) -> int:
    """Bytes of valid cache rows one decode step reads with n_ctx rows already cached."""
    return 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * 2 * n_ctx * batch
