"""Counter-based random-init weights, bit-identical on CPU and GPU.

value(seed, tensor_id, i) = std * z, where z is the centred, unit-variance sum
of four 16-bit uniforms taken from two 32-bit hashes of the element counter i
(an Irwin-Hall approximation of a normal, |z| <= 3.47).  All hashing is exact
integer arithmetic on int64 tensors (every intermediate < 2**50), the integer
sum converts to fp32 exactly, and one fp32 multiply plus one round-to-nearest
-even conversion to bf16 are IEEE-defined, so any device gives the same bytes.
"""
import math

import torch

_M32 = 0xFFFFFFFF

# tensor ids inside one layer; global id = layer * 16 + local id
TENSOR_IDS = {
    "wq": 0, "wk": 1, "wv": 2, "wo": 3, "wg": 4, "wu": 5, "wd": 6, "g1": 7, "g2": 8, "gq": 9, "gk": 10,
}
_EMBED_ID = 1_000_000
_LMHEAD_ID = 1_000_001
_FINAL_NORM_ID = 1_000_002

# standard deviation of the sum of four independent uniforms on {0..65535}
_SUM4_STD = math.sqrt(4.0 * (65536.0 ** 2 - 1.0) / 12.0)
_SUM4_MEAN = 2 * 65535


def _mul32(x: torch.Tensor, m: int) -> torch.Tensor:
    """(x * m) mod 2**32 for 0 <= x < 2**32 without overflowing int64."""
    lo = x * (m & 0xFFFF)
    hi = ((x * (m >> 16)) & 0xFFFF) << 16
    return (lo + hi) & _M32


def hash32(x: torch.Tensor) -> torch.Tensor:
    """A 32-bit avalanche mix (xorshift-multiply) of an int64 tensor of values < 2**32."""
    x = x ^ (x >> 16)
    x = _mul32(x, 0x7FEB352D)
    x = x ^ (x >> 15)
    x = _mul32(x, 0x846CA68B)
    x = x ^ (x >> 16)
    return x


def _key(seed: int, tensor_id: int) -> int:
    k = (seed * 0x9E3779B1 + tensor_id * 0x85EBCA77 + 0x165667B1) & _M32
    # scalar version of hash32
    k ^= k >> 16
    k = (k * 0x7FEB352D) & _M32
    k ^= k >> 15
    k = (k * 0x846CA68B) & _M32
    k ^= k >> 16
    return k


def gen_normal(seed: int, tensor_id: int, shape, std: float, dtype: torch.dtype,
               device="cpu", chunk: int = 1 << 24) -> torch.Tensor:
    """Tensor of `shape` with element i (row-major) = std * z(seed, tensor_id, i)."""
    numel = 1
    for s in shape:
        numel *= int(s)
    assert numel < (1 << 32)
    out = torch.empty(numel, dtype=dtype, device=device)
    key = _key(seed, tensor_id)
    scale = torch.tensor(std / _SUM4_STD, dtype=torch.float32, device=device)
    for start in range(0, numel, chunk):
        n = min(chunk, numel - start)
        i = torch.arange(start, start + n, dtype=torch.int64, device=device)
        h1 = hash32(i ^ key)
        h2 = hash32((h1 + 0x9E3779B9) & _M32)
        s = (h1 & 0xFFFF) + (h1 >> 16) + (h2 & 0xFFFF) + (h2 >> 16) - _SUM4_MEAN
        out[start:start + n] = (s.to(torch.float32) * scale).to(dtype)
    return out.view(*shape)


def _torch_dtype(shape_dtype: str) -> torch.dtype:
    return {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[shape_dtype]


def norm_gain(shape, seed: int, tensor_id: int, jitter: float, device="cpu", width: int = 0) -> torch.Tensor:
    """RMSNorm gain: all ones (benchmark configs) or 1 + jitter*z (tests that must
    notice a dropped or misplaced gain).  `width` defaults to the hidden size."""
    dt = _torch_dtype(shape.dtype)
    width = width or shape.hidden
    if jitter == 0.0:
        return torch.ones(width, dtype=dt, device=device)
    z = gen_normal(seed, tensor_id, (width,), jitter, torch.float32, device)
    return (1.0 + z).to(dt)


def layer_weights(shape, seed: int, layer: int, device="cpu", std: float = 0.02,
                  gain_jitter: float = 0.0) -> dict:
    """All tensors of one decoder layer, stored [out, in] like the projection y = x W^T."""
    dt = _torch_dtype(shape.dtype)
    h, q, kv, f = shape.hidden, shape.qkv_dim, shape.kv_dim, shape.ffn
    base = layer * 16
    dims = {"wq": (q, h), "wk": (kv, h), "wv": (kv, h), "wo": (h, q),
            "wg": (f, h), "wu": (f, h), "wd": (h, f)}
    out = {}
    for name, d in dims.items():
        out[name] = gen_normal(seed, base + TENSOR_IDS[name], d, std, dt, device)
    out["g1"] = norm_gain(shape, seed, base + TENSOR_IDS["g1"], gain_jitter, device)
    out["g2"] = norm_gain(shape, seed, base + TENSOR_IDS["g2"], gain_jitter, device)
    if shape.qk_norm:
        out["gq"] = norm_gain(shape, seed, base + TENSOR_IDS["gq"], gain_jitter, device, width=shape.head_dim)
        out["gk"] = norm_gain(shape, seed, base + TENSOR_IDS["gk"], gain_jitter, device, width=shape.head_dim)
    return out


def embedding(shape, seed: int, device="cpu", std: float = 0.02) -> torch.Tensor:
    return gen_normal(seed, _EMBED_ID, (shape.vocab, shape.hidden), std, _torch_dtype(shape.dtype), device)


def lm_head(shape, seed: int, device="cpu", std: float = 0.02) -> torch.Tensor:
    return gen_normal(seed, _LMHEAD_ID, (shape.vocab, shape.hidden), std, _torch_dtype(shape.dtype), device)


def final_norm(shape, seed: int, device="cpu", gain_jitter: float = 0.0) -> torch.Tensor:
    return norm_gain(shape, seed, _FINAL_NORM_ID, gain_jitter, device)
