"""Model shapes of the benchmark configurations (random-init Llama-style decoders).

The paper evaluates Vicuna-7B/13B/33B (Sec. 5.1 "Setup"); the shapes below are
those architectures' public dimensions.  Trained weights are not used: every
tensor is random-init from a seed (see weights.py).
"""
from dataclasses import dataclass


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    hidden: int
    n_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    dtype: str = "bf16"  # storage type of weights and KV cache: "bf16", "f16" or "f32"
    n_kv_heads: int = 0  # key/value heads (grouped-query attention); 0 = as many as query heads
    qk_norm: bool = False  # RMSNorm over head_dim on q and k before the rotary embedding

    @property
    def qkv_dim(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads or self.n_heads

    @property
    def kv_dim(self) -> int:
        return self.kv_heads * self.head_dim

    def layer_param_count(self) -> int:
        h, q, kv, f = self.hidden, self.qkv_dim, self.kv_dim, self.ffn
        return q * h + 2 * kv * h + h * q + 3 * f * h

    def weight_bytes_per_layer(self) -> int:
        return self.layer_param_count() * (4 if self.dtype == "f32" else 2)


SHAPES = {
    # 2-layer oracle-scale model, fp32
    "tiny": ModelShape("tiny", 2, 256, 4, 64, 688, 1024, dtype="f32"),
    # same tiny dimensions stored in bf16 (exercises the MFMA path at oracle scale)
    "tiny_bf16": ModelShape("tiny_bf16", 2, 256, 4, 64, 688, 1024, dtype="bf16"),
    # a mid-size bf16 model with head_dim 128 that the oracle still finishes in seconds
    "small_bf16": ModelShape("small_bf16", 3, 1024, 8, 128, 2752, 4096, dtype="bf16"),
    "7b": ModelShape("7b", 32, 4096, 32, 128, 11008, 32000),
    "13b": ModelShape("13b", 40, 5120, 40, 128, 13824, 32000),
    "33b": ModelShape("33b", 60, 6656, 52, 128, 17920, 32000),
    # the grouped-query models the paper also evaluates (Sec. 5.1): public dimensions of Llama-3-8B and Qwen3-8B
    "llama3_8b": ModelShape("llama3_8b", 32, 4096, 32, 128, 14336, 128256, rope_base=500000.0, n_kv_heads=8),
    "qwen3_8b": ModelShape("qwen3_8b", 36, 4096, 32, 128, 12288, 151936, rope_base=1000000.0, rms_eps=1e-6,
                           n_kv_heads=8, qk_norm=True),
    # fp16 storage, the precision the paper runs in (App. C): oracle-scale models and the 7B shape
    "tiny_f16": ModelShape("tiny_f16", 2, 256, 4, 64, 688, 1024, dtype="f16"),
    "small_gqa_qknorm_f16": ModelShape("small_gqa_qknorm_f16", 3, 1024, 8, 128, 2752, 4096, dtype="f16",
                                       n_kv_heads=2, qk_norm=True, rms_eps=1e-6),
    "7b_f16": ModelShape("7b_f16", 32, 4096, 32, 128, 11008, 32000, dtype="f16"),
    # oracle-scale models with the same structure
    "tiny_gqa_bf16": ModelShape("tiny_gqa_bf16", 2, 256, 4, 64, 688, 1024, dtype="bf16", n_kv_heads=2),
    "small_gqa_qknorm_bf16": ModelShape("small_gqa_qknorm_bf16", 3, 1024, 8, 128, 2752, 4096, dtype="bf16",
                                        n_kv_heads=2, qk_norm=True, rms_eps=1e-6),
}


def shape_by_name(name: str) -> ModelShape:
    return SHAPES[name]
