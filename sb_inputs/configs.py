"""Shapes and workloads of the five benchmark configurations.

The paper evaluates on Vicuna / CodeLlama-Instruct 7B and 13B (Sec. 4.1,
"Backbone Models") with Spec-Bench prompts; neither the weights nor the prompts
are available here, so each configuration keeps the *shape* of such a model and
draws seeded random weights and uniform-random prompts instead.
"""
from dataclasses import dataclass, field, replace
from typing import Dict

FP32 = 0
BF16 = 1


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    weight_dtype: int          # FP32 or BF16
    kv_dtype: int              # FP32 or BF16 (K/V rounded on cache store)
    n_exit_heads: int          # exit heads exist after layers 1..n_exit_heads
    rms_eps: float = 1e-6
    rope_base: float = 10000.0

    @property
    def qkv_rows(self) -> int:
        return (self.n_heads + 2 * self.n_kv_heads) * self.head_dim

    def layer_weight_bytes(self) -> int:
        es = 2 if self.weight_dtype == BF16 else 4
        d, f = self.d_model, self.d_ffn
        return es * (self.qkv_rows * d + d * self.n_heads * self.head_dim
                     + 2 * f * d + d * f)

    def head_weight_bytes(self) -> int:
        es = 2 if self.weight_dtype == BF16 else 4
        return es * self.vocab * self.d_model

    def kv_bytes_per_token_layer(self) -> int:
        es = 2 if self.kv_dtype == BF16 else 4
        return 2 * self.n_kv_heads * self.head_dim * es


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    prompt_len: int
    gen_len: int
    d_max: int
    w_max: int
    T_first: float             # temperature at layer 1
    T_last: float              # temperature at layer d_max
    threshold: float
    exit_lo: int               # forced exit layer ~ U{exit_lo..d_max}
    weight_seed: int
    prompt_seed: int
    sched_seed: int
    max_seq: int = 0           # 0: prompt_len + gen_len + w_max rounded up to 16

    def seq_capacity(self) -> int:
        if self.max_seq:
            return self.max_seq
        n = self.prompt_len + self.gen_len + self.w_max + 1
        return (n + 15) // 16 * 16

    def temperatures(self):
        """Linear schedule T_first -> T_last over layers 1..d_max (an input array)."""
        if self.d_max == 1:
            return [float(self.T_first)]
        step = (self.T_last - self.T_first) / (self.d_max - 1)
        return [float(self.T_first + step * i) for i in range(self.d_max)]


def tiny_shape(n_layers: int = 4, n_exit_heads: int = 2, **kw) -> ModelShape:
    base = ModelShape(n_layers=n_layers, d_model=256, n_heads=4, n_kv_heads=4,
                      head_dim=64, d_ffn=688, vocab=1024, weight_dtype=FP32,
                      kv_dtype=FP32, n_exit_heads=n_exit_heads)
    return replace(base, **kw)


_7B = ModelShape(n_layers=32, d_model=4096, n_heads=32, n_kv_heads=32, head_dim=128,
                 d_ffn=11008, vocab=32000, weight_dtype=BF16, kv_dtype=BF16,
                 n_exit_heads=8)
_13B = ModelShape(n_layers=40, d_model=5120, n_heads=40, n_kv_heads=40, head_dim=128,
                  d_ffn=13824, vocab=32000, weight_dtype=BF16, kv_dtype=BF16,
                  n_exit_heads=10)
_8B = ModelShape(n_layers=32, d_model=4096, n_heads=32, n_kv_heads=8, head_dim=128,
                 d_ffn=14336, vocab=128256, weight_dtype=BF16, kv_dtype=BF16,
                 n_exit_heads=8, rope_base=500000.0)

CONFIGS: Dict[str, Workload] = {
    "C1": Workload("C1-tiny-fp32", tiny_shape(), 32, 64, 2, 4, 2.0, 1.0, 0.5, 1,
                   1001, 2001, 3001),
    "C2": Workload("C2-7B-512+512", _7B, 512, 512, 8, 6, 2.0, 1.0, 0.6, 2,
                   1002, 2002, 3002),
    "C3": Workload("C3-7B-4096+256", _7B, 4096, 256, 8, 8, 2.0, 1.0, 0.6, 2,
                   1002, 2003, 3003),
    "C4": Workload("C4-13B-1024+1024", _13B, 1024, 1024, 10, 6, 2.0, 1.0, 0.6, 2,
                   1004, 2004, 3004),
    "C5": Workload("C5-8B-GQA-V128256", _8B, 2048, 1024, 8, 6, 2.0, 1.0, 0.6, 2,
                   1005, 2005, 3005),
}
