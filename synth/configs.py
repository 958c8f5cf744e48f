"""Model shapes of the five workloads (tiny fp32 parity model and four VLM-shaped
bf16 models).  Pure data: no arithmetic of the method.

Notation follows the paper (section 3.2): v visual embeddings, l text tokens,
d hidden size, N target decoder layers, lambda (here K) chain draft length.
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class HivisConfig:
    name: str
    n_layers: int          # N, target decoder layers (the drafter always has one)
    d: int                 # hidden size
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int               # SwiGLU inner width F
    vocab: int
    dtype: str             # "f32" or "bf16": storage type of weights and KV cache
    n_vis: int             # v
    n_text: int            # l at prefill
    K: int                 # chain draft length (paper's lambda)
    batch: int
    gen_tokens: int        # tokens to generate (C1: 16 cycles -> see gen_cycles)
    gen_cycles: int        # if >0, run exactly this many draft-verify cycles instead
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5
    n_resid: int = 4       # r^0..r^3 (section 4, training setup); r^3 reused afterwards
    qkv_bias: bool = False # the attention's q/k/v projections carry bias vectors (the Qwen2.5 language model does)

    @property
    def q_dim(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim

    def scaled(self, **kw):
        return replace(self, **kw)


CONFIGS = {
    "C1": HivisConfig("C1-tiny-f32", 2, 256, 4, 4, 64, 688, 1024, "f32", 64, 32, 4, 1, 0, 16),
    "C2": HivisConfig("C2-llava15-7b", 32, 4096, 32, 32, 128, 11008, 32000, "bf16", 576, 64, 5, 1, 128, 0),
    "C3": HivisConfig("C3-llavanext-7b", 32, 4096, 32, 32, 128, 11008, 32000, "bf16", 2880, 128, 5, 1, 256, 0),
    "C4": HivisConfig("C4-qwen25vl-7b", 28, 3584, 28, 4, 128, 18944, 152064, "bf16", 1024, 96, 6, 1, 256, 0,
                      rope_theta=1.0e6, rms_eps=1e-6),
    "C5": HivisConfig("C5-llava15-13b", 40, 5120, 40, 40, 128, 13824, 32000, "bf16", 576, 256, 7, 4, 512, 0),
}


def get_config(name: str) -> HivisConfig:
    return CONFIGS[name]
