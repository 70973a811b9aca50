"""Model shapes used by tests and the benchmark.

Shapes "tiny_fp32", "llama8b" and "qwen32b" are the three decoder shapes the
workload list names (a 2-layer fp32 toy, a Llama-3-8B-shaped and a 32B-class
decoder); the remaining entries are small shapes for parity tests that still
span several tiles and ragged tails.  Architecture: pre-norm decoder block with
RMSNorm, rotary embedding (rotate-half pairing), grouped-query attention,
SwiGLU feed-forward, no biases, untied embedding / lm_head.
"""
from dataclasses import dataclass, replace

DTYPE_F32 = 0
DTYPE_BF16 = 1


@dataclass(frozen=True)
class ModelConfig:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5
    dtype: int = DTYPE_BF16        # storage dtype of weights and KV cache
    norm_init: str = "ones"        # "ones" or "random" (1 + 0.1 N(0,1))

    @property
    def q_dim(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads

    def streamed_params(self):
        """Matrix parameters read once per verify step (embedding excluded)."""
        d = self.d_model
        per_layer = d * self.q_dim + 2 * d * self.kv_dim + self.q_dim * d + 3 * d * self.d_ffn
        return self.n_layers * per_layer + self.vocab * d

    def kv_bytes_per_token(self):
        esz = 4 if self.dtype == DTYPE_F32 else 2
        return self.n_layers * 2 * self.kv_dim * esz

    def with_(self, **kw):
        return replace(self, **kw)


CONFIGS = {
    # workload 1: 2 layers, d 256, 4x64 MHA, FFN 1024, vocab 4096, fp32
    "tiny_fp32": ModelConfig("tiny_fp32", 2, 256, 4, 4, 64, 1024, 4096,
                             rope_theta=10000.0, dtype=DTYPE_F32),
    # workloads 2-4: Llama-3-8B shape
    "llama8b": ModelConfig("llama8b", 32, 4096, 32, 8, 128, 14336, 128256,
                           rope_theta=500000.0, dtype=DTYPE_BF16),
    # workload 5: 32B-class shape (q_dim 8192 != d_model)
    "qwen32b": ModelConfig("qwen32b", 64, 5120, 64, 8, 128, 25600, 151936,
                           rope_theta=1000000.0, dtype=DTYPE_BF16),
    # the first 8 layers of the 32B-class shape (same per-layer and lm_head launch shapes)
    "qwen32b_8l": ModelConfig("qwen32b_8l", 8, 5120, 64, 8, 128, 25600, 151936,
                              rope_theta=1000000.0, dtype=DTYPE_BF16),
    # ---- small parity shapes -------------------------------------------------
    # fp32, GQA 2:1, ragged vocab, random norm gains
    "micro_fp32": ModelConfig("micro_fp32", 2, 64, 4, 2, 16, 96, 131,
                              dtype=DTYPE_F32, norm_init="random"),
    "small_fp32": ModelConfig("small_fp32", 3, 192, 6, 2, 32, 320, 1031,
                              dtype=DTYPE_F32, norm_init="random"),
    # bf16, head_dim 128 like the big shapes, GQA 4:1, ragged vocab
    "small_bf16": ModelConfig("small_bf16", 3, 512, 8, 2, 128, 1536, 8209,
                              rope_theta=500000.0, dtype=DTYPE_BF16, norm_init="random"),
    # bf16, head_dim 64, GQA 2:1
    "small_bf16_hd64": ModelConfig("small_bf16_hd64", 2, 256, 4, 2, 64, 768, 4099,
                                   dtype=DTYPE_BF16, norm_init="random"),
    # bf16, 2 layers of the exact 8B layer shape with a cut vocabulary
    "llama8b_2l": ModelConfig("llama8b_2l", 2, 4096, 32, 8, 128, 14336, 32000,
                              rope_theta=500000.0, dtype=DTYPE_BF16),
}


def get_config(name):
    return CONFIGS[name]
