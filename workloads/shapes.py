"""Model shapes and batch recipes of the five synthetic workloads.

The decoder is Llama-style (RMSNorm, rotary embedding, grouped-query attention,
gated SiLU MLP, untied LM head).  Each recipe states the distributions that
`workloads.gen.draw_batch` samples from.
"""
from dataclasses import dataclass


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5

    @property
    def q_dim(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads

    @property
    def layer_params(self):
        d, f = self.d_model, self.d_ffn
        return d * self.q_dim * 2 + d * self.kv_dim * 2 + 3 * d * f

    @property
    def matmul_params(self):
        return self.n_layers * self.layer_params + self.vocab * self.d_model


@dataclass(frozen=True)
class BatchRecipe:
    name: str
    shape: ModelShape
    seed: int
    batch: int
    ctx_dist: str          # "uniform" | "loguniform" | "lognormal"
    ctx_lo: int
    ctx_hi: int
    k_lo: int              # chunk length k drawn uniformly in k_lo..k_hi
    k_hi: int
    p_match: float         # per-token probability that a draft equals the LLM's greedy token
    permute_pages: bool = False
    ctx_median: int = 0    # lognormal only
    ctx_sigma: float = 1.0  # lognormal only (ln-space)
    real_prefill: bool = False  # cached context comes from a real prefill of random ids


TINY = ModelShape("tiny", 2, 256, 4, 4, 64, 1024, 4096)
LLAMA_8B = ModelShape("8b", 32, 4096, 32, 8, 128, 14336, 32000)
LLAMA_70B = ModelShape("70b", 80, 8192, 64, 8, 128, 28672, 32000)

CONFIGS = {
    1: BatchRecipe("c1_tiny_b4_k4", TINY, 1001, 4, "uniform", 32, 128, 4, 4, 0.7,
                   real_prefill=True),
    2: BatchRecipe("c2_8b_b16_k8", LLAMA_8B, 1002, 16, "uniform", 512, 2048, 8, 8, 0.75),
    3: BatchRecipe("c3_8b_b64_ragged", LLAMA_8B, 1003, 64, "loguniform", 128, 4096, 1, 16, 0.6),
    4: BatchRecipe("c4_70b_b32_k8", LLAMA_70B, 1004, 32, "uniform", 1024, 4096, 8, 8, 0.75),
    5: BatchRecipe("c5_8b_b256_permuted", LLAMA_8B, 1005, 256, "lognormal", 64, 8192, 1, 8, 0.7,
                   permute_pages=True, ctx_median=1024, ctx_sigma=1.0),
}

# Standalone confidence workload that accompanies config 5.
C5B_ROWS = 256 * 8
C5B_VOCAB = 128256
C5B_STD = 3.0
C5B_BOOST_HI = 10.0


def config(n: int) -> BatchRecipe:
    return CONFIGS[n]
