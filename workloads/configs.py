"""The five workload configurations (model shape + context + verify recipe)."""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    index: int                 # 1..5, selects the seed stream
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str                 # "f32" | "bf16"
    rope_theta: float
    rms_eps: float
    ctx: int                   # prefilled context length (config 5: median)
    chunk: int                 # prefill chunk length
    k: int                     # draft tokens per verify (config 5: maximum)
    steps: int                 # successive verify steps
    mode: str                  # "greedy" | "stochastic" | "mixed"
    temperature: float = 0.0
    p_copy: float = 0.0        # probability that a draft is a copied context span
    batch: int = 1
    page_tokens: int = 0       # 0 = contiguous KV cache

    @property
    def rows(self):
        return self.k + 1

    def weight_bytes(self):
        """Bytes of every weight matrix once (tied embedding counted once)."""
        es = 4 if self.dtype == "f32" else 2
        d, hd = self.d_model, self.head_dim
        per_layer = ((self.n_q_heads + 2 * self.n_kv_heads) * hd * d + d * self.n_q_heads * hd
                     + 3 * self.d_ffn * d)
        return es * (self.n_layers * per_layer + self.vocab * d)

    def kv_bytes_per_token(self):
        es = 4 if self.dtype == "f32" else 2
        return es * 2 * self.n_layers * self.n_kv_heads * self.head_dim


CONFIGS = {
    "tiny_f32": WorkloadConfig("tiny_f32", 1, 2, 256, 4, 4, 64, 1024, 4096, "f32", 1e4, 1e-6,
                               ctx=512, chunk=128, k=4, steps=1, mode="greedy", p_copy=0.5),
    "0.5b_k8": WorkloadConfig("0.5b_k8", 2, 24, 896, 14, 2, 64, 4864, 151936, "bf16", 1e6, 1e-6,
                              ctx=1024, chunk=256, k=8, steps=1, mode="greedy", p_copy=0.6),
    "1.5b_k16": WorkloadConfig("1.5b_k16", 3, 28, 1536, 12, 2, 128, 8960, 151936, "bf16", 1e6, 1e-6,
                               ctx=2048, chunk=256, k=16, steps=64, mode="stochastic",
                               temperature=0.8),
    "3b_k32": WorkloadConfig("3b_k32", 4, 28, 3072, 24, 8, 128, 8192, 128256, "bf16", 5e5, 1e-6,
                             ctx=4096, chunk=256, k=32, steps=1, mode="greedy"),
    "1.5b_rag_mix": WorkloadConfig("1.5b_rag_mix", 5, 28, 1536, 12, 2, 128, 8960, 151936, "bf16",
                                   1e6, 1e-6, ctx=2048, chunk=256, k=32, steps=1, mode="mixed",
                                   temperature=0.8, batch=16, page_tokens=64),
}


def scaled(cfg: WorkloadConfig, **kw) -> WorkloadConfig:
    """A reduced copy of a config (fewer layers, shorter context ...) for tests
    the CPU oracle must finish in seconds; the seed stream stays the same."""
    return replace(cfg, **kw)
