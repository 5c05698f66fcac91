"""Model shapes and workload sizes of the synthetic stand-in configurations.

The paper evaluates on Llama-family checkpoints fine-tuned for early exit and on
public text datasets (Section 5.1, Appendix B.1).  Neither is available here, so
each configuration below takes the *shape* of one of the paper's models
(Table 1 rows), random weights whose residual branches shrink geometrically with
depth (so that early-exit agreement rises with depth, the property the method
exploits), and a uniform-random prompt.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict


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
    rope_theta: float
    tied_embeddings: bool
    weight_dtype: str          # "fp32" or "bf16"
    branch_decay: float        # attn-out and ffn-down of layer l scaled by decay**l
    prompt_len: int
    gen_len: int
    d_max: int                 # cap on the speculation length
    config_id: int             # enters the seeds
    rms_eps: float = 1e-5
    init_std: float = 0.02
    norm_gain_std: float = 0.0  # 0 => all norm gains are exactly 1
    prefill_window: int = 32   # Appendix B.2: last 32 context tokens seed the statistics
    omega: float = 0.95        # Appendix B.2: decay factor of the weighted sum

    @property
    def weight_seed(self) -> int:
        return 0xDE100000 + self.config_id

    @property
    def prompt_seed(self) -> int:
        return 0x5EED0000 + self.config_id

    @property
    def max_context(self) -> int:
        return self.prompt_len + self.gen_len + self.d_max + 1

    def n_params(self) -> int:
        d, f, v = self.d_model, self.d_ffn, self.vocab
        attn = d * self.n_q_heads * self.head_dim * 2 + d * self.n_kv_heads * self.head_dim * 2
        ffn = 3 * d * f
        head = v * d * (1 if self.tied_embeddings else 2)
        return self.n_layers * (attn + ffn + 2 * d) + head + d

    def layer_weight_bytes(self) -> int:
        d, f = self.d_model, self.d_ffn
        attn = d * self.n_q_heads * self.head_dim * 2 + d * self.n_kv_heads * self.head_dim * 2
        return (attn + 3 * d * f) * (2 if self.weight_dtype == "bf16" else 4)

    def head_weight_bytes(self) -> int:
        return self.vocab * self.d_model * (2 if self.weight_dtype == "bf16" else 4)

    def as_dict(self) -> dict:
        return asdict(self)


CONFIGS = {
    # C1: tiny fp32 decoder, oracle finishes in seconds.
    "tiny": ModelConfig("tiny", 4, 256, 4, 4, 64, 688, 4096, 1e4, False, "fp32", 0.5,
                        32, 64, 4, 1),
    # C2: Llama-3.2-1B shape, tied embeddings, GQA 32/8.
    "llama1b": ModelConfig("llama1b", 16, 2048, 32, 8, 64, 8192, 128256, 5e5, True, "bf16", 0.5,
                           512, 256, 8, 2),
    # C3: Llama-2-7B shape (headline).
    "llama7b": ModelConfig("llama7b", 32, 4096, 32, 32, 128, 11008, 32000, 1e4, False, "bf16", 0.8,
                           1024, 256, 8, 3),
    # C4: Llama-2-13B shape.
    "llama13b": ModelConfig("llama13b", 40, 5120, 40, 40, 128, 13824, 32000, 1e4, False, "bf16", 0.85,
                            2048, 512, 10, 4),
    # C5: Llama-2-70B shape, GQA 64/8.
    "llama70b": ModelConfig("llama70b", 80, 8192, 64, 8, 128, 28672, 32000, 1e4, False, "bf16", 0.93,
                            1024, 256, 12, 5),
    # Reduced shapes for element-by-element parity: several tiles, ragged tails,
    # GQA, tied head, non-unit norm gains.
    "mini_gqa": ModelConfig("mini_gqa", 6, 512, 8, 2, 64, 1384, 8008, 5e5, True, "bf16", 0.6,
                            45, 48, 6, 11, norm_gain_std=0.1),
    "mini_mha": ModelConfig("mini_mha", 5, 384, 3, 3, 128, 1000, 5000, 1e4, False, "bf16", 0.7,
                            70, 40, 9, 12, norm_gain_std=0.1),
    # one kv head for eight query heads, n_q*head_dim != d_model
    "mini_g8": ModelConfig("mini_g8", 4, 256, 8, 1, 128, 704, 3000, 1e4, False, "bf16", 0.6,
                           53, 40, 7, 14, norm_gain_std=0.1),
    # the paper's cap on the speculation length (Appendix B.2: d_max = 18): rounds of more than 16 rows
    "mini_d18": ModelConfig("mini_d18", 5, 512, 8, 2, 64, 1384, 5000, 1e4, False, "bf16", 0.6,
                            40, 64, 18, 15, norm_gain_std=0.1),
    # d_model of the 7B shape on three layers: 128 k tiles per row and at least 256 row blocks in every matrix
    # (the shapes for which the one-row GEMV takes several row blocks per work-group), ragged vocabulary
    "wide_d4096": ModelConfig("wide_d4096", 3, 4096, 32, 8, 128, 4096, 4111, 1e4, False, "bf16", 0.6,
                              40, 40, 6, 16, norm_gain_std=0.1),
    # d_model of the 13B shape on three layers: 160 k tiles per row (the one-row GEMV then takes groups of 5 tiles),
    # as many kv heads as query heads, the feed-forward width equal to d_model so that the down projection takes
    # the same kernel
    "wide_d5120": ModelConfig("wide_d5120", 3, 5120, 40, 40, 128, 5120, 4111, 1e4, False, "bf16", 0.6,
                              40, 40, 6, 18, norm_gain_std=0.1),
    "mini_fp32": ModelConfig("mini_fp32", 3, 192, 6, 2, 32, 520, 3000, 1e4, False, "fp32", 0.6,
                             21, 24, 5, 13, norm_gain_std=0.1),
}


def get_config(name: str) -> ModelConfig:
    return CONFIGS[name]
