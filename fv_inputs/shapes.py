"""Decoder shapes of the target LLM families the paper evaluates (Experiments,
"Models and Tasks": Vicuna 7B/13B, LLaMA2-Chat 7B/13B), plus a tiny instance
for fast CPU checks and a grouped-query 70B-class shape as an extrapolation.
All are Llama-style: RMSNorm, rotary positions, SwiGLU FFN, no biases, untied
embedding and LM head."""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int      # NL
    hidden: int        # h
    n_q_heads: int     # Hq
    n_kv_heads: int    # Hkv
    head_dim: int      # d
    ffn: int           # F
    vocab: int         # V
    dtype: str         # "f32" | "bf16"  (storage type of the weight matrices)
    rope_base: float = 10000.0
    rms_eps: float = 1e-5

    def with_layers(self, n_layers: int) -> "ModelShape":
        return replace(self, n_layers=n_layers, name=f"{self.name}-L{n_layers}")

    def weight_params(self) -> int:
        """Parameters streamed by one forward pass (all matrices, LM head included,
        embedding table excluded: only T rows of it are touched)."""
        per_layer = (self.hidden * self.n_q_heads * self.head_dim
                     + 2 * self.hidden * self.n_kv_heads * self.head_dim
                     + self.n_q_heads * self.head_dim * self.hidden
                     + 3 * self.hidden * self.ffn)
        return self.n_layers * per_layer + self.vocab * self.hidden

    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    def step_bytes(self, prefix_len: int, n_nodes: int) -> int:
        """Algorithmic HBM bytes of one tree-verification step: every weight matrix
        once, K and V of prefix + tree once per layer, embedding rows of the tree."""
        e = self.elem_bytes()
        w = self.weight_params() * e
        kv = self.n_layers * 2 * (prefix_len + n_nodes) * self.n_kv_heads * self.head_dim * e
        emb = n_nodes * self.hidden * e
        return w + kv + emb


SHAPES = {
    "tiny": ModelShape("tiny", 1, 256, 4, 4, 64, 688, 1000, "f32"),
    "tiny-bf16": ModelShape("tiny-bf16", 1, 256, 4, 4, 64, 688, 1000, "bf16"),
    # two layers, grouped-query heads, head_dim 128: exercises everything the big shapes do
    "small-gqa": ModelShape("small-gqa", 2, 512, 8, 2, 128, 1376, 2000, "bf16"),
    "small-gqa-f32": ModelShape("small-gqa-f32", 2, 512, 8, 2, 128, 1376, 2000, "f32"),
    "7b": ModelShape("7b", 32, 4096, 32, 32, 128, 11008, 32000, "bf16"),
    "13b": ModelShape("13b", 40, 5120, 40, 40, 128, 13824, 32000, "bf16"),
    "70b": ModelShape("70b", 80, 8192, 64, 8, 128, 28672, 32000, "bf16"),
}


def shape_by_name(name: str) -> ModelShape:
    return SHAPES[name]
