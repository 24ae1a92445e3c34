"""Model shapes of the synthetic workloads (decoder-only, pre-norm, GQA, SwiGLU).

The paper names model families only (LLaMA-2/3, Qwen-2.5; Experimental Setup,
"Models and Datasets"); the shapes below are the family shapes the benchmark
configuration fixes.  `ctx` and `r` are the default context length and number
of candidate tokens verified per step (r plays the role of the paper's
communication ratio, Experimental Setup: 5:1 and 7:1).
"""
from dataclasses import dataclass, replace


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
    rope_theta: float = 1.0e4
    rms_eps: float = 1.0e-5
    ctx: int = 128
    r: int = 4

    def with_layers(self, n_layers: int) -> "ModelShape":
        """Same widths at reduced depth (used to bound oracle time)."""
        return replace(self, n_layers=n_layers, name=f"{self.name}-L{n_layers}")

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def weight_elems_per_layer(self) -> int:
        d = self.d_model
        return d * self.q_dim + 2 * d * self.kv_dim + self.q_dim * d + 3 * d * self.d_ffn

    def streamed_weight_bytes(self) -> int:
        """bf16 bytes one verify step must read: all layers + the vocab head."""
        return 2 * (self.n_layers * self.weight_elems_per_layer() + self.vocab * self.d_model)

    def kv_bytes(self, ctx: int) -> int:
        """bf16 K and V bytes read by verify-attention at context length ctx."""
        return 2 * 2 * self.n_layers * self.kv_dim * ctx


SHAPES = {
    "tiny": ModelShape("tiny", 2, 256, 4, 2, 64, 688, 1024, ctx=128, r=4),
    "llama1b": ModelShape("llama1b", 16, 2048, 32, 8, 64, 8192, 128256, ctx=1024, r=8),
    "llama8b": ModelShape("llama8b", 32, 4096, 32, 8, 128, 14336, 128256, ctx=1024, r=8),
    "llama70b": ModelShape("llama70b", 80, 8192, 64, 8, 128, 28672, 128256, ctx=2048, r=8),
    "qwen7b": ModelShape("qwen7b", 28, 3584, 28, 4, 128, 18944, 152064, ctx=4096, r=8),
}


def shape_by_name(name: str) -> ModelShape:
    return SHAPES[name]
