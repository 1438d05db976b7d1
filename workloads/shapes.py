"""Model shapes of the five benchmark configurations (decoder-only, pre-norm,
RMSNorm, rotary positions, grouped-query attention, SwiGLU MLP, no biases)."""
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
    rope_base: float
    rms_eps: float
    dtype: str          # "f32" or "bf16": storage type of weights and KV

    @property
    def qkv_cols(self):
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2

    @property
    def kv_bytes_per_token_layer(self):
        return 2 * self.n_kv_heads * self.head_dim * self.elem_bytes

    def with_layers(self, n_layers):
        """Same widths, fewer layers (bounded parity slices)."""
        return ModelShape(self.name + f"-L{n_layers}", n_layers, self.d_model,
                          self.n_q_heads, self.n_kv_heads, self.head_dim,
                          self.d_ffn, self.vocab, self.rope_base, self.rms_eps,
                          self.dtype)

    def with_vocab(self, vocab):
        return ModelShape(self.name + f"-V{vocab}", self.n_layers, self.d_model,
                          self.n_q_heads, self.n_kv_heads, self.head_dim,
                          self.d_ffn, vocab, self.rope_base, self.rms_eps,
                          self.dtype)


SHAPES = {
    # config 1: tiny fp32 decoder
    "tiny": ModelShape("tiny", 2, 256, 4, 4, 64, 688, 1000, 10000.0, 1e-5, "f32"),
    # configs 2-4: Llama-3-8B-shaped, bf16
    "8b": ModelShape("8b", 32, 4096, 32, 8, 128, 14336, 128256, 500000.0, 1e-5, "bf16"),
    # config 5: one TP=8 shard of a 70B-shaped model (vocab shard 128256/8)
    "70b-tp8": ModelShape("70b-tp8", 80, 8192, 8, 1, 128, 3584, 16032, 500000.0, 1e-5, "bf16"),
    # small bf16 shapes for parity tests that span several tiles and ragged tails
    "mini-bf16": ModelShape("mini-bf16", 3, 512, 8, 2, 128, 1408, 2000, 500000.0, 1e-5, "bf16"),
    "mini64-bf16": ModelShape("mini64-bf16", 2, 256, 4, 4, 64, 688, 1000, 10000.0, 1e-5, "bf16"),
    # head_dim 64 with two query heads per KV head, and head_dim 128 with three (an odd group)
    "mini64-gqa2-bf16": ModelShape("mini64-gqa2-bf16", 2, 256, 4, 2, 64, 688, 1000, 10000.0, 1e-5, "bf16"),
    "mini128-gqa3-bf16": ModelShape("mini128-gqa3-bf16", 2, 384, 3, 1, 128, 1024, 1000, 500000.0, 1e-5, "bf16"),
}


def shape_by_name(name):
    return SHAPES[name]
