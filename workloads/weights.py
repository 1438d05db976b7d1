"""Random-init weights, N(0, 0.02), from a counter-based generator keyed by
(seed, tensor id, layer) so any tensor can be regenerated alone.

Matrices are stored output-major: W[out_features, in_features], so a linear
map is  y = x @ W.T .  Norm gains are 1.0.  For bf16 models the drawn values
are rounded to bf16 (round-to-nearest-even) here, once, because the bf16 value
*is* the model's weight; consumers get either the raw 16-bit patterns or the
exactly-equal float32 upcast.
"""
import numpy as np

_TENSOR_IDS = {"embed": 1, "lm_head": 2, "wqkv": 3, "wo": 4, "w_gate": 5,
               "w_up": 6, "w_down": 7}
INIT_STD = 0.02


def bf16_bits(x):
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rnd) >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(b):
    """uint16 bf16 bit patterns -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32)
            << np.uint32(16)).view(np.float32)


def bf16_round(x):
    """float32 array -> float32 array holding the nearest bf16 values."""
    return bits_to_f32(bf16_bits(x))


class WeightSource:
    """Regenerates any weight tensor of a model on demand."""

    def __init__(self, shape, seed, cache=False):
        self.shape = shape
        self.seed = int(seed)
        self._cache = {} if cache else None

    def dims(self, name):
        s = self.shape
        return {
            "embed": (s.vocab, s.d_model),
            "lm_head": (s.vocab, s.d_model),
            "wqkv": (s.qkv_cols, s.d_model),      # rows: all Q heads, then K heads, then V heads
            "wo": (s.d_model, s.n_q_heads * s.head_dim),
            "w_gate": (s.d_ffn, s.d_model),
            "w_up": (s.d_ffn, s.d_model),
            "w_down": (s.d_model, s.d_ffn),
        }[name]

    def _draw(self, name, layer):
        tid = _TENSOR_IDS[name]
        bitgen = np.random.Philox(key=[self.seed, 0x43464C57],
                                  counter=[0, 0, int(layer) + 1, tid])
        g = np.random.Generator(bitgen)
        rows, cols = self.dims(name)
        w = g.standard_normal((rows, cols), dtype=np.float32)
        w *= np.float32(INIT_STD)
        return w

    def f32(self, name, layer=-1):
        """float32 values the model uses (bf16-rounded for bf16 models)."""
        if self._cache is not None and (name, layer) in self._cache:
            return self._cache[(name, layer)]
        w = self._draw(name, layer)
        if self.shape.dtype == "bf16":
            w = bf16_round(w)
        if self._cache is not None:
            self._cache[(name, layer)] = w
        return w

    def storage(self, name, layer=-1):
        """Array in the model's storage format: float32, or uint16 bf16 bits."""
        w = self._draw(name, layer)
        if self.shape.dtype == "bf16":
            return bf16_bits(w)
        return w

    def norm_gain(self):
        return np.ones(self.shape.d_model, dtype=np.float32)

    def layer_f32(self, layer):
        return {n: self.f32(n, layer) for n in
                ("wqkv", "wo", "w_gate", "w_up", "w_down")}
