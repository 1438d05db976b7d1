"""Seeded request batches shaped like the five benchmark configurations, plus
page-pool churn scripts and hand-written integer cost tables for planner tests.

The length distributions stand in for the multi-turn chat and agentic traces
the method was evaluated on; no item of those traces is reproduced here.
"""
from dataclasses import dataclass, field
import numpy as np

from .shapes import SHAPES

CONFIG_NAMES = ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5")
PAGE_TOKENS = 16


@dataclass
class BatchSpec:
    config: str
    shape_name: str
    n_ctx: list                 # context length per request
    n_new: list                 # new-turn prompt length per request
    ctx_tokens: list            # list of int32 arrays
    new_tokens: list            # list of int32 arrays
    chunk_tokens: int           # C
    forced_splits: list = field(default_factory=list)   # [(k_i, c_i)] or []
    forced_mode: int = -1       # -1 planner decides by L_delta, 0 token-wise, 1 layer-wise
    weight_seed: int = 0

    @property
    def shape(self):
        return SHAPES[self.shape_name]


def _ids(rng, n, vocab):
    return rng.integers(0, vocab, size=int(n), dtype=np.int64).astype(np.int32)


def make_batch(config, scale=1.0, vocab=None):
    """Build the batch of one configuration.  `scale` < 1 shrinks every
    context length (kept >= 1 page) for bounded parity cases; the length
    *distribution* is unchanged."""
    if config.startswith("sweep:"):
        # "sweep:<B>:<n>[:<mode>]": B requests of exactly n context tokens on the 8B shape, 128
        # new tokens each (length / batch-size sweeps and the token-wise vs layer-wise crossover)
        f = config.split(":")
        b_req, n = int(f[1]), int(f[2])
        cfg = 6
        rng = np.random.default_rng(1000 + 97 * b_req + n)
        shape_name, n_ctx, n_new = "8b", [n] * b_req, [128] * b_req
        chunk, forced, mode = 512, [], int(f[3]) if len(f) > 3 else -1
    else:
        cfg = {"cfg1": 1, "cfg2": 2, "cfg3": 3, "cfg4": 4, "cfg5": 5}[config]
        rng = np.random.default_rng(1000 + cfg)
    if cfg == 6:
        pass
    elif cfg == 1:
        shape_name, n_ctx, n_new = "tiny", [128, 64], [16, 16]
        chunk, forced, mode = 16, [(64, 2), (32, 2)], 0
    elif cfg == 2:
        shape_name = "8b"
        n_ctx = rng.integers(2048, 16384 + 1, size=8).tolist()
        n_new, chunk, forced, mode = [128] * 8, 512, [], 0
    elif cfg == 3:
        shape_name, n_ctx, n_new = "8b", [131072], [256]
        chunk, forced, mode = 512, [], 1
    elif cfg == 4:
        shape_name = "8b"
        ln = np.exp(rng.normal(np.log(4096.0), 1.0, size=32))
        n_ctx = np.clip(np.rint(ln), 256, 32768).astype(np.int64).tolist()
        n_new = rng.integers(64, 512 + 1, size=32).tolist()
        chunk, forced, mode = 512, [], -1
    else:
        shape_name = "70b-tp8"
        n_ctx = rng.integers(8192, 32768 + 1, size=16).tolist()
        n_new, chunk, forced, mode = [128] * 16, 512, [], -1
    if scale != 1.0:
        n_ctx = [max(PAGE_TOKENS, int(round(n * scale))) for n in n_ctx]
        n_new = [max(1, int(round(m * min(1.0, scale * 4)))) for m in n_new]
    v = vocab if vocab is not None else SHAPES[shape_name].vocab
    ctx = [_ids(rng, n, v) for n in n_ctx]
    new = [_ids(rng, m, v) for m in n_new]
    return BatchSpec(config, shape_name, [int(n) for n in n_ctx],
                     [int(m) for m in n_new], ctx, new, chunk, forced, mode,
                     weight_seed=7000 + cfg)


def random_batch(seed, shape_name, n_req, n_lo, n_hi, m_lo, m_hi, chunk=16):
    """Free-form seeded batch for parity sweeps (ragged lengths on purpose)."""
    rng = np.random.default_rng(seed)
    shape = SHAPES[shape_name]
    n_ctx = rng.integers(n_lo, n_hi + 1, size=n_req).tolist()
    n_new = rng.integers(m_lo, m_hi + 1, size=n_req).tolist()
    ctx = [_ids(rng, n, shape.vocab) for n in n_ctx]
    new = [_ids(rng, m, shape.vocab) for m in n_new]
    return BatchSpec(f"rand{seed}", shape_name, n_ctx, n_new, ctx, new, chunk,
                     [], -1, weight_seed=9000 + seed)


def churn_script(seed, n_pages, n_ops=64, max_tokens=200):
    """Alloc/free script that fragments a page pool: list of
    ("alloc", req_id, n_tokens) / ("free", req_id) in order."""
    rng = np.random.default_rng(seed)
    live, ops, used, next_id = {}, [], 0, 1
    for _ in range(n_ops):
        if live and (rng.random() < 0.45 or used > n_pages // 2):
            rid = sorted(live)[int(rng.integers(0, len(live)))]
            used -= live.pop(rid)
            ops.append(("free", rid))
        else:
            n_tok = int(rng.integers(1, max_tokens + 1))
            need = -(-n_tok // PAGE_TOKENS)
            if used + need > n_pages // 2:
                continue
            live[next_id] = need
            used += need
            ops.append(("alloc", next_id, n_tok))
            next_id += 1
    return ops


def hand_cost_model(kind="balanced"):
    """Integer cost tables (picoseconds) for planner tests that need no GPU.
    Keys follow the cost model's fields: f_c, alpha, beta, f_io, gamma."""
    table = {
        # per layer: fixed, per token, per 1024 causal (q,k) pairs; per copy: fixed, per MiB
        # roughly an 8B-shaped model at ~1 PFLOP/s against a ~55 GB/s host link
        "mi355x_like": dict(f_c=30_000_000, alpha=440_000, beta=16_800,
                            f_io=10_000_000, gamma=19_000_000),
        # compute and I/O of one mid-size chunk cost about the same
        "balanced": dict(f_c=30_000_000, alpha=440_000, beta=16_800,
                         f_io=10_000_000, gamma=140_000_000),
        # a 10 Gbit/s store: recompute wins almost everywhere
        "slow_io": dict(f_c=30_000_000, alpha=440_000, beta=16_800,
                        f_io=10_000_000, gamma=800_000_000),
        # batched recompute: per-unit overheads folded into one-time engine start-ups
        "startup": dict(f_c=0, alpha=464_000, beta=75_000, f_io=0, gamma=18_750_000,
                        s_c=32_000_000_000, s_io=340_000_000),
        # no fixed overheads, no attention term: uniform unit costs
        "uniform": dict(f_c=0, alpha=1_000_000, beta=0, f_io=0,
                        gamma=64_000_000),
    }
    return dict(table[kind])
