"""Runs causal self-attention of ONE request of a given length through the
library: an all-recompute restore of a two-layer model with the 8B widths
(32 query heads, 8 KV heads, head_dim 128), so that the attention kernel sees
the benchmark's head geometry at a chosen context length.  Meant to be run
plain (prints the attention kernel's event-timed rate) or under rocprofv3:

    python3 -m paper_2604_25080_amd.attention_probe --tokens 16384
    rocprofv3 --pmc SQ_INSTS_MFMA SQ_INSTS_VALU ... -- python3 -m paper_2604_25080_amd.attention_probe --tokens 16384
"""
import argparse

import numpy as np

from .runtime import Session


def main(argv=None):
    from workloads import SHAPES, WeightSource
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=16384)
    ap.add_argument("--reps", type=int, default=2)
    a = ap.parse_args(argv)
    n = a.tokens
    shape = SHAPES["8b"].with_layers(2).with_vocab(4096)
    sess = Session(shape, WeightSource(shape, 5), max_batch=1, max_tokens=n + 128, max_positions=n + 256,
                   n_pages=n // 16 + 64)
    toks = np.random.default_rng(0).integers(0, 4096, size=n).astype(np.int32)
    sess.cache.alloc(1, n + 128)
    sess.ctx.profile(["attention"])
    req = [dict(req_id=1, ctx_tokens=toks, new_tokens=toks[:128], host_kv=None)]
    for _ in range(a.reps):
        sess.restore(req, [(0, n, 2)], want_logits=False)
    st = sess.ctx.profile_read()["attention"]
    pairs = n * (n + 1) / 2
    print(f"tokens {n}: {st['launches']} attention launches, {st['total_ms'] / st['launches']:.3f} ms each, "
          f"{st['work'] / st['total_ms'] / 1e9:.1f} TFLOP/s "
          f"({pairs * 4 * shape.n_q_heads * shape.head_dim / 1e12:.2f} TFLOP per launch: 4*Hq*hd per causal pair)",
          flush=True)
    sess.close()


if __name__ == "__main__":
    main()
