"""Runs the GEMMs of one decoder layer at a given row count through the
library (cf_op_gemm), plus a plain device copy of known size whose hardware
counters calibrate HBM-traffic counters.  Meant to be run under rocprofv3:

    rocprofv3 --kernel-trace --stats -- python3 -m paper_2604_25080_amd.kernel_probe --shape 8b --rows 10752
    rocprofv3 --pmc FETCH_SIZE -- python3 -m paper_2604_25080_amd.kernel_probe ...
"""
import argparse
import sys

import numpy as np
import torch

from . import binding as cf
from .runtime import Session

COPY_BYTES = 1 << 30


class _TinyWeights:
    """Weight stand-in for a context that is only used to launch single kernels."""

    def __init__(self, shape):
        self.shape = shape

    def storage(self, name, layer=-1):
        s = self.shape
        dims = {"embed": (s.vocab, s.d_model), "lm_head": (s.vocab, s.d_model),
                "wqkv": (s.qkv_cols, s.d_model), "wo": (s.d_model, s.n_q_heads * s.head_dim),
                "w_gate": (s.d_ffn, s.d_model), "w_up": (s.d_ffn, s.d_model),
                "w_down": (s.d_model, s.d_ffn)}[name]
        return np.zeros(dims, dtype=np.uint16 if s.dtype == "bf16" else np.float32)

    def norm_gain(self):
        return np.ones(self.shape.d_model, dtype=np.float32)


def main(argv=None):
    from types import SimpleNamespace
    ap = argparse.ArgumentParser()
    ap.add_argument("--d-model", type=int, default=4096)
    ap.add_argument("--q-cols", type=int, default=4096)
    ap.add_argument("--qkv-cols", type=int, default=6144)
    ap.add_argument("--ffn", type=int, default=14336)
    ap.add_argument("--rows", type=int, default=10752)
    ap.add_argument("--reps", type=int, default=3)
    a = ap.parse_args(argv)
    # a one-layer bf16 context with small matrices: only its streams and dtype are used
    tiny = SimpleNamespace(name="probe", n_layers=1, d_model=256, n_q_heads=2, n_kv_heads=2, head_dim=128,
                           d_ffn=256, vocab=256, rope_base=10000.0, rms_eps=1e-5, dtype="bf16",
                           qkv_cols=768, elem_bytes=2)
    sess = Session(tiny, _TinyWeights(tiny), max_batch=1, max_tokens=256, max_positions=256, n_pages=4)
    dev = torch.device("cuda:0")
    src = torch.zeros(COPY_BYTES, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)                                      # reference copy: reads and writes COPY_BYTES
    torch.cuda.synchronize()
    M, d = a.rows, a.d_model
    gemms = [("gemm_qkv", a.qkv_cols, d, cf.EPI_STORE_F32), ("gemm_oproj", d, a.q_cols, cf.EPI_STORE_F32),
             ("gemm_gate_up", a.ffn, d, cf.EPI_SILU_MUL), ("gemm_down", d, a.ffn, cf.EPI_STORE_F32)]
    for name, N, K, epi in gemms:
        A = torch.randn(M, K, device=dev).to(torch.bfloat16)
        W = (torch.randn(N, K, device=dev) * 0.02).to(torch.bfloat16)
        W2 = (torch.randn(N, K, device=dev) * 0.02).to(torch.bfloat16)
        Cf = torch.zeros(M, N, dtype=torch.float32, device=dev)
        Dt = torch.zeros(M, N, dtype=torch.bfloat16, device=dev)
        torch.cuda.synchronize()
        ms = sess.ctx.op_gemm(A.data_ptr(), W.data_ptr(), W2.data_ptr(), Cf.data_ptr(), Dt.data_ptr(),
                              M, N, K, epi, 0, a.reps)
        fl = 2.0 * M * N * K * (2 if epi == cf.EPI_SILU_MUL else 1)
        in_bytes = (M * K + N * K * (2 if epi == cf.EPI_SILU_MUL else 1)) * 2
        out_bytes = M * N * (2 if epi == cf.EPI_SILU_MUL else 4)
        print(f"{name}: M={M} N={N} K={K} {ms:.4f} ms/launch {fl / ms / 1e9:.1f} TFLOP/s; "
              f"algorithmic bytes in {in_bytes} out {out_bytes}; copy reference {COPY_BYTES} B each way",
              flush=True)
    sess.close()


if __name__ == "__main__":
    main(sys.argv[1:])
