"""Device-memory plumbing around the C-ABI library: uploads weights, owns the
page pool, the workspace, the pinned host KV blocks and the two HIP streams
(all through PyTorch-ROCm), and hands raw addresses to the library.  No step
of the restoration path is computed here."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

from . import binding as cf

_LAYER_MATS = ("wqkv", "wo", "w_gate", "w_up", "w_down")


def _to_device(arr, device):
    if arr.dtype == np.uint16:        # bf16 bit patterns
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


class Session:
    """One model + one page pool + one library context on one GPU.

    weight_source: object with .storage(name, layer) -> numpy array in the
    model's storage format (float32, or uint16 bf16 bits) and .norm_gain()."""

    def __init__(self, shape, weight_source, max_batch, max_tokens, max_positions, n_pages,
                 chunk_rows=0, staging_bytes=0, device="cuda:0", gen_threads=8,
                 pool_fill=None):
        if not torch.cuda.is_available():
            raise RuntimeError("the restoration path needs a GPU; there is no CPU fallback")
        self.shape = shape
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.desc = cf.model_desc(shape)
        self.dtype = cf.CF_F32 if shape.dtype == "f32" else cf.CF_BF16
        self.tdtype = torch.float32 if shape.dtype == "f32" else torch.bfloat16
        self._keep = []

        gain = torch.from_numpy(weight_source.norm_gain()).to(self.device)
        self._keep.append(gain)
        jobs = [("embed", -1), ("lm_head", -1)] + [(n, l) for l in range(shape.n_layers)
                                                   for n in _LAYER_MATS]

        def gen(job):
            return job, weight_source.storage(*job)

        tensors = {}
        with ThreadPoolExecutor(max_workers=gen_threads) as ex:
            for job, arr in ex.map(gen, jobs):
                tensors[job] = _to_device(arr, self.device)
        self.weights = tensors
        layers = []
        for l in range(shape.n_layers):
            d = {n: tensors[(n, l)].data_ptr() for n in _LAYER_MATS}
            d["attn_norm"] = gain.data_ptr()
            d["mlp_norm"] = gain.data_ptr()
            layers.append(d)
        wdict = dict(embed=tensors[("embed", -1)].data_ptr(),
                     lm_head=tensors[("lm_head", -1)].data_ptr(),
                     final_norm=gain.data_ptr(), layers=layers)

        self.page_bytes = 2 * shape.n_kv_heads * cf.PAGE_TOKENS * shape.head_dim * shape.elem_bytes
        self.n_pages = n_pages
        self.pool = torch.empty(shape.n_layers * n_pages * self.page_bytes, dtype=torch.uint8,
                                device=self.device)
        if pool_fill is not None:
            self.pool.fill_(pool_fill)
        self.cache = cf.Cache(self.pool.data_ptr(), self.pool.numel(), shape.n_layers,
                              shape.n_kv_heads, shape.head_dim, self.dtype)
        self.opts = cf.ctx_opts(max_batch, max_tokens, max_positions, chunk_rows, staging_bytes)
        ws_bytes = cf.workspace_bytes(self.desc, self.opts)
        self.workspace = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=self.device)
        ws_ptr = (self.workspace.data_ptr() + 255) // 256 * 256
        self.compute_stream = torch.cuda.Stream(device=self.device)
        self.copy_stream = torch.cuda.Stream(device=self.device)
        torch.cuda.synchronize()
        self.ctx = cf.Ctx(self.desc, wdict, self.opts, ws_ptr, ws_bytes,
                          self.compute_stream.cuda_stream, self.copy_stream.cuda_stream)
        self.logits = torch.zeros(max_batch, shape.vocab, dtype=torch.float32, device=self.device)

    def close(self):
        torch.cuda.synchronize()
        self.ctx.close()
        self.cache.close()

    # ------------------------------------------------------------ host KV blocks
    def host_kv_bytes(self, n_ctx):
        s = self.shape
        return cf.host_kv_bytes(s.n_layers, s.n_kv_heads, s.head_dim, self.dtype, n_ctx)

    def pinned(self, n_bytes):
        return torch.empty(max(n_bytes, 1), dtype=torch.uint8, pin_memory=True)

    def pin_host_kv(self, block):
        """numpy array in the host layout (float32, or uint16 bf16 bits) -> pinned tensor."""
        raw = np.ascontiguousarray(block).view(np.uint8).reshape(-1)
        t = self.pinned(raw.size)
        t[:raw.size].copy_(torch.from_numpy(raw))
        return t

    def offload(self, req_id, n_ctx):
        t = self.pinned(self.host_kv_bytes(n_ctx))
        self.ctx.offload(self.cache, req_id, n_ctx, t.data_ptr())
        return t

    # ------------------------------------------------------------------ the path
    def restore(self, requests, splits, want_logits=True):
        """requests: list of dict(req_id, ctx_tokens, new_tokens, host_kv=pinned tensor or
        None[, boundary_h=float32 host tensor [n_ctx, d] for a stage above layer 0]).
        Returns (logits tensor [B, vocab] or None, timing dict)."""
        # the library's streams do not order against torch's: finish pending torch work
        # (fills, copies into the pool) before the blocking call
        torch.cuda.current_stream(self.device).synchronize()
        reqs = []
        for r in requests:
            hk, bh = r.get("host_kv"), r.get("boundary_h")
            reqs.append(dict(req_id=r["req_id"], ctx_tokens=r["ctx_tokens"],
                             new_tokens=r["new_tokens"],
                             host_kv=hk.data_ptr() if hk is not None else 0,
                             boundary_h=(bh.data_ptr() if hasattr(bh, "data_ptr") else bh) if bh is not None else 0))
        tm = self.ctx.restore_batch(self.cache, reqs, splits,
                                    self.logits.data_ptr() if want_logits else 0)
        return (self.logits[:len(requests)] if want_logits else None), tm

    def restore_dynamic(self, requests, cost, opts, want_logits=True, step_cap_ps=0, order=0,
                        units_per_request=0, overlap=None):
        """Restore without a precomputed split: the engines claim units at run time.
        Returns (logits or None, splits [(mode,k,cut)], timing dict, stats dict)."""
        torch.cuda.current_stream(self.device).synchronize()
        reqs = [dict(req_id=r["req_id"], ctx_tokens=r["ctx_tokens"], new_tokens=r["new_tokens"],
                     host_kv=r["host_kv"].data_ptr() if r.get("host_kv") is not None else 0)
                for r in requests]
        splits, tm, st = self.ctx.restore_dynamic(self.cache, reqs, cost, opts,
                                                  self.logits.data_ptr() if want_logits else 0,
                                                  step_cap_ps, order, units_per_request, overlap)
        return (self.logits[:len(requests)] if want_logits else None), splits, tm, st

    # -------------------------------------------------------------- introspection
    def read_pages(self, req_id, n_tokens, layers=None):
        """Raw page bytes of a request: uint8 numpy [L, n_pages_req, page_bytes] (or only the
        listed layers, in that order)."""
        table = self.cache.page_table(req_id)[:-(-n_tokens // cf.PAGE_TOKENS)]
        view = self.pool.view(self.shape.n_layers, self.n_pages, self.page_bytes)
        idx = torch.tensor(table, dtype=torch.long, device=self.device)
        if layers is not None:
            lidx = torch.tensor(list(layers), dtype=torch.long, device=self.device)
            return view[lidx[:, None], idx[None, :]].cpu().numpy()
        return view[:, idx].cpu().numpy()
