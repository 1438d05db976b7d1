#!/usr/bin/env python3
"""Benchmark of batched hybrid KV-cache restoration on one MI355X.

One step = one pass of the whole hot path over one batch: plan the splits
(cf_plan_batch: the two-pointer scheduler over the calibrated cost model, with
the new turn, contention and the two extremes taken into account), recompute ‖
load+scatter, join, prefill the new-turn tokens over the restored pages,
first-token logits, and the closed-loop correction of the cost model.  Inputs
are synthetic (seeded token ids, random-init weights of the named shape) and
already resident (weights in HBM, host KV in pinned memory) when the timed
region starts.

    python bench.py --gpus 1 --steps K --warmup W [--config cfg4] [--plan planner]

The timed workload is configuration 4 (the largest single-GPU one: 32
requests, log-normal context lengths); after the timed region the other
configurations get a short run each (`configs` in the output; --no-extras
skips them).  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0       # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3


def log(*a):
    print(*a, file=sys.stderr, flush=True)



def host_cores():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline(batch, n_tok=4096, n_layers=6):
    """Time the CPU oracle (as it stands) on bounded samples: a slice of the timed workload's
    recompute, configuration 1 end to end, and the planner on every configuration's batch."""
    import numpy as np
    from oracle import planner as OP
    from oracle import transformer as T
    from workloads import WeightSource, hand_cost_model, make_batch
    import paper_2604_25080_amd as cf
    shape = batch.shape
    ws = WeightSource(shape, batch.weight_seed, cache=True)
    longest = int(np.argmax(batch.n_ctx))
    n_tok = min(n_tok, batch.n_ctx[longest])
    n_layers = min(n_layers, shape.n_layers)
    ws.f32("embed")
    for l in range(n_layers):
        ws.layer_f32(l)
    t0 = time.perf_counter()
    T.prefill(shape, ws, batch.ctx_tokens[longest][:n_tok], n_layers=n_layers, dtype=np.float32)
    dt = time.perf_counter() - t0
    tok_layers_per_s = n_tok * n_layers / dt
    # configuration 1 end to end: full prefill, hybrid restore under the forced splits, new turn, logits
    b1 = make_batch("cfg1")
    ws1 = WeightSource(b1.shape, b1.weight_seed, cache=True)
    t0 = time.perf_counter()
    for i in range(len(b1.n_ctx)):
        kv_full, _ = T.prefill(b1.shape, ws1, b1.ctx_tokens[i])
        cache = T.restore(b1.shape, ws1, b1.ctx_tokens[i], kv_full, *b1.forced_splits[i])
        T.first_token_logits(b1.shape, ws1, cache, b1.new_tokens[i])
    dt1 = time.perf_counter() - t0
    # planner: microseconds per plan, oracle (pure Python) against the library (C++)
    planner = {}
    for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
        bb = make_batch(name)
        d = hand_cost_model("startup")
        model = (bb.shape.n_layers, bb.shape.d_model, bb.shape.n_q_heads, bb.shape.n_kv_heads, bb.shape.head_dim,
                 bb.shape.d_ffn, bb.shape.elem_bytes)
        l_delta = 4096 if bb.forced_mode < 0 else 0
        reps_o = 3
        t0 = time.perf_counter()
        for _ in range(reps_o):
            OP.plan_batch(OP.CostModel(**d), (1000, 1000), model, bb.chunk_tokens, l_delta, bb.forced_mode, 0, True,
                          bb.n_ctx, bb.n_new)
        t_o = (time.perf_counter() - t0) / reps_o
        cm, ov, desc = cf.cost_model(**d), cf.overlap_model(), cf.model_desc(bb.shape)
        bo = cf.batch_plan_opts(bb.chunk_tokens, l_delta, bb.forced_mode)
        reps_c = 50
        t0 = time.perf_counter()
        for _ in range(reps_c):
            cf.plan_batch(cm, ov, desc, bo, bb.n_ctx, bb.n_new)
        t_c = (time.perf_counter() - t0) / reps_c
        planner[name] = {"oracle_us": t_o * 1e6, "library_us": t_c * 1e6}
    return {
        "value": tok_layers_per_s / shape.n_layers, "unit": "restored tokens/s",
        "cores": host_cores(), "kind": "oracle",
        "sample": (f"oracle float32 recompute of the first {n_tok} tokens of the longest request through "
                   f"{n_layers} of {shape.n_layers} layers ({dt:.2f} s), scaled by layer count; "
                   "loading is a memcpy and is not part of the sample"),
        "token_layers_per_s": tok_layers_per_s,
        "cfg1_end_to_end": {"seconds": dt1, "restored_tokens_per_s": sum(b1.n_ctx) / dt1,
                            "what": "oracle float64: full prefill, hybrid restore under the forced splits, "
                                    "new turn and logits of both requests"},
        "planner_us_per_plan": planner,
    }


class _ZeroWeights:
    """Weight stand-in for a context that is only used to launch single kernels."""

    def __init__(self, shape):
        self.shape = shape

    def storage(self, name, layer=-1):
        import numpy as np
        s = self.shape
        dims = {"embed": (s.vocab, s.d_model), "lm_head": (s.vocab, s.d_model),
                "wqkv": (s.qkv_cols, s.d_model), "wo": (s.d_model, s.n_q_heads * s.head_dim),
                "w_gate": (s.d_ffn, s.d_model), "w_up": (s.d_ffn, s.d_model),
                "w_down": (s.d_model, s.d_ffn)}[name]
        return np.zeros(dims, dtype=np.uint16 if s.dtype == "bf16" else np.float32)

    def norm_gain(self):
        import numpy as np
        return np.ones(self.shape.d_model, dtype=np.float32)


def probe_gemm(a):
    """--probe gemm: the four GEMMs of one decoder layer of the 8B shape at --rows rows through
    cf_op_gemm, after a plain 1 GiB device copy whose FETCH_SIZE / WRITE_SIZE readings calibrate
    those counters.  For rocprofv3 (--kernel-trace --stats, or --pmc) runs."""
    import torch
    import paper_2604_25080_amd as cf
    from paper_2604_25080_amd.runtime import Session
    from workloads import SHAPES
    copy_bytes = 1 << 30
    big = SHAPES["8b"]
    tiny = SHAPES["mini-bf16"].with_layers(1)        # only the context's streams and dtype are used
    sess = Session(tiny, _ZeroWeights(tiny), max_batch=1, max_tokens=256, max_positions=256, n_pages=4)
    dev = torch.device("cuda:0")
    src = torch.zeros(copy_bytes, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)                                      # reference copy: reads and writes copy_bytes
    torch.cuda.synchronize()
    M, d = a.rows, big.d_model
    gemms = [("gemm_qkv", big.qkv_cols, d, cf.EPI_STORE_F32),
             ("gemm_oproj", d, big.n_q_heads * big.head_dim, cf.EPI_STORE_F32),
             ("gemm_gate_up", big.d_ffn, d, cf.EPI_SILU_MUL), ("gemm_down", d, big.d_ffn, cf.EPI_STORE_F32)]
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
              f"algorithmic bytes in {in_bytes} out {out_bytes}; copy reference {copy_bytes} B each way",
              flush=True)
    sess.close()


def probe_attention(a):
    """--probe attention: causal self-attention of ONE request of --tokens tokens -- an
    all-recompute restore of a two-layer model with the 8B widths -- so that the attention
    kernel sees the benchmark's head geometry at a chosen context length."""
    import numpy as np
    from paper_2604_25080_amd.runtime import Session
    from workloads import SHAPES, WeightSource
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



class Bench:
    """One model on the GPU and the batches that run on it."""

    def __init__(self, args, batches):
        import torch
        import paper_2604_25080_amd as cf
        from paper_2604_25080_amd.runtime import Session
        from workloads import WeightSource
        self.args, self.cf, self.torch = args, cf, torch
        self.shape = batches[0].shape
        self.calib_tokens = 8192
        pages = max(sum(-(-(n + m) // 16) for n, m in zip(b.n_ctx, b.n_new)) for b in batches)
        pages += 2 * self.calib_tokens // 16 + 64
        t0 = time.perf_counter()
        self.sess = Session(self.shape, WeightSource(self.shape, batches[0].weight_seed),
                            max_batch=max(max(len(b.n_ctx) for b in batches), 8),
                            max_tokens=max(max(sum(b.n_ctx) + sum(b.n_new) for b in batches), self.calib_tokens),
                            max_positions=max(max(max(n + m for n, m in zip(b.n_ctx, b.n_new)) for b in batches),
                                              self.calib_tokens) + 16,
                            n_pages=pages, chunk_rows=args.chunk_rows, gen_threads=16)
        log(f"[bench] {self.shape.name}: weights + pool + workspace ready in {time.perf_counter() - t0:.1f} s")
        self.sess.ctx.set_pipelined_join(not args.sequential_join)
        self.sess.ctx.set_load_path({"auto": 0, "staged": 1, "direct": 2}[args.load_path], args.load_workgroups)
        self.desc = cf.model_desc(self.shape)
        self.cost = self.overlap = None

    # ---- manufacture the host KV of a batch (not timed): full prefill on the GPU, then offload
    def prepare(self, batch, stage=None):
        sess, torch = self.sess, self.torch
        B, L = len(batch.n_ctx), self.shape.n_layers
        t0 = time.perf_counter()
        reqs = []
        for i in range(B):
            sess.cache.alloc(1 + i, batch.n_ctx[i] + batch.n_new[i])
            reqs.append(dict(req_id=1 + i, ctx_tokens=batch.ctx_tokens[i], new_tokens=batch.new_tokens[i],
                             host_kv=None))
        sum_ctx = sum(batch.n_ctx)
        if stage:
            cap = torch.empty(sum_ctx, self.shape.d_model, dtype=torch.float32, device="cuda")
            sess.ctx.capture_boundary(stage[0], cap.data_ptr(), sum_ctx)
        _, tm_full = sess.restore(reqs, [(0, n, L) for n in batch.n_ctx], want_logits=False)
        if stage:      # packed order of an all-recompute pass with equal cuts = call order
            off = 0
            for i in range(B):
                bh = torch.empty(batch.n_ctx[i], self.shape.d_model, dtype=torch.float32, pin_memory=True)
                bh.copy_(cap[off:off + batch.n_ctx[i]])
                reqs[i]["boundary_h"] = bh
                off += batch.n_ctx[i]
            del cap
        for i in range(B):
            reqs[i]["host_kv"] = sess.pinned(sess.host_kv_bytes(batch.n_ctx[i]))
        t_off = time.perf_counter()
        for i in range(B):
            sess.ctx.offload(sess.cache, 1 + i, batch.n_ctx[i], reqs[i]["host_kv"].data_ptr())
        t_off = time.perf_counter() - t_off
        offload_gbs = sum(sess.host_kv_bytes(n) for n in batch.n_ctx) / t_off / 1e9
        log(f"[bench] {batch.config}: B={B} sum n_ctx={sum_ctx} sum n_new={sum(batch.n_new)}; host KV manufactured in "
            f"{time.perf_counter() - t0:.1f} s (offload {offload_gbs:.1f} GB/s, all-recompute pass "
            f"{tm_full['compute_ms']:.1f} ms, {tm_full['recompute_flops'] / tm_full['compute_ms'] / 1e9:.0f} TFLOP/s)")
        return reqs, tm_full, offload_gbs

    def release(self, batch, reqs):
        for i in range(len(batch.n_ctx)):
            self.sess.cache.free(1 + i)
        for r in reqs:
            r["host_kv"] = None
            r.pop("boundary_h", None)
        self.torch.cuda.empty_cache()

    # ---- measured rooflines of the load path, and the cost model (Sec. 3.1: profiled costs)
    def calibrate(self, reqs):
        sess, torch, cf = self.sess, self.torch, self.cf
        sess.ctx.set_link_throttle(self.args.link_gbps / 8.0)
        big = max(reqs, key=lambda r: r["host_kv"].numel())["host_kv"]
        h2d_bytes = min(big.numel(), 1 << 30)
        dev_scratch = torch.empty(h2d_bytes, dtype=torch.uint8, device="cuda")
        self.h2d_gbs = sess.ctx.measure_h2d(big.data_ptr(), dev_scratch.data_ptr(), h2d_bytes, reps=4)
        del dev_scratch
        need = sess.host_kv_bytes(self.calib_tokens)
        scratch = big if big.numel() >= need else sess.pinned(need)
        self.cost = sess.ctx.calibrate(sess.cache, scratch.data_ptr(), scratch.numel())
        self.overlap = sess.ctx.calibrate_overlap(sess.cache, scratch.data_ptr(), scratch.numel(), self.cost)
        self.cost0 = self.cost_dict()
        self.dyn_seeded = False
        opts = cf.plan_opts(512, 0, self.shape.n_layers, self.shape.kv_bytes_per_token_layer, -1)
        self.l_delta = cf.derive_l_delta(self.cost, opts, 32768)
        self.kv_only = cf.plan_batch(self.cost, self.overlap, self.desc, cf.batch_plan_opts(512, 0), [512])[1].kv_only_permille
        log(f"[bench] H2D {self.h2d_gbs:.1f} GB/s; cost model {self.cost0}; L_delta {self.l_delta}")

    def cost_dict(self):
        c, o = self.cost, self.overlap
        return dict(f_c=c.f_c, alpha=c.alpha, beta=c.beta, f_io=c.f_io, gamma=c.gamma, s_c=c.s_c, s_io=c.s_io,
                    overlap_comp_permille=o.comp_permille, overlap_io_permille=o.io_permille)

    # ---- one step of the hot path
    def step(self, batch, reqs, plan, stage=None):
        cf, sess, args = self.cf, self.sess, self.args
        L = (stage[1] - stage[0]) if stage else self.shape.n_layers
        if plan == "dynamic":
            opts = cf.plan_opts(batch.chunk_tokens, self.l_delta, L, self.shape.kv_bytes_per_token_layer,
                                batch.forced_mode, kv_only_permille=self.kv_only)
            cost = self.cost
            if args.model_skew:       # a deliberately wrong cost table in front of the run-time scheduler
                fc, fio = (float(x) for x in args.model_skew.split(":"))
                cost = cf.cost_model(**{k: int(getattr(self.cost, k) * (fc if k in ("f_c", "alpha", "beta", "s_c") else fio))
                                        for k in ("f_c", "alpha", "beta", "f_io", "gamma", "s_c", "s_io")})
            _, splits, tm, st = sess.restore_dynamic(reqs, cost, opts, want_logits=True,
                                                     step_cap_ps=int(args.step_cap_ms * 1e9),
                                                     units_per_request=args.units_per_request,
                                                     overlap=None if self.dyn_seeded else self.overlap)
            self.dyn_seeded = True    # from here on the context's own measured ratios carry over
            log(f"[bench]   {batch.config} run-time: comp {tm['compute_ms']:.1f} (waited {tm['compute_wait_ms']:.1f}) "
                f"copy {tm['copy_ms']:.1f} ttft {tm['total_ms']:.1f} ms; recomputed "
                f"{sum(s_[1] for s_ in splits if s_[2] > 0)} tokens; {st}")
            return splits, dict(kind="run-time", stats=st), tm
        info = None
        if plan == "planner" and batch.forced_splits:
            splits = [(0, k, c) for k, c in batch.forced_splits]
        elif plan in ("planner", "per_request"):
            bo = cf.batch_plan_opts(batch.chunk_tokens, self.l_delta, batch.forced_mode,
                                    pipelined_join=not args.sequential_join, stage_layers=L if stage else 0,
                                    stage_first_layer=stage[0] if stage else 0)
            if plan == "planner":
                splits, info = cf.plan_batch(self.cost, self.overlap, self.desc, bo, batch.n_ctx, batch.n_new)
            else:   # comparison plan: every request planned alone, as if it had both engines to itself
                splits = [cf.plan_batch(self.cost, self.overlap, self.desc, bo, [n], [m])[0][0]
                          for n, m in zip(batch.n_ctx, batch.n_new)]
        elif plan == "all_recompute":
            splits = [(0, n, L) for n in batch.n_ctx]
        elif plan == "all_load":
            splits = [(0, 0, L) for n in batch.n_ctx]
        elif plan.startswith("cut="):
            splits = [(1, n, int(plan[4:])) for n in batch.n_ctx]
        else:
            raise SystemExit(f"unknown plan {plan}")
        _, tm = sess.restore(reqs, splits, want_logits=not stage)
        if info is not None:
            cf.plan_feedback(self.cost, self.overlap, info, tm)
            log(f"[bench]   {batch.config} {['hybrid', 'all_load', 'all_recompute'][info.kind]}: predicted comp "
                f"{info.t_comp / 1e9:.1f} io {info.t_io / 1e9:.1f} ttft {info.ttft / 1e9:.1f} (hybrid "
                f"{info.ttft_hybrid / 1e9:.1f}, all-load {info.ttft_all_load / 1e9:.1f}) ms; measured comp "
                f"{tm['compute_ms']:.1f} (waited {tm['compute_wait_ms']:.1f}) copy {tm['copy_ms']:.1f} ttft {tm['total_ms']:.1f} ms; recomputed "
                f"{sum(s[1] for s in splits if s[2] > 0)} tokens; overlap now {self.overlap.comp_permille}/"
                f"{self.overlap.io_permille}")
        return splits, info, tm

    def run(self, batch, reqs, plan, steps, warmup, stage=None, profile=True):
        """warmup + `steps` timed steps of one configuration; returns the result dict."""
        sess, torch, np_ = self.sess, self.torch, __import__("numpy")
        gemm_kernels = ["gemm_qkv", "gemm_oproj", "gemm_gate_up", "gemm_down", "gemm_lm_head"]
        prof_kernels = gemm_kernels + ["attention", "rope_write", "rmsnorm", "h2d_copy", "page_scatter"]
        # HIP events bracket every launch of a profiled kernel class and cost stream time, so the
        # warm-up and the timed steps time the dominant kernel only (the roofline needs its live
        # average over the timed region); the per-kernel table comes from one extra step afterwards
        sess.ctx.profile(["gemm_gate_up"] if profile else [])
        for _ in range(warmup):
            self.step(batch, reqs, plan, stage)
        sess.ctx.profile_read(reset=True)
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        tms = []
        for _ in range(steps):
            splits, info, tm = self.step(batch, reqs, plan, stage)
            tms.append(tm)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_begin
        prof = sess.ctx.profile_read(reset=True)
        kernels = {}
        all_gemm_ms = all_gemm_fl = 0.0
        if profile:
            sess.ctx.profile(prof_kernels)
            self.step(batch, reqs, plan, stage)
            prof_all = sess.ctx.profile_read(reset=True)
            for k in prof_kernels:
                p = prof_all[k]
                if not p["launches"]:
                    continue
                by_bytes = k in ("h2d_copy", "page_scatter", "rope_write", "rmsnorm")
                kernels[k] = {"launches": p["launches"], "total_ms_per_step": p["total_ms"],
                              ("GB/s" if by_bytes else "TFLOP/s"): p["work"] / (p["total_ms"] * 1e-3) / (1e9 if by_bytes else 1e12)}
            all_gemm_ms = sum(prof_all[k]["total_ms"] for k in gemm_kernels)
            all_gemm_fl = sum(prof_all[k]["work"] for k in gemm_kernels)
        sess.ctx.profile([])
        mean = lambda k: float(np_.mean([t[k] for t in tms]))
        sum_ctx = sum(batch.n_ctx)
        peak = PEAK_BF16_TFLOPS if self.shape.dtype == "bf16" else PEAK_FP32_TFLOPS
        ttft_ms, compute_ms, copy_ms = mean("total_ms"), mean("compute_ms"), mean("copy_ms")
        rec_fl, suf_fl, loaded = tms[-1]["recompute_flops"], tms[-1]["suffix_flops"], tms[-1]["loaded_bytes"]
        piped = not (self.args.sequential_join or plan == "dynamic")
        comp_tflops = ((rec_fl + suf_fl) / (ttft_ms * 1e-3) if piped else rec_fl / max(compute_ms, 1e-9) / 1e-3) / 1e12
        copy_gbs = loaded / (copy_ms * 1e-3) / 1e9 if copy_ms > 0 and loaded else 0.0
        out = {
            "workload": f"{batch.config}: {self.shape.name} shape, B={len(batch.n_ctx)}, sum n_ctx={sum_ctx}, "
                        f"n_new={sum(batch.n_new)}, plan={plan}, chunk C={batch.chunk_tokens}, "
                        + (f"stage layers [{stage[0]},{stage[1]}) of {self.shape.n_layers} from boundary activations, "
                           if stage else "") + f"{'pipelined' if piped else 'sequential'} join",
            "steps": steps, "warmup": warmup, "ms_per_step": wall / steps * 1e3,
            "restored_tokens_per_s": sum_ctx * steps / wall,
            "ttft_ms": ttft_ms, "restore_ms": mean("restore_ms"), "compute_stream_ms": compute_ms,
            "copy_stream_ms": copy_ms, "suffix_ms": mean("suffix_ms"),
            "plan_kind": None if not isinstance(info, self.cf.cf_batch_plan) else
                         ["hybrid", "all_load", "all_recompute"][info.kind],
            "predicted_ttft_ms": None if not isinstance(info, self.cf.cf_batch_plan) else
                                 {"plan": info.ttft / 1e9, "hybrid": info.ttft_hybrid / 1e9,
                                  "all_load": info.ttft_all_load / 1e9, "all_recompute": info.ttft_all_recompute / 1e9},
            "recompute": {"tokens": int(sum(s[1] for s in splits if s[2] > 0)),
                          "cells": int(tms[-1]["recomputed_cells"]),
                          "compute_stream_tflops": comp_tflops, "frac_of_mfma_peak": comp_tflops / peak,
                          "all_gemm_tflops": all_gemm_fl / (all_gemm_ms * 1e-3) / 1e12 if all_gemm_ms else None},
            "copy": {"bytes": int(loaded), "GB/s": copy_gbs, "h2d_measured_GB/s": self.h2d_gbs,
                     "frac_of_measured_h2d": copy_gbs / self.h2d_gbs if self.h2d_gbs else 0.0},
            "splits": [list(x) for x in splits] if len(splits) <= 8 else
                      {"token_wise_k": sorted(x[1] for x in splits if x[0] == 0),
                       "layer_wise_cut": sorted(x[2] for x in splits if x[0] == 1)},
            "dynamic": info["stats"] if isinstance(info, dict) else None,
            "kernels": kernels,
        }
        return out, prof["gemm_gate_up"]


def roofline_of(dom, config, is_bf16):
    """`roofline` object of the dominant kernel (the gate/up GEMM) from its live event timings."""
    if not dom["launches"]:
        return None
    peak = PEAK_BF16_TFLOPS if is_bf16 else PEAK_FP32_TFLOPS
    avg_ms = dom["total_ms"] / dom["launches"]
    ach = dom["work"] / dom["launches"] / (avg_ms * 1e-3) / 1e12
    traffic = None          # HBM-side bytes per launch from rocprofv3 --pmc runs, stored under profiles/
    tpath = os.path.join(ROOT, "profiles", "traffic.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            f = line.split()
            if len(f) == 4 and f[0] == "8b:gemm_gate_up" and is_bf16:
                traffic = {"source": "stored: profiles/traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of "
                                     "`bench.py --probe gemm`, scaled by a 1 GiB copy), not measured in this run",
                           "rows_per_launch": int(f[1]), "fetch_bytes": float(f[2]), "write_bytes": float(f[3]),
                           "bytes": float(f[2]) + float(f[3])}
    return {"bound": "mfma" if is_bf16 else "alu", "kernel": "gemm_gate_up (MFMA GEMM, SiLU*mul epilogue)",
            "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
            "traffic": None if traffic is None else traffic["bytes"], "traffic_detail": traffic,
            "launches": dom["launches"], "avg_launch_ms": avg_ms, "flops_per_launch": dom["work"] / dom["launches"]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", default="cfg4",
                    help="cfg1 .. cfg5, or sweep:<B>:<n>[:<mode>] = B requests of n tokens on the 8B shape "
                         "(mode 0 token-wise, 1 layer-wise, default by L_delta)")
    ap.add_argument("--plan", default="planner",
                    help="planner | dynamic (claims at run time, no precomputed split) | per_request | "
                         "all_recompute | all_load | cut=<L> (layer cut for every request)")
    ap.add_argument("--step-cap-ms", type=float, default=0.0,
                    help="--plan dynamic: a compute step stops taking units at this predicted duration (0: no cap)")
    ap.add_argument("--units-per-request", type=int, default=0,
                    help="--plan dynamic: most consecutive chunks of one request in a step (0: no limit)")
    ap.add_argument("--model-skew", default="",
                    help="--plan dynamic: c:io -- multiply the calibrated compute / load costs by these factors "
                         "before the run-time scheduler sees them (a wrong cost model)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the short runs of the other configurations and plans after the timed region")
    ap.add_argument("--chunk-rows", type=int, default=0)
    ap.add_argument("--load-path", choices=["auto", "staged", "direct"], default="auto",
                    help="direct: load kernel reading pinned host memory; staged: DMA + scatter")
    ap.add_argument("--load-workgroups", type=int, default=0,
                    help="resident workgroups of the direct load kernel (0: library default)")
    ap.add_argument("--stage", default="",
                    help="b:e -- restore only layers [b, e), one pipeline stage's share, recomputing from "
                         "boundary activations captured at layer b (no logits; value = the stage's tokens/s)")
    ap.add_argument("--link-gbps", type=float, default=0.0,
                    help="pace the copy stream to this many Gbit/s (emulates a slower storage tier; 0: off)")
    ap.add_argument("--sequential-join", action="store_true",
                    help="restore, wait for both streams, then prefill the new tokens (default: pipelined join)")
    ap.add_argument("--probe", choices=["gemm", "attention"], default=None,
                    help="run one kernel class alone (for rocprofv3 counter runs) instead of the benchmark: "
                         "gemm = the layer GEMMs of the 8B shape at --rows rows; attention = one request of "
                         "--tokens tokens")
    ap.add_argument("--rows", type=int, default=10752)
    ap.add_argument("--tokens", type=int, default=16384)
    ap.add_argument("--reps", type=int, default=3)
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
            f"--gpus {args.gpus} is not supported.")
        sys.exit(2)
    if args.probe:
        return probe_gemm(args) if args.probe == "gemm" else probe_attention(args)

    from workloads import make_batch
    batch = make_batch(args.config)
    shape = batch.shape
    stage = tuple(int(x) for x in args.stage.split(":")) if args.stage else None
    extras = not args.no_extras and not stage and args.config == "cfg4" and args.plan == "planner"
    same_model = [make_batch(c) for c in ("cfg2", "cfg3")] if extras else []
    bench = Bench(args, [batch] + same_model)
    reqs, tm_full, offload_gbs = bench.prepare(batch, stage)
    bench.calibrate(reqs)
    if stage:
        bench.sess.ctx.set_stage(*stage)
    res, dom = bench.run(batch, reqs, args.plan, args.steps, args.warmup, stage)
    peak = PEAK_BF16_TFLOPS if shape.dtype == "bf16" else PEAK_FP32_TFLOPS
    out = {
        "metric": "restored tokens/s", "value": res["restored_tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": res["workload"], "n_ctx": batch.n_ctx, "splits": res["splits"]},
    }
    out.update({k: res[k] for k in ("ttft_ms", "restore_ms", "compute_stream_ms", "copy_stream_ms", "suffix_ms",
                                    "plan_kind", "predicted_ttft_ms", "recompute", "copy", "dynamic", "kernels")})
    out["copy"]["offload_d2h_GB/s"] = offload_gbs
    out["copy"]["link_throttle_GB/s"] = args.link_gbps / 8.0
    out["all_recompute_pass"] = {"ms": tm_full["compute_ms"],
                                 "tflops": tm_full["recompute_flops"] / tm_full["compute_ms"] / 1e9,
                                 "frac_of_mfma_peak": tm_full["recompute_flops"] / tm_full["compute_ms"] / 1e9 / peak}
    out["planner"] = {"cost_model_ps": bench.cost0, "l_delta": bench.l_delta,
                      "cost_model_after_feedback_ps": bench.cost_dict()}
    out["roofline"] = roofline_of(dom, args.config, shape.dtype == "bf16")

    if extras:
        short = lambda r: {k: r[k] for k in ("workload", "steps", "ms_per_step", "restored_tokens_per_s", "ttft_ms",
                                             "compute_stream_ms", "copy_stream_ms", "plan_kind", "recompute", "copy",
                                             "splits")}
        configs = {}
        # configuration 4 under the two extremes (the recompute-only and load-only baselines)
        for plan in ("all_load", "all_recompute"):
            r, _ = bench.run(batch, reqs, plan, 1, 1 if plan == "all_load" else 0, profile=False)
            configs[f"cfg4:{plan}"] = short(r)
        bench.release(batch, reqs)
        # configurations 2 and 3 on the same model
        for b2 in same_model:
            reqs2, _, _ = bench.prepare(b2)
            r, d2 = bench.run(b2, reqs2, "planner", 3, 4, profile=False)
            configs[b2.config] = short(r)
            if b2.config == "cfg3":      # layer-cut sweep of the 131072-token request
                sweep = {}
                for cut in (0, 4, 8, 16, 32):
                    rc, _ = bench.run(b2, reqs2, f"cut={cut}", 1, 0, profile=False)
                    sweep[str(cut)] = {"ttft_ms": rc["ttft_ms"], "restored_tokens_per_s": rc["restored_tokens_per_s"]}
                configs["cfg3"]["layer_cut_sweep"] = sweep
            bench.release(b2, reqs2)
        bench.sess.close()
        del bench
        import torch
        torch.cuda.empty_cache()
        # configuration 5: one tensor-parallel shard of the 70B shape, its own model
        b5 = make_batch("cfg5")
        bench5 = Bench(args, [b5])
        reqs5, _, _ = bench5.prepare(b5)
        bench5.calibrate(reqs5)
        r, _ = bench5.run(b5, reqs5, "planner", 3, 4, profile=False)
        configs["cfg5"] = short(r)
        r, _ = bench5.run(b5, reqs5, "all_load", 1, 1, profile=False)
        configs["cfg5:all_load"] = short(r)
        bench5.sess.close()
        out["configs"] = configs
    else:
        bench.sess.close()
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on bounded samples ...")
        out["cpu_baseline"] = cpu_baseline(batch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
