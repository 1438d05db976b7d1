#!/usr/bin/env python3
"""Benchmark of batched hybrid KV-cache restoration on one MI355X.

One step = one pass of the whole hot path over one batch: plan the splits
(host scheduler over the calibrated cost model), recompute ‖ load+scatter,
join, prefill the new-turn tokens over the restored pages, first-token logits.
Inputs are synthetic (seeded token ids, random-init weights of the named
shape) and already resident (weights in HBM, host KV in pinned memory) when
the timed region starts.

    python bench.py --gpus 1 --steps K --warmup W [--config cfg2] [--plan planner]

Prints ONE JSON line.
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


def cpu_baseline(batch, n_tok=4096, n_layers=6):
    """Time the CPU oracle (as it stands) on a bounded slice of the workload."""
    import numpy as np
    from oracle import transformer as T
    from workloads import WeightSource
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    shape = batch.shape
    ws = WeightSource(shape, batch.weight_seed, cache=True)
    n_tok = min(n_tok, batch.n_ctx[0])
    n_layers = min(n_layers, shape.n_layers)
    ws.f32("embed")
    for l in range(n_layers):
        ws.layer_f32(l)
    t0 = time.perf_counter()
    T.prefill(shape, ws, batch.ctx_tokens[0][:n_tok], n_layers=n_layers, dtype=np.float32)
    dt = time.perf_counter() - t0
    tok_layers_per_s = n_tok * n_layers / dt
    return {
        "value": tok_layers_per_s / shape.n_layers, "unit": "restored tokens/s",
        "cores": int(cores), "kind": "oracle",
        "sample": (f"oracle float32 recompute of the first {n_tok} tokens of request 0 through "
                   f"{n_layers} of {shape.n_layers} layers ({dt:.2f} s), scaled by layer count; "
                   "loading is a memcpy and is not part of the sample"),
        "token_layers_per_s": tok_layers_per_s,
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", default="cfg2",
                    help="cfg1 .. cfg5, or sweep:<B>:<n>[:<mode>] = B requests of n tokens on the 8B shape "
                         "(mode 0 token-wise, 1 layer-wise, default by L_delta)")
    ap.add_argument("--plan", default="planner",
                    help="planner | dynamic (claims at run time, no precomputed split) | per_request | "
                         "all_recompute | all_load | cut=<L> (layer cut for every request)")
    ap.add_argument("--step-cap-ms", type=float, default=0.0, help="dynamic: cap of a compute step (0: library default)")
    ap.add_argument("--claim-order", choices=["cheapest", "shortest"], default="cheapest",
                    help="dynamic: order of the compute engine's candidates")
    ap.add_argument("--model-skew", default="1:1",
                    help="c:io -- multiply the calibrated compute / load costs by these before planning "
                         "(a deliberately wrong cost model, to see what each scheduler makes of it)")
    ap.add_argument("--no-feedback", action="store_true",
                    help="planner: do not correct the cost model from measured steps")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink context lengths (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--chunk-rows", type=int, default=0)
    ap.add_argument("--load-path", choices=["auto", "staged", "direct"], default="auto",
                    help="direct: load kernel reading pinned host memory; staged: DMA + scatter")
    ap.add_argument("--load-workgroups", type=int, default=0,
                    help="resident workgroups of the direct load kernel (0: library default)")
    ap.add_argument("--no-guard", action="store_true",
                    help="planner mode: never fall back to all-load (skip the probe step)")
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

    import numpy as np
    import torch
    import paper_2604_25080_amd as cf
    from paper_2604_25080_amd.runtime import Session
    from workloads import WeightSource, make_batch

    batch = make_batch(args.config, scale=args.scale)
    shape = batch.shape
    B = len(batch.n_ctx)
    L = shape.n_layers
    sum_ctx, sum_new = sum(batch.n_ctx), sum(batch.n_new)
    log(f"[bench] {args.config}: {shape.name} B={B} sum n_ctx={sum_ctx} sum n_new={sum_new}")

    t0 = time.perf_counter()
    calib_tokens = 8192
    pages = sum(-(-(n + m) // 16) for n, m in zip(batch.n_ctx, batch.n_new)) + calib_tokens // 16 + 64
    sess = Session(shape, WeightSource(shape, batch.weight_seed), max_batch=max(B, 8),
                   max_tokens=max(sum_ctx + sum_new, calib_tokens),
                   max_positions=max(max(n + m for n, m in zip(batch.n_ctx, batch.n_new)), calib_tokens) + 16,
                   n_pages=pages, chunk_rows=args.chunk_rows, gen_threads=16)
    log(f"[bench] weights + pool + workspace ready in {time.perf_counter() - t0:.1f} s")
    sess.ctx.set_pipelined_join(not args.sequential_join)
    sess.ctx.set_load_path({"auto": 0, "staged": 1, "direct": 2}[args.load_path], args.load_workgroups)

    # ---- manufacture the host KV (not timed): full prefill on the GPU, then offload
    t0 = time.perf_counter()
    reqs = []
    for i in range(B):
        sess.cache.alloc(1 + i, batch.n_ctx[i] + batch.n_new[i])
        reqs.append(dict(req_id=1 + i, ctx_tokens=batch.ctx_tokens[i], new_tokens=batch.new_tokens[i],
                         host_kv=None))
    stage = tuple(int(x) for x in args.stage.split(":")) if args.stage else None
    if stage:
        cap = torch.empty(sum_ctx, shape.d_model, dtype=torch.float32, device="cuda")
        sess.ctx.capture_boundary(stage[0], cap.data_ptr(), sum_ctx)
    _, tm_full = sess.restore(reqs, [(0, n, L) for n in batch.n_ctx], want_logits=False)
    if stage:      # packed order of an all-recompute pass with equal cuts = call order
        off = 0
        for i in range(B):
            bh = torch.empty(batch.n_ctx[i], shape.d_model, dtype=torch.float32, pin_memory=True)
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
    log(f"[bench] host KV manufactured in {time.perf_counter() - t0:.1f} s "
        f"(offload {offload_gbs:.1f} GB/s, "
        f"all-recompute pass: {tm_full['compute_ms']:.1f} ms, "
        f"{tm_full['recompute_flops'] / tm_full['compute_ms'] / 1e9:.0f} TFLOP/s)")

    sess.ctx.set_link_throttle(args.link_gbps / 8.0)

    # ---- measured rooflines of the load path and the cost model
    big = max(reqs, key=lambda r: r["host_kv"].numel())["host_kv"]
    h2d_bytes = min(big.numel(), 1 << 30)
    dev_scratch = torch.empty(h2d_bytes, dtype=torch.uint8, device="cuda")
    h2d_gbs = sess.ctx.measure_h2d(big.data_ptr(), dev_scratch.data_ptr(), h2d_bytes, reps=4)
    del dev_scratch
    need = sess.host_kv_bytes(calib_tokens)
    scratch = big if big.numel() >= need else sess.pinned(need)
    cm = sess.ctx.calibrate(sess.cache, scratch.data_ptr(), scratch.numel())
    cost = dict(f_c=cm.f_c, alpha=cm.alpha, beta=cm.beta, f_io=cm.f_io, gamma=cm.gamma,
                s_c=cm.s_c, s_io=cm.s_io)
    if stage:
        # the stage's share: plan and restore layers [b, e) only; the compute start-up that
        # calibration measured is per layer of the pass
        sess.ctx.set_stage(*stage)
        cm.s_c = cm.s_c * (stage[1] - stage[0]) // L
        L = stage[1] - stage[0]
    # the executor stops a request's last recomputed layer after its K/V write: price it so
    qkv_fl = 2.0 * shape.d_model * shape.qkv_cols
    lin_fl = qkv_fl + 2.0 * shape.n_q_heads * shape.head_dim * shape.d_model + 6.0 * shape.d_model * shape.d_ffn
    opts = cf.plan_opts(batch.chunk_tokens, 0, L, shape.kv_bytes_per_token_layer, batch.forced_mode,
                        kv_only_permille=int(round(1000 * qkv_fl / lin_fl)))
    l_delta = cf.derive_l_delta(cm, opts, 32768)
    opts.l_delta = l_delta
    log(f"[bench] H2D {h2d_gbs:.1f} GB/s; cost model {cost}; L_delta {l_delta}")
    skew_c, skew_io = (float(x) for x in args.model_skew.split(":"))
    if (skew_c, skew_io) != (1.0, 1.0):
        for f in ("f_c", "alpha", "beta", "s_c"):
            setattr(cm, f, int(getattr(cm, f) * skew_c))
        for f in ("f_io", "gamma", "s_io"):
            setattr(cm, f, int(getattr(cm, f) * skew_io))

    def plan_model():
        """The cost table the planner sees: with the pipelined join the new-turn prefill shares
        the compute stream with the recompute, so its cost starts the compute clock."""
        if stage or args.sequential_join:
            return cm
        m2 = cf.cost_model(f_c=cm.f_c, alpha=cm.alpha, beta=cm.beta, f_io=cm.f_io, gamma=cm.gamma,
                           s_c=cm.s_c, s_io=cm.s_io)
        m2.s_c += cf.prefill_cost(cm, shape.n_layers, batch.n_ctx, batch.n_new)
        return m2

    # Measured guard: the two streams slow each other down, and where recompute buys little (a
    # TP shard: I/O is ~18x cheaper per token) the hybrid's small saving can be less than that
    # slow-down.  One warm-up step therefore runs the all-load extreme, and from then on the
    # hybrid is kept only while its last measured TTFT beats the extreme's.
    guard = {"all_load_ms": None, "hybrid_ms": None, "n_hybrid": 0, "all_load_steps": 0,
             "probe": args.warmup >= 4 and not args.no_guard}

    def make_plan():
        if args.plan == "planner":
            if batch.forced_splits:
                return [(0, k, c) for k, c in batch.forced_splits], None
            all_load = [(0, 0, L) for _ in batch.n_ctx]
            if guard["probe"]:
                guard["probe"] = False
                return all_load, "probe"
            # (the hybrid gets three steps of feedback before it is judged, by its best step)
            if (guard["all_load_ms"] is not None and guard["n_hybrid"] >= 3 and
                    guard["all_load_ms"] < 0.99 * guard["hybrid_ms"]):
                guard["all_load_steps"] += 1
                return all_load, None
            splits, stats, _ = cf.restore_plan(plan_model(), opts, batch.n_ctx)
            return splits, stats
        if args.plan == "per_request":
            # comparison plan: every request planned alone, as if it had both engines to itself
            # (a per-request bidirectional planner); no batch awareness
            out = []
            for n in batch.n_ctx:
                sp, _, _ = cf.restore_plan(plan_model(), opts, [n])
                out.append(sp[0])
            return out, None
        if args.plan == "all_recompute":
            return [(0, n, L) for n in batch.n_ctx], None
        if args.plan == "all_load":
            return [(0, 0, L) for n in batch.n_ctx], None
        if args.plan.startswith("cut="):
            c = int(args.plan[4:])
            return [(1, n, c) for n in batch.n_ctx], None
        raise SystemExit(f"unknown plan {args.plan}")

    gemm_kernels = ["gemm_qkv", "gemm_oproj", "gemm_gate_up", "gemm_down", "gemm_lm_head"]
    prof_kernels = gemm_kernels + ["attention", "h2d_copy", "page_scatter"]

    dyn_stats = []

    def step():
        if args.plan == "dynamic":
            # no plan: the engines claim units while the call runs; the cost model only seeds
            # the predictions (no start-ups: they are not per-unit costs)
            _, splits, tm, st = sess.restore_dynamic(reqs, cm, opts, want_logits=True,
                                                     step_cap_ps=int(args.step_cap_ms * 1e9),
                                                     order={"cheapest": 0, "shortest": 1}[args.claim_order])
            dyn_stats.append(st)
            return splits, None, tm
        splits, stats = make_plan()
        logits, tm = sess.restore(reqs, splits, want_logits=not stage)
        if stats == "probe":
            guard["all_load_ms"] = tm["total_ms"]
            return splits, None, tm
        if stats is not None:
            guard["n_hybrid"] += 1
            guard["hybrid_ms"] = min(guard["hybrid_ms"] or tm["total_ms"], tm["total_ms"])
            # closed loop: correct the cost model by what the two streams actually took (they
            # slow each other down when they overlap, which calibration in isolation cannot see)
            # The plan's t_comp is when the compute stream would finish ALL its work, the
            # new-turn prefill included.  cf_timing.compute_ms marks the end of the last
            # recomputed layer, which is the same thing for token-wise splits (cut = L) but not
            # for a low layer cut, where the new-turn rows still have the upper layers to go:
            # when the compute stream finishes well after the copy stream, its end is the
            # measurement.
            meas_comp = tm["total_ms"] if tm["total_ms"] > 1.02 * tm["copy_ms"] else tm["compute_ms"]
            if not args.no_feedback:
                cf.cost_feedback(cm, stats["t_comp"], int(meas_comp * 1e9), stats["t_io"],
                                 int(tm["copy_ms"] * 1e9))
        return splits, stats, tm

    # HIP events bracket every launch of a profiled kernel class and cost stream time, so the
    # warm-up and the timed steps time the dominant kernel only (the roofline needs its live
    # average over the timed region); the per-kernel table comes from one extra step afterwards
    sess.ctx.profile(["gemm_gate_up"])
    for _ in range(args.warmup):
        step()
    sess.ctx.profile_read(reset=True)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    tms, all_splits = [], []
    for _ in range(args.steps):
        splits, stats, tm = step()
        tms.append(tm)
        all_splits.append(splits)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_begin
    prof = sess.ctx.profile_read(reset=True)
    sess.ctx.profile(prof_kernels)
    step()
    prof_all = sess.ctx.profile_read(reset=True)
    sess.ctx.profile([])

    ms_per_step = wall / args.steps * 1e3
    mean = lambda k: float(np.mean([t[k] for t in tms]))
    restore_ms, ttft_ms = mean("restore_ms"), mean("total_ms")
    compute_ms, copy_ms, suffix_ms = mean("compute_ms"), mean("copy_ms"), mean("suffix_ms")
    rec_flops, suf_flops = tms[-1]["recompute_flops"], tms[-1]["suffix_flops"]
    loaded_bytes = tms[-1]["loaded_bytes"]

    # dominant kernel of the recompute path: the gate/up GEMM (SiLU*mul epilogue)
    dom = prof["gemm_gate_up"]
    is_bf16 = shape.dtype == "bf16"
    peak = PEAK_BF16_TFLOPS if is_bf16 else PEAK_FP32_TFLOPS
    roofline = None
    if dom["launches"]:
        avg_ms = dom["total_ms"] / dom["launches"]
        ach = dom["work"] / dom["launches"] / (avg_ms * 1e-3) / 1e12
        traffic = None          # HBM bytes per launch from rocprofv3 --pmc runs (profiles/)
        tpath = os.path.join(ROOT, "profiles", "traffic.txt")
        if os.path.exists(tpath):
            for line in open(tpath):
                f = line.split()
                if len(f) == 4 and f[0] == f"{args.config}:gemm_gate_up":
                    traffic = {"rows_per_launch": int(f[1]), "fetch_bytes": float(f[2]),
                               "write_bytes": float(f[3]), "bytes": float(f[2]) + float(f[3])}
        roofline = {"bound": "mfma" if is_bf16 else "alu", "kernel": "gemm_gate_up (MFMA GEMM, SiLU*mul epilogue)",
                    "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
                    # HBM-side bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size)
                    "traffic": None if traffic is None else traffic["bytes"], "traffic_detail": traffic,
                    "launches": dom["launches"], "avg_launch_ms": avg_ms,
                    "flops_per_launch": dom["work"] / dom["launches"]}
    kernels = {}      # from the one extra step after the timed region, every class profiled
    for k in prof_kernels:
        p = prof_all[k]
        if not p["launches"]:
            continue
        rate = p["work"] / (p["total_ms"] * 1e-3)
        kernels[k] = {"launches": p["launches"], "total_ms_per_step": p["total_ms"],
                      ("GB/s" if k in ("h2d_copy", "page_scatter") else "TFLOP/s"):
                          rate / (1e9 if k in ("h2d_copy", "page_scatter") else 1e12)}
    all_gemm_ms = sum(prof_all[k]["total_ms"] for k in gemm_kernels)
    all_gemm_fl = sum(prof_all[k]["work"] for k in gemm_kernels)
    copy_gbs = loaded_bytes / (copy_ms * 1e-3) / 1e9 if copy_ms > 0 and loaded_bytes else 0.0

    seq_join = args.sequential_join or args.plan == "dynamic"   # run-time scheduling joins before the new turn
    out = {
        "metric": "restored tokens/s", "value": sum_ctx * args.steps / wall, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"{args.config}: {shape.name} shape, B={B}, sum n_ctx={sum_ctx}, "
                               f"n_new={sum_new}, plan={args.plan}, chunk C={batch.chunk_tokens}, "
                               + (f"stage layers [{stage[0]},{stage[1]}) of {shape.n_layers} from boundary activations, "
                                  if stage else "") +
                               
                               f"{'sequential' if seq_join else 'pipelined'} join",
                   "n_ctx": batch.n_ctx, "splits": [list(s) for s in splits]},
        "ttft_ms": ttft_ms, "restore_ms": restore_ms, "compute_stream_ms": compute_ms,
        "copy_stream_ms": copy_ms, "suffix_ms": suffix_ms,
        "restore_tokens_per_s": sum_ctx / (restore_ms * 1e-3),
        # the compute stream runs the recompute AND (pipelined join) the new-turn prefill
        "recompute": {"tokens": int(sum(s[1] for s in splits if s[2] > 0)),
                      "compute_stream_tflops": (rec_flops + suf_flops) / (max(compute_ms, ttft_ms - 0.0) * 1e-3) / 1e12
                      if not seq_join else rec_flops / (compute_ms * 1e-3) / 1e12,
                      "frac_of_mfma_peak": ((rec_flops + suf_flops) / (ttft_ms * 1e-3) / 1e12 / peak)
                      if not seq_join else rec_flops / (compute_ms * 1e-3) / 1e12 / peak,
                      "all_gemm_tflops": all_gemm_fl / (all_gemm_ms * 1e-3) / 1e12 if all_gemm_ms else 0.0},
        "copy": {"bytes": int(loaded_bytes), "GB/s": copy_gbs, "h2d_measured_GB/s": h2d_gbs,
                 "frac_of_measured_h2d": copy_gbs / h2d_gbs if h2d_gbs else 0.0,
                 "offload_d2h_GB/s": offload_gbs, "link_throttle_GB/s": args.link_gbps / 8.0},
        "all_recompute_pass": {"ms": tm_full["compute_ms"],
                               "tflops": tm_full["recompute_flops"] / tm_full["compute_ms"] / 1e9,
                               "frac_of_mfma_peak": tm_full["recompute_flops"] / tm_full["compute_ms"] / 1e9 / peak},
        "planner": {"cost_model_ps": cost, "l_delta": l_delta, "all_load_guard_steps": guard["all_load_steps"],
                    "cost_model_after_feedback_ps": dict(f_c=cm.f_c, alpha=cm.alpha, beta=cm.beta, f_io=cm.f_io,
                                                         gamma=cm.gamma, s_c=cm.s_c, s_io=cm.s_io),
                    "predicted_ms": None if stats is None else stats["makespan"] / 1e9},
        "dynamic": None if not dyn_stats else dict(
            dyn_stats[-1],
            # what the static planner would have fixed in advance from the same cost model
            static_plan_splits=[list(x) for x in cf.restore_plan(plan_model(), opts, batch.n_ctx)[0]],
            recomputed_tokens_per_step=[int(sum(x[1] for x in sp if x[2] > 0)) for sp in all_splits]),
        "kernels": kernels,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a bounded slice ...")
        out["cpu_baseline"] = cpu_baseline(batch)
    sess.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
