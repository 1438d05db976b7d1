"""GPU parity at full size for configurations 3, 4 and 5, in the launch
configuration bench.py times (planner splits, pipelined join, direct loads),
with checks the CPU oracle can afford at 10^5 tokens:

 1. layer 0, every cell of one whole request: K/V of layer 0 need no
    attention, so the oracle computes them for all positions (embedding,
    RMSNorm, K/V projection, rotary turn) -- pins token gather, rotary angles up
    to position 131071 and the page placement of every token;
 2. layer 1, sampled positions (first, last, middle, page edges): the oracle
    runs layer 0 for those rows only -- attention of one query over ALL earlier
    keys of its own layer-0 cache -- and projects the result to layer-1 K/V.
    Pins the causal mask, the online-softmax normalisation over up to 131072
    keys, GQA mapping and the MLP at full context length;
 3. (configuration 5, the shape no other test covers) prefix exactness through
    all 80 layers, held to the bf16 noise floor as for configuration 2;
 4. the planner's hybrid restore reproduces the all-recompute cache byte for
    byte (recomputed cells do not depend on the split, loaded cells are copies),
    and the first-token logits match the oracle's head on the final hidden rows.

The 8B-shaped configurations 3 and 4 share one session (same weights); the
70B tensor-parallel shard of configuration 5 gets its own.
"""
import numpy as np
import pytest
import torch

from oracle import transformer as T
from oracle.pagetable import PageTable
from workloads import WeightSource, hand_cost_model, make_batch

from gpu_util import decode_pages, kv_tolerance_ok, teacher_forced_layer_checks, teacher_forced_samples

pytestmark = pytest.mark.gpu

_sessions = {}


def session_for(shape, weight_seed, max_tokens, max_positions, n_pages, max_batch):
    from paper_2604_25080_amd.runtime import Session
    key = shape.name
    if key not in _sessions:
        sess = Session(shape, WeightSource(shape, weight_seed), max_batch=max_batch, max_tokens=max_tokens,
                       max_positions=max_positions, n_pages=n_pages, gen_threads=16)
        _sessions[key] = (sess, WeightSource(shape, weight_seed, cache=True))
    return _sessions[key]


@pytest.fixture(scope="module", autouse=True)
def close_sessions():
    yield
    for sess, _ in _sessions.values():
        sess.close()
    _sessions.clear()


def build(config):
    """Allocate the batch, prefill it on the GPU (all-recompute), offload to pinned host blocks."""
    b = make_batch(config)
    shape = b.shape
    if shape.name == "8b":
        # capacity for the larger of configurations 3 and 4
        caps = [make_batch(c) for c in ("cfg3", "cfg4")]
    else:
        caps = [b]
    max_tokens = max(sum(c.n_ctx) + sum(c.n_new) for c in caps)
    max_pos = max(max(n + m for n, m in zip(c.n_ctx, c.n_new)) for c in caps) + 16
    pages = max(sum(-(-(n + m) // 16) for n, m in zip(c.n_ctx, c.n_new)) for c in caps) + 64
    sess, ws = session_for(shape, caps[0].weight_seed, max_tokens, max_pos, pages, max(len(c.n_ctx) for c in caps))
    B = len(b.n_ctx)
    opt = PageTable(pages)
    reqs = []
    for i in range(B):
        sess.cache.alloc(1 + i, b.n_ctx[i] + b.n_new[i])
        assert sess.cache.page_table(1 + i) == opt.alloc(1 + i, b.n_ctx[i] + b.n_new[i])
        reqs.append(dict(req_id=1 + i, ctx_tokens=b.ctx_tokens[i], new_tokens=b.new_tokens[i], host_kv=None))
    # hidden rows entering every layer, sampled in the longest, the shortest and the first request
    picked = sorted({0, int(np.argmax(b.n_ctx)), int(np.argmin(b.n_ctx))})
    rows, rows_req, rows_pos = teacher_forced_samples(b.n_ctx, picked)
    if len(rows) < 64:       # a single request: add evenly spaced positions
        more = np.setdiff1d(np.linspace(0, b.n_ctx[0] - 1, 48).astype(np.int64), rows_pos)
        rows = np.concatenate([rows, more.astype(np.int32)])
        rows_req, rows_pos = np.concatenate([rows_req, np.zeros(len(more), dtype=np.int64)]), np.concatenate([rows_pos, more])
    hid = torch.full((2 * shape.n_layers + 1, len(rows), shape.d_model), float("nan"), dtype=torch.float32, device="cuda")
    sess.ctx.capture_rows(rows, hid.data_ptr())
    sess.restore(reqs, [(0, n, shape.n_layers) for n in b.n_ctx], want_logits=False)
    sess.teacher = (hid.cpu().numpy(), rows_req, rows_pos)
    del hid
    for i in range(B):
        reqs[i]["host_kv"] = sess.offload(1 + i, b.n_ctx[i])
    return b, sess, ws, reqs


def check_teacher_forced(b, sess, ws, reqs, out_layers):
    """K/V cells of the sampled rows at EVERY layer and the layer output rows at `out_layers`,
    element by element against the unrounded oracle fed with the GPU's own hidden rows."""
    hid, rows_req, rows_pos = sess.teacher
    assert len(rows_req) >= 64
    return teacher_forced_layer_checks(b.shape, ws, sess, b.n_ctx, [r["host_kv"] for r in reqs], hid, rows_req,
                                       rows_pos, out_layers=set(out_layers), label=b.config)


def release(b, sess):
    for i in range(len(b.n_ctx)):
        sess.cache.free(1 + i)


def host_layer(sess, b, reqs, i, layer):
    """(K, V) float32 [n, Hkv, hd] of one layer of request i from its host block."""
    n = b.n_ctx[i]
    raw = reqs[i]["host_kv"].numpy()[:sess.host_kv_bytes(n)].reshape(b.shape.n_layers, -1, sess.page_bytes)
    k, v = decode_pages(b.shape, raw[layer:layer + 1], n)
    return k[0], v[0]


def oracle_layer0_kv(shape, ws, tokens, chunk=8192, act="exact"):
    """Layer-0 K/V of every position (no attention needed), float32.  act="bf16" rounds where a
    bf16 model stores (the normalised row, V, K after the rotary turn), as the oracle's
    bf16-storage forward does."""
    st = T.round_bf16 if act == "bf16" else (lambda x: x)
    lw, gain = ws.layer_f32(0), ws.norm_gain()
    nq, nk = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    wkv = lw["wqkv"][nq:].astype(np.float32)
    ks, vs = [], []
    for a in range(0, len(tokens), chunk):
        t = tokens[a:a + chunk]
        x = st(T.rmsnorm(T.embed(ws, t, np.float32), gain, shape.rms_eps, np.float32))
        kv = x @ wkv.T
        pos = np.arange(a, a + len(t))
        ks.append(st(T.rope(kv[:, :nk].reshape(len(t), shape.n_kv_heads, shape.head_dim), pos, shape.rope_base,
                            np.float32)))
        vs.append(st(kv[:, nk:].reshape(len(t), shape.n_kv_heads, shape.head_dim)))
    return np.concatenate(ks), np.concatenate(vs)


def layer1_noise_floor(shape, ws, tokens):
    """RMS and max distance of the oracle's own bf16-storage forward to its unrounded forward on
    layer-1 K/V cells (what rounding where a bf16 model stores costs, on the CPU alone)."""
    st, _ = T.prefill(shape, ws, tokens[:64], n_layers=2, dtype=np.float32, act="bf16")
    ex, _ = T.prefill(shape, ws, tokens[:64], n_layers=2, dtype=np.float32)
    e = np.concatenate([(st.k[1] - ex.k[1]).ravel(), (st.v[1] - ex.v[1]).ravel()]).astype(np.float64)
    return float(np.sqrt(np.mean(e ** 2))), float(np.abs(e).max())


def check_layers_0_and_1(b, sess, ws, reqs, i):
    shape, n = b.shape, b.n_ctx[i]
    tokens = b.ctx_tokens[i]
    k0, v0 = oracle_layer0_kv(shape, ws, tokens)
    gk, gv = host_layer(sess, b, reqs, i, 0)
    ks, vs = None, None
    for got, ref, nm in ((gk, k0, "K"), (gv, v0, "V")):
        ok, worst, _ = kv_tolerance_ok(shape, got, ref.astype(np.float64))
        if not ok:
            # width 8192: the rounding of the stored tensors alone passes 2e-2 in the tail of 4M
            # cells (V cells have std 1.8, so an ulp is 1.6e-2); hold the GPU to that noise floor
            if ks is None:
                ks, vs = oracle_layer0_kv(shape, ws, tokens, act="bf16")
            fl = (ks if nm == "K" else vs).astype(np.float64) - ref
            e = got.astype(np.float64) - ref
            print(f"{b.config} request {i} layer 0 {nm}: max abs err {worst:.4f} > 2e-2; bf16 noise floor "
                  f"max {np.abs(fl).max():.4f} rms {np.sqrt(np.mean(fl ** 2)):.5f}; gpu rms {np.sqrt(np.mean(e ** 2)):.5f}")
            assert shape.d_model > 4096, f"{b.config} request {i} layer 0 {nm}: max abs err {worst}"
            assert np.abs(e).max() <= 1.6 * np.abs(fl).max() and np.sqrt(np.mean(e ** 2)) <= 1.3 * np.sqrt(np.mean(fl ** 2)), \
                f"{b.config} request {i} layer 0 {nm}: beyond the bf16 noise floor"
    pos = np.unique(np.array([0, 1, 15, 16, 17, n // 3, n // 2, n - 17, n - 2, n - 1]).clip(0, n - 1))
    h0 = T.embed(ws, tokens[pos], np.float32)
    _, _, h1 = T.layer_rows_teacher_forced(shape, ws.layer_f32(0), ws.norm_gain(), h0, pos, k0, v0, np.float32)
    lw1 = ws.layer_f32(1)
    nq, nk = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    kv1 = T.rmsnorm(h1, ws.norm_gain(), shape.rms_eps, np.float32) @ lw1["wqkv"][nq:].astype(np.float32).T
    k1 = T.rope(kv1[:, :nk].reshape(len(pos), shape.n_kv_heads, shape.head_dim), pos, shape.rope_base, np.float32)
    v1 = kv1[:, nk:].reshape(len(pos), shape.n_kv_heads, shape.head_dim)
    gk1, gv1 = host_layer(sess, b, reqs, i, 1)
    floor_rms, floor_max = layer1_noise_floor(shape, ws, tokens)
    for got, ref, nm in ((gk1[pos], k1, "K"), (gv1[pos], v1, "V")):
        err = got.astype(np.float64) - ref
        rms, mx = float(np.sqrt(np.mean(err ** 2))), float(np.abs(err).max())
        print(f"{b.config} request {i} layer 1 {nm} at {len(pos)} sampled positions up to {pos[-1]}: "
              f"rms {rms:.4f} max {mx:.4f} (bf16 noise floor rms {floor_rms:.4f} max {floor_max:.4f})")
        assert rms <= 1.5 * floor_rms + 1e-4 and mx <= 2.0 * floor_max + 1e-3, \
            f"{b.config} request {i} layer 1 {nm}: rms {rms} max {mx} vs floor {floor_rms} / {floor_max}"


def check_hybrid_restore(b, sess, ws, reqs):
    import paper_2604_25080_amd as cf
    shape, L, B = b.shape, b.shape.n_layers, len(b.n_ctx)
    opts = cf.plan_opts(b.chunk_tokens, 0, L, shape.kv_bytes_per_token_layer, b.forced_mode)
    # the first hand cost table under which the plan is a real hybrid (a 131072-token context is
    # all-load under a fast link: its quadratic attention makes even one layer slower than the copy)
    for kind in ("startup", "balanced", "slow_io"):
        splits, stats, _ = cf.restore_plan(cf.cost_model(**hand_cost_model(kind)), opts, b.n_ctx)
        recomputes = any(s[1] > 0 and s[2] > 0 for s in splits)
        loads = any(s[1] < n or s[2] < L for s, n in zip(splits, b.n_ctx))
        if recomputes and loads:
            break
    assert recomputes and loads, "no hand cost table gives a hybrid plan"
    print(f"{b.config}: cost table '{kind}', splits {splits[:4]}{' ...' if len(splits) > 4 else ''}")
    sess.pool.fill_(0xFF)
    logits, tm = sess.restore(reqs, splits)
    assert tm["loaded_cells"] + tm["recomputed_cells"] == sum(b.n_ctx) * L
    for i in range(B):
        n = b.n_ctx[i]
        full = n // 16                      # pages without unused slots
        got = sess.read_pages(1 + i, n)
        ref = reqs[i]["host_kv"].numpy()[:sess.host_kv_bytes(n)].reshape(L, -1, sess.page_bytes)
        assert np.array_equal(got[:, :full], ref[:, :full]), f"{b.config} request {i}: cache differs"
        if n % 16:
            gk, gv = decode_pages(shape, got[:, full:], n - 16 * full)
            rk, rv = decode_pages(shape, ref[:, full:], n - 16 * full)
            assert np.array_equal(gk, rk) and np.array_equal(gv, rv), f"{b.config} request {i}: last page"
        del got
    hid = sess.ctx.read_final_hidden(B)
    out = logits.cpu().numpy()
    for i in sorted({0, B - 1}):
        ref = T.logits_last(shape, ws, hid[i].astype(np.float64), act="bf16")
        err = np.abs(out[i] - ref).max()
        assert err <= 2e-2, f"{b.config} request {i}: logits max abs err {err}"
    return splits


def check_run_time_scheduled_restore(b, sess, ws, reqs, l_delta):
    """cf_restore_dynamic on the full batch (token-wise above l_delta, layer-wise below, or the
    configuration's forced mode): loaded cells are the host block's bytes; recomputed cells --
    chunk by chunk or layer by layer, in steps -- are compared with what cf_restore_batch
    recomputes under the very splits that resulted: bit for bit in layer 0 (no attention feeds
    it), else to within two bf16 ulps of the cell on at least 97 % of the cells and a quarter of
    the tensor's spread everywhere -- a second net only: both calls run the same kernels on the
    same rows, but the attention of a pass splits its key ranges by how many rows the pass holds
    and where a request's rows fall in it, so the summation order, and with it the last bits of
    every later layer, depends on how the schedule packed its steps.  (Against the single-pass
    prefill that made the host block the same figures are printed, not asserted: that pass packs
    whole contexts, and 40 layers of an 8192-wide residual stream carry a last-bit difference
    in one attention row a long way.)  The element-wise statements about this path are the
    loaded cells (bytes), layer 0 (bits), the logits (oracle head on the final hidden rows) and
    the small shapes, where the oracle runs the whole batch."""
    import paper_2604_25080_amd as cf
    shape, L, B = b.shape, b.shape.n_layers, len(b.n_ctx)
    opts = cf.plan_opts(b.chunk_tokens, l_delta, L, shape.kv_bytes_per_token_layer, b.forced_mode)
    for kind in ("startup", "balanced", "slow_io"):
        cm = cf.cost_model(**hand_cost_model(kind))
        sess.pool.fill_(0xFF)
        logits, splits, tm, st = sess.restore_dynamic(reqs, cm, opts, overlap=cf.overlap_model(1000, 1000))
        if tm["recomputed_cells"] > 0 and tm["loaded_cells"] > 0:
            break
    print(f"{b.config} run-time scheduling, cost table '{kind}': {st}, splits {splits[:6]}{' ...' if B > 6 else ''}")
    assert tm["recomputed_cells"] > 0 and tm["loaded_cells"] > 0, "no hand cost table gave a hybrid"
    assert tm["loaded_cells"] + tm["recomputed_cells"] == sum(b.n_ctx) * L
    hid = sess.ctx.read_final_hidden(B)
    out = logits.cpu().numpy().copy()
    layers = sorted({0, 1, L // 2, L - 1})
    got_all = [sess.read_pages(1 + i, b.n_ctx[i], layers) for i in range(B)]
    # the same splits through the planned path
    sess.pool.fill_(0xFF)
    sess.restore(reqs, splits, want_logits=True)
    n_exact = n_cmp = 0
    worst_host = (1.0, 0.0)
    for i in range(B):
        n, (mode, kk, cc) = b.n_ctx[i], splits[i]
        want_mode = b.forced_mode if b.forced_mode >= 0 else (0 if n >= l_delta else 1)
        assert mode == want_mode and 0 <= kk <= n and 0 <= cc <= L
        planned = sess.read_pages(1 + i, n, layers)
        ref = reqs[i]["host_kv"].numpy()[:sess.host_kv_bytes(n)].reshape(L, -1, sess.page_bytes)
        for li, l in enumerate(layers):
            gk, gv = decode_pages(shape, got_all[i][li:li + 1], n)
            pk, pv = decode_pages(shape, planned[li:li + 1], n)
            rk, rv = decode_pages(shape, ref[l:l + 1], n)
            lo = kk if l < cc else 0                       # cells [lo, n) of this layer were loaded
            assert np.array_equal(gk[0, lo:], rk[0, lo:]) and np.array_equal(gv[0, lo:], rv[0, lo:]), \
                f"{b.config} request {i} layer {l}: loaded cells differ from the host block"
            for g, p_, r, nm in ((gk[0, :lo], pk[0, :lo], rk[0, :lo], "K"), (gv[0, :lo], pv[0, :lo], rv[0, :lo], "V")):
                if lo == 0:
                    continue
                assert np.isfinite(g).all(), f"{b.config} request {i} layer {l} {nm}: unwritten slot"
                n_cmp += 1
                dh = np.abs(g - r)
                ulp_h = np.maximum(np.abs(r), 1.0) * 2.0 ** -7
                worst_host = (min(worst_host[0], float((dh <= 2 * ulp_h).mean())), max(worst_host[1], float(dh.max())))
                if np.array_equal(g, p_):
                    n_exact += 1
                    continue
                d = np.abs(g - p_)
                ulp = np.maximum(np.abs(p_), 1.0) * 2.0 ** -7
                assert l > 0, f"{b.config} request {i} layer 0 {nm}: recomputed cells differ from the planned path's"
                assert (d <= 2 * ulp).mean() >= 0.97 and d.max() <= 0.25 * p_.std() + 0.05, \
                    f"{b.config} request {i} layer {l} {nm}: max diff {d.max()}, within 2 ulp {(d <= 2 * ulp).mean()}"
        del planned
    del got_all
    print(f"{b.config}: {n_exact} of {n_cmp} recomputed (request, layer, K|V) blocks bit-identical to the planned path "
          f"under the same splits; against the single-pass prefill: at worst {worst_host[0]:.3f} of a block's cells "
          f"within 2 ulp, max difference {worst_host[1]:.4f}")
    for i in sorted({0, B - 1}):
        ref = T.logits_last(shape, ws, hid[i].astype(np.float64), act="bf16")
        err = np.abs(out[i] - ref).max()
        assert err <= 2e-2, f"{b.config} request {i}: run-time scheduled logits max abs err {err}"


@pytest.mark.timeout(900)
@pytest.mark.parametrize("config", ["cfg3", "cfg4"])
def test_8b_configurations_at_full_size(config):
    b, sess, ws, reqs = build(config)
    try:
        longest = int(np.argmax(b.n_ctx))
        check_layers_0_and_1(b, sess, ws, reqs, longest)
        L = b.shape.n_layers
        check_teacher_forced(b, sess, ws, reqs, out_layers=(0, 1, L // 2, L - 2) if config == "cfg3"
                             else (0, 1, 2, L // 2 - 1, L // 2, L - 3, L - 2))
        splits = check_hybrid_restore(b, sess, ws, reqs)
        if config == "cfg3":
            assert splits[0][1] == b.n_ctx[0] and 0 < splits[0][2] < b.shape.n_layers   # layer-wise
        check_run_time_scheduled_restore(b, sess, ws, reqs, l_delta=4096)
    finally:
        release(b, sess)
        for r in reqs:
            r["host_kv"] = None
        torch.cuda.empty_cache()


@pytest.mark.timeout(900)
def test_tp_shard_configuration_5_at_full_size():
    b, sess, ws, reqs = build("cfg5")
    try:
        shape, L = b.shape, b.shape.n_layers
        longest = int(np.argmax(b.n_ctx))
        check_layers_0_and_1(b, sess, ws, reqs, longest)
        # prefix exactness through all layers against the bf16 noise floor
        P = 64
        toks = b.ctx_tokens[0][:P]
        stored, _ = T.prefill(shape, ws, toks, dtype=np.float32, act="bf16")
        exact, _ = T.prefill(shape, ws, toks, dtype=np.float32)
        for l in range(L):
            gk, gv = host_layer(sess, b, reqs, 0, l)
            for got, st, ex, nm in ((gk[:P], stored.k[l], exact.k[l], "K"), (gv[:P], stored.v[l], exact.v[l], "V")):
                ex = ex.astype(np.float64)
                e_gpu, e_ref = got - ex, st - ex
                gr, gm = float(np.sqrt(np.mean(e_gpu ** 2))), float(np.abs(e_gpu).max())
                rr, rm = float(np.sqrt(np.mean(e_ref ** 2))), float(np.abs(e_ref).max())
                if l in (0, 1, 39, 79):
                    print(f"cfg5 layer {l} {nm}: gpu rms {gr:.5f} max {gm:.5f}; bf16 cpu rms {rr:.5f} max {rm:.5f}")
                assert gr <= 1.3 * rr + 1e-4 and gm <= 1.6 * rm + 1e-3, \
                    f"layer {l} {nm}: rms {gr} max {gm} vs noise floor {rr} / {rm}"
        check_teacher_forced(b, sess, ws, reqs, out_layers=(0, 1, 2, L // 2 - 1, L // 2, L - 3, L - 2))
        check_hybrid_restore(b, sess, ws, reqs)
        check_run_time_scheduled_restore(b, sess, ws, reqs, l_delta=16384)
    finally:
        release(b, sess)
