"""GPU parity, configuration 1 (tiny float32 decoder, B=2, n=(128,64), forced
splits k=(64,32), 16 new tokens each): page tables bit-exact, KV and
first-token logits within 1e-4 of the oracle, loaded cells byte-identical."""
import numpy as np
import pytest
import torch

from oracle import transformer as T
from oracle.pagetable import PageTable
from workloads import WeightSource, churn_script, make_batch

from gpu_util import decode_pages, host_block, kv_tolerance_ok, oracle_batch, stack_kv

pytestmark = pytest.mark.gpu

N_PAGES = 64


@pytest.fixture(scope="module")
def env():
    from paper_2604_25080_amd.runtime import Session
    b = make_batch("cfg1")
    refs, ws = oracle_batch(b)
    sess = Session(b.shape, ws, max_batch=4, max_tokens=512, max_positions=256, n_pages=N_PAGES,
                   chunk_rows=256, pool_fill=0xFF)
    host = [sess.pin_host_kv(host_block(b.shape, T.kv_to_pages(b.shape, refs[i][0], b.n_ctx[i])))
            for i in range(len(b.n_ctx))]
    yield b, refs, ws, sess, host
    sess.close()


def fragment(sess, oracle_pt, seed):
    for op in churn_script(seed, N_PAGES, n_ops=40, max_tokens=60):
        if op[0] == "alloc":
            sess.cache.alloc(1000 + op[1], op[2])
            oracle_pt.alloc(1000 + op[1], op[2])
        else:
            sess.cache.free(1000 + op[1])
            oracle_pt.release(1000 + op[1])


def run_and_check(env, splits, seed=3, check_logits=True, dynamic=None):
    """`dynamic` = (cost model, plan options[, keyword arguments of Session.restore_dynamic]): no
    splits are given, the library schedules at run time and reports the splits that resulted;
    everything is then checked against those."""
    b, refs, ws, sess, host = env
    sess.pool.fill_(0xFF)                       # NaN pattern: every owned slot must be overwritten
    opt = PageTable(N_PAGES)
    stale = [r for r in list(opt.tables)]
    assert not stale
    fragment(sess, opt, seed)
    reqs = []
    try:
        for i in range(len(b.n_ctx)):
            rid = 1 + i
            sess.cache.alloc(rid, b.n_ctx[i] + b.n_new[i])
            assert sess.cache.page_table(rid) == opt.alloc(rid, b.n_ctx[i] + b.n_new[i])
            reqs.append(dict(req_id=rid, ctx_tokens=b.ctx_tokens[i], new_tokens=b.new_tokens[i],
                             host_kv=host[i]))
        if dynamic is None:
            logits, tm = sess.restore(reqs, [(0, k, c) for k, c in splits])
        else:
            logits, got_splits, tm, st = sess.restore_dynamic(reqs, *dynamic[:2], **(dynamic[2] if len(dynamic) > 2 else {}))
            splits = [(k, c) for _, k, c in got_splits]
            tm = dict(tm, splits=got_splits, stats=st)
        for i in range(len(b.n_ctx)):
            n, m = b.n_ctx[i], b.n_new[i]
            raw = sess.read_pages(1 + i, n + m)
            k, v = decode_pages(b.shape, raw, n + m)
            rk, rv = stack_kv(b.shape, refs[i][0], refs[i][1])
            for got, ref, nm in ((k, rk, "K"), (v, rv, "V")):
                assert np.isfinite(got).all(), f"request {i}: unwritten {nm} slot"
                ok, worst, _ = kv_tolerance_ok(b.shape, got, ref)
                assert ok, f"request {i} {nm}: max abs err {worst}"
            # loaded cells are byte-identical to the host block
            kk, cc = splits[i]
            hk, hv = decode_pages(b.shape, host[i].numpy()[:sess.host_kv_bytes(n)].reshape(
                b.shape.n_layers, -1, sess.page_bytes), n)
            for l in range(b.shape.n_layers):
                lo = kk if l < cc else 0
                assert np.array_equal(k[l, lo:n], hk[l, lo:n]) and np.array_equal(v[l, lo:n], hv[l, lo:n])
            if check_logits:
                err = np.abs(logits[i].cpu().numpy().astype(np.float64) - refs[i][2]).max()
                assert err <= 1e-4, f"request {i}: logits max abs err {err}"
        return tm
    finally:
        for rid in list(opt.tables):
            sess.cache.free(rid)
        assert sess.cache.n_free == N_PAGES


def test_cfg1_forced_splits(env):
    b = env[0]
    tm = run_and_check(env, b.forced_splits)
    assert tm["recomputed_cells"] == (64 + 32) * 2
    assert tm["loaded_cells"] == (64 + 32) * 2
    assert tm["loaded_bytes"] >= tm["loaded_cells"] * b.shape.kv_bytes_per_token_layer


def test_cfg1_sequential_join_mode(env):
    b, refs, ws, sess, host = env
    sess.ctx.set_pipelined_join(False)
    try:
        run_and_check(env, b.forced_splits, seed=9)
        run_and_check(env, [(0, 2), (64, 1)], seed=10)
    finally:
        sess.ctx.set_pipelined_join(True)


def test_cfg1_staged_load_path_and_pageable_host_memory(env):
    import paper_2604_25080_amd as cf
    b, refs, ws, sess, host = env
    try:
        # staged path (DMA into staging slots + scatter kernel) instead of the direct load kernel
        sess.ctx.set_load_path(1)
        run_and_check(env, b.forced_splits, seed=12)
        run_and_check(env, [(17, 1), (0, 2)], seed=13)
        sess.ctx.set_pipelined_join(False)
        run_and_check(env, [(33, 2), (47, 1)], seed=14)
        sess.ctx.set_pipelined_join(True)
        # host blocks in pageable memory: the automatic choice falls back to the staged path,
        # the forced direct path refuses them with an error instead of faulting
        pageable = [torch.from_numpy(h.numpy().copy()) for h in host]
        assert not pageable[0].is_pinned()
        env2 = (b, refs, ws, sess, pageable)
        sess.ctx.set_load_path(0)
        run_and_check(env2, b.forced_splits, seed=15)
        sess.ctx.set_load_path(2)
        with pytest.raises(cf.CfError) as e:
            run_and_check(env2, b.forced_splits, seed=15)
        assert e.value.status == cf.CF_ERR_INVALID_ARG
        run_and_check(env, b.forced_splits, seed=16)          # forced direct path, pinned blocks
        sess.ctx.set_load_path(2, 3)                          # fewer workgroups than virtual blocks
        run_and_check(env, [(17, 1), (5, 2)], seed=17)
    finally:
        sess.ctx.set_pipelined_join(True)
        sess.ctx.set_load_path(0, 8)


def test_cfg1_offload_returns_the_oracle_pages_on_both_paths(env):
    """Pages -> host block: the store kernel (pinned block) and the staged copy (pageable block or
    forced) give the same bytes, and they decode to the oracle's K/V within the float32 bound."""
    b, refs, ws, sess, host = env
    for i in range(len(b.n_ctx)):
        sess.cache.alloc(1 + i, b.n_ctx[i] + b.n_new[i])
    reqs = [dict(req_id=1 + i, ctx_tokens=b.ctx_tokens[i], new_tokens=b.new_tokens[i], host_kv=None)
            for i in range(len(b.n_ctx))]
    try:
        sess.restore(reqs, [(0, n, b.shape.n_layers) for n in b.n_ctx], want_logits=False)
        for i, n in enumerate(b.n_ctx):
            nbytes = sess.host_kv_bytes(n)
            direct = sess.offload(1 + i, n).numpy()[:nbytes].copy()
            sess.ctx.set_load_path(1)
            staged = sess.offload(1 + i, n).numpy()[:nbytes].copy()
            sess.ctx.set_load_path(0)
            pageable = torch.zeros(nbytes, dtype=torch.uint8)
            sess.ctx.offload(sess.cache, 1 + i, n, pageable.data_ptr())
            assert np.array_equal(direct, staged) and np.array_equal(direct, pageable.numpy())
            k, v = decode_pages(b.shape, direct.reshape(b.shape.n_layers, -1, sess.page_bytes), n)
            rk, rv = stack_kv(b.shape, refs[i][0], refs[i][1])
            assert np.abs(k - rk[:, :n]).max() <= 1e-4 and np.abs(v - rv[:, :n]).max() <= 1e-4
    finally:
        sess.ctx.set_load_path(0)
        for i in range(len(b.n_ctx)):
            sess.cache.free(1 + i)


def test_cfg1_waits_above_a_layer_cut_are_not_counted_as_waits_of_the_recompute(env):
    """cf_timing.compute_ms ends with the last recomputed layer; compute_wait_ms is the part of it
    that the stream stood waiting for loads.  With layer 0 recomputed, layer 1 loaded over a
    slow link and the pipelined join, the new turn's attention in layer 1 waits for nearly the
    whole copy -- after compute_ms has ended: none of that may show up in compute_wait_ms (the
    policy subtracts it from compute_ms).  With every layer recomputed for a prefix and the rest
    loaded, the same waits lie inside compute_ms and are reported."""
    b, refs, ws, sess, host = env
    L = b.shape.n_layers
    assert L == 2
    try:
        rate = 0.004                              # GB/s: a copy of ~100 ms against ~1 ms of compute
        sess.ctx.set_link_throttle(rate)
        tm = run_and_check(env, [(n, 1) for n in b.n_ctx], seed=31)
        floor_ms = tm["loaded_bytes"] / (rate * 1e9) * 1e3
        assert tm["total_ms"] >= 0.9 * floor_ms > 5 * tm["compute_ms"], (tm, floor_ms)
        assert tm["compute_wait_ms"] <= tm["compute_ms"], tm
        tm = run_and_check(env, [(n // 2, L) for n in b.n_ctx], seed=32)
        floor_ms = tm["loaded_bytes"] / (rate * 1e9) * 1e3
        assert tm["compute_ms"] >= 0.5 * floor_ms, (tm, floor_ms)      # it ended late because it waited ...
        assert 0.5 * tm["compute_ms"] <= tm["compute_wait_ms"] <= tm["compute_ms"], tm     # ... and says so
    finally:
        sess.ctx.set_link_throttle(0.0)


def test_cfg1_link_throttle_paces_the_copy_stream_and_changes_no_result(env):
    b, refs, ws, sess, host = env
    rate = 0.05                                   # GB/s
    try:
        for path in (0, 1):
            sess.ctx.set_load_path(path)
            sess.ctx.set_link_throttle(rate)
            tm = run_and_check(env, b.forced_splits, seed=21 + path)
            floor_ms = tm["loaded_bytes"] / (rate * 1e9) * 1e3
            assert tm["copy_ms"] >= 0.95 * floor_ms, (tm["copy_ms"], floor_ms)
            assert tm["copy_ms"] <= floor_ms + 20.0, (tm["copy_ms"], floor_ms)
            sess.ctx.set_link_throttle(0.0)
            tm = run_and_check(env, b.forced_splits, seed=21 + path)
            assert tm["copy_ms"] < 0.5 * floor_ms
    finally:
        sess.ctx.set_link_throttle(0.0)
        sess.ctx.set_load_path(0)


def test_cfg1_all_recompute_and_all_load(env):
    b = env[0]
    run_and_check(env, [(n, 2) for n in b.n_ctx], seed=4)
    tm = run_and_check(env, [(0, 2) for n in b.n_ctx], seed=5)
    assert tm["recomputed_cells"] == 0
    run_and_check(env, [(n, 0) for n in b.n_ctx], seed=5)     # cut 0: everything loaded


def test_cfg1_every_cut_and_a_sweep_of_unaligned_splits(env):
    b = env[0]
    ks = [0, 1, 15, 16, 17, 31, 33, 47, 63, 64]
    for c in (0, 1, 2):
        for k in ks:
            run_and_check(env, [(min(2 * k, b.n_ctx[0]), c), (k, 2 - c if k % 2 else c)], seed=6 + c,
                          check_logits=(k % 16 == 1))


def test_cfg1_pages_outside_the_batch_are_untouched(env):
    b, refs, ws, sess, host = env
    sess.pool.fill_(0xAB)
    sess.cache.alloc(50, 16 * 3)            # guard pages 0..2
    reqs = []
    for i in range(2):
        sess.cache.alloc(1 + i, b.n_ctx[i] + b.n_new[i])
        reqs.append(dict(req_id=1 + i, ctx_tokens=b.ctx_tokens[i], new_tokens=b.new_tokens[i], host_kv=host[i]))
    used = set(sess.cache.page_table(1) + sess.cache.page_table(2))
    sess.restore(reqs, [(0, 64, 2), (0, 32, 2)])
    view = sess.pool.view(b.shape.n_layers, N_PAGES, sess.page_bytes)
    other = [p for p in range(N_PAGES) if p not in used]
    assert bool((view[:, other] == 0xAB).all())
    for rid in (50, 1, 2):
        sess.cache.free(rid)


def test_cfg1_error_paths_return_codes_not_faults(env):
    import paper_2604_25080_amd as cf
    b, refs, ws, sess, host = env
    sess.cache.alloc(1, b.n_ctx[0] + b.n_new[0])
    r = dict(req_id=1, ctx_tokens=b.ctx_tokens[0], new_tokens=b.new_tokens[0], host_kv=host[0])
    try:
        for bad, code in (((0, 129, 2), cf.CF_ERR_INVALID_PLAN), ((0, 64, 3), cf.CF_ERR_INVALID_PLAN)):
            with pytest.raises(cf.CfError) as e:
                sess.restore([r], [bad])
            assert e.value.status == code
        with pytest.raises(cf.CfError) as e:
            sess.restore([dict(r, req_id=99)], [(0, 64, 2)])
        assert e.value.status == cf.CF_ERR_UNKNOWN_REQUEST
        with pytest.raises(cf.CfError) as e:
            sess.restore([dict(r, host_kv=None)], [(0, 64, 2)])
        assert e.value.status == cf.CF_ERR_INVALID_ARG
        toks = b.ctx_tokens[0].copy()
        toks[3] = 1000
        with pytest.raises(cf.CfError):
            sess.restore([dict(r, ctx_tokens=toks)], [(0, 64, 2)])
        sess.restore([dict(r, host_kv=None)], [(0, 128, 2)])      # nothing loaded: no host KV needed
    finally:
        sess.cache.free(1)


def test_cfg1_failure_after_enqueue_drains_the_streams_and_leaves_the_context_usable(env):
    """An error reported after work was enqueued (forced from the host: nothing on the GPU
    fails) must come back only when all three streams are idle -- the caller may free its host
    blocks right away -- and the same context must then restore the batch correctly."""
    import paper_2604_25080_amd as cf
    b, refs, ws, sess, host = env
    for nth in (1, 5, 8, 12):
        for i in range(len(b.n_ctx)):
            sess.cache.alloc(1 + i, b.n_ctx[i] + b.n_new[i])
        try:
            blocks = [h.clone().pin_memory() for h in host]
            reqs = [dict(req_id=1 + i, ctx_tokens=b.ctx_tokens[i], new_tokens=b.new_tokens[i], host_kv=blocks[i])
                    for i in range(len(b.n_ctx))]
            sess.ctx.inject_failure(nth)
            with pytest.raises(cf.CfError) as e:
                sess.restore(reqs, [(0, k, c) for k, c in b.forced_splits])
            assert e.value.status == cf.CF_ERR_HIP
            for blk in blocks:                       # the call has returned: scribbling must be harmless
                blk.fill_(0xFF)
            del blocks, reqs
        finally:
            for i in range(len(b.n_ctx)):
                sess.cache.free(1 + i)
        run_and_check(env, b.forced_splits, seed=20 + nth)      # the hook is one shot; results are right again


def test_cfg1_repeated_request_id_is_rejected(env):
    import paper_2604_25080_amd as cf
    b, refs, ws, sess, host = env
    sess.cache.alloc(1, b.n_ctx[0] + b.n_new[0])
    r = dict(req_id=1, ctx_tokens=b.ctx_tokens[0], new_tokens=b.new_tokens[0], host_kv=host[0])
    try:
        with pytest.raises(cf.CfError) as e:
            sess.restore([r, dict(r)], [(0, 64, 2), (0, 32, 2)])
        assert e.value.status == cf.CF_ERR_INVALID_ARG
    finally:
        sess.cache.free(1)


def test_cfg1_degenerate_batches(env):
    """Empty batch; a request with no context at all (pure new-turn prefill); one new token;
    a context of one token; all in one batch with an ordinary request."""
    b, refs, ws, sess, host = env
    shape = b.shape
    # empty batch: nothing to do, no error
    logits, tm = sess.restore([], [])
    assert tm["loaded_cells"] == 0 and tm["recomputed_cells"] == 0
    rng = np.random.default_rng(12)
    cases = [(0, 5), (1, 1), (17, 3), (b.n_ctx[1], b.n_new[1])]
    toks = [(rng.integers(0, shape.vocab, size=n).astype(np.int32), rng.integers(0, shape.vocab, size=m).astype(np.int32))
            for n, m in cases[:-1]] + [(b.ctx_tokens[1], b.new_tokens[1])]
    ref = []
    for c, nw in toks:
        if len(c):
            ref.append(T.full_reference(shape, ws, c, nw))
        else:                                     # no context: the new turn is the whole sequence
            kv_new, h = T.prefill(shape, ws, nw)
            ref.append((None, kv_new, T.logits_last(shape, ws, h[-1])))
    sess.pool.fill_(0xFF)
    reqs, splits = [], []
    try:
        for i, ((n, m), (c, nw)) in enumerate(zip(cases, toks)):
            sess.cache.alloc(1 + i, n + m)
            hk = sess.pin_host_kv(host_block(shape, T.kv_to_pages(shape, ref[i][0], n))) if n else None
            reqs.append(dict(req_id=1 + i, ctx_tokens=c, new_tokens=nw, host_kv=hk))
            splits.append((0, n // 2, shape.n_layers))
        logits, tm = sess.restore(reqs, splits)
        for i, (n, m) in enumerate(cases):
            k, v = decode_pages(shape, sess.read_pages(1 + i, n + m), n + m)
            if n:
                rk, rv = stack_kv(shape, ref[i][0], ref[i][1])
            else:
                rk, rv = np.stack(ref[i][1].k), np.stack(ref[i][1].v)
            assert np.isfinite(k).all() and np.isfinite(v).all()
            assert np.abs(k - rk).max() <= 1e-4 and np.abs(v - rv).max() <= 1e-4, f"case {cases[i]}"
            assert np.abs(logits[i].cpu().numpy() - ref[i][2]).max() <= 1e-4, f"case {cases[i]} logits"
    finally:
        for i in range(len(cases)):
            sess.cache.free(1 + i)


# ------------------------------------------------------------ run-time scheduling
def dyn_args(shape, kind, mode, l_delta=0, chunk=16):
    import paper_2604_25080_amd as cf
    tables = {
        # loads look ruinous: the compute engine takes every unit, the channel declines all
        "recompute": dict(f_c=1000, alpha=1000, beta=10, f_io=10 ** 12, gamma=10 ** 12),
        # recomputation looks ruinous: the channel takes every unit
        "load": dict(f_c=10 ** 12, alpha=10 ** 12, beta=10 ** 9, f_io=1000, gamma=1000),
        # the same order of magnitude as this tiny model really shows: a race, any split is legal
        "race": dict(f_c=25_000_000, alpha=300_000, beta=100_000, f_io=15_000_000, gamma=40_000_000),
    }
    return (cf.cost_model(**tables[kind]),
            cf.plan_opts(chunk, l_delta, shape.n_layers, shape.kv_bytes_per_token_layer, mode))


@pytest.mark.parametrize("mode", [0, 1, -1])
def test_cfg1_run_time_scheduling_restores_the_same_cache(env, mode):
    b = env[0]
    L = b.shape.n_layers
    total = sum(b.n_ctx) * L
    # mode -1 with l_delta 100: request 0 (128 tokens) token-wise, request 1 (64) layer-wise
    import paper_2604_25080_amd as cf
    # a step may hold any number of consecutive chunks of a request (the default; the last
    # recompute step then carries the planned tail itself when the batch has no layer-wise
    # group), one chunk per request, or be capped in time; a contended machine seeds the ratios
    # (passing overlap factors also restarts the ratios measured / predicted that a context
    # carries from call to call: each of these made-up cost tables starts from a clean slate)
    variants = ({"overlap": cf.overlap_model(1000, 1000)}, {"units_per_request": 1},
                {"step_cap_ps": 30_000_000, "units_per_request": 2}, {"overlap": cf.overlap_model(1300, 1200)})
    for seed, (kind, extra) in enumerate((k, e) for k in ("recompute", "load", "race", "race") for e in variants):
        tm = run_and_check(env, None, seed=30 + seed, dynamic=dyn_args(b.shape, kind, mode, l_delta=100) + (extra,))
        splits, st = tm["splits"], tm["stats"]
        # without a layer-wise group the last recompute step is recognised before its launch
        # and runs the new turns in the same pass
        assert st["last_step_merged"] == (1 if mode == 0 and tm["recomputed_cells"] > 0 else 0)
        assert tm["recomputed_cells"] + tm["loaded_cells"] == total
        for (m, k, c), n in zip(splits, b.n_ctx):
            assert m == (mode if mode >= 0 else (0 if n >= 100 else 1))
            assert (k % 16 == 0 or k == n) and 0 <= k <= n and 0 <= c <= L
            assert c == L if m == 0 else k == n
        rec = sum(k * c if m == 0 else n * c for (m, k, c), n in zip(splits, b.n_ctx))
        assert tm["recomputed_cells"] == rec
        if kind == "recompute":
            assert tm["loaded_cells"] == 0 and st["io_units"] == 0, (kind, extra, splits, st)
        if kind == "load":
            assert tm["recomputed_cells"] == 0 and st["compute_units"] == 0, (kind, extra, splits, st)
        assert st["compute_steps"] >= 1          # the new turn, at the least


def test_cfg1_run_time_scheduling_chunk_sizes_throttle_and_errors(env):
    import paper_2604_25080_amd as cf
    b, refs, ws, sess, host = env
    # larger chunks (ragged last chunk of request 1: 64 = 48 + 16), throttled link
    run_and_check(env, None, seed=40, dynamic=dyn_args(b.shape, "race", 0, chunk=48))
    sess.ctx.set_link_throttle(0.05)
    try:
        tm = run_and_check(env, None, seed=41, dynamic=dyn_args(b.shape, "race", 0, chunk=32))
        assert tm["copy_ms"] >= 0.9 * tm["loaded_bytes"] / 0.05e9 * 1e3
    finally:
        sess.ctx.set_link_throttle(0.0)
    # argument errors come back as codes
    sess.cache.alloc(1, b.n_ctx[0] + b.n_new[0])
    r = dict(req_id=1, ctx_tokens=b.ctx_tokens[0], new_tokens=b.new_tokens[0], host_kv=host[0])
    try:
        cost, opts = dyn_args(b.shape, "race", 0, chunk=24)          # not a multiple of the page size
        with pytest.raises(cf.CfError) as e:
            sess.restore_dynamic([r], cost, opts)
        assert e.value.status == cf.CF_ERR_INVALID_ARG
        cost, opts = dyn_args(b.shape, "race", 0)
        pageable = torch.from_numpy(host[0].numpy().copy())
        with pytest.raises(cf.CfError) as e:
            sess.restore_dynamic([dict(r, host_kv=pageable)], cost, opts)
        assert e.value.status == cf.CF_ERR_INVALID_ARG
        with pytest.raises(cf.CfError) as e:
            sess.restore_dynamic([dict(r, req_id=77)], cost, opts)
        assert e.value.status == cf.CF_ERR_UNKNOWN_REQUEST
        sess.ctx.set_stage(1, 2)
        with pytest.raises(cf.CfError):
            sess.restore_dynamic([r], cost, opts)
        sess.ctx.set_stage(0, b.shape.n_layers)
        logits, splits, tm, st = sess.restore_dynamic([], cost, opts)
        assert splits == [] and tm["loaded_cells"] == 0
    finally:
        sess.ctx.set_stage(0, b.shape.n_layers)
        sess.cache.free(1)
