"""GPU parity for bf16 models on small shapes that still span several GEMM
and attention tiles with ragged tails: hybrid restoration (random token and
layer splits, fragmented page pool) against the float64 oracle run with the
same bf16-rounded weights.  KV within 2e-2 (one bf16 ulp where an ulp exceeds that, |ref| >= 4),
logits within 2e-2, loaded cells byte-identical, and the MFMA kernels
against the plain-FMA kernels of the same library."""
import numpy as np
import pytest
import torch

from oracle import transformer as T
from oracle.pagetable import PageTable
from workloads import SHAPES, WeightSource, churn_script
from workloads.batches import random_batch

from gpu_util import decode_pages, host_block, kv_tolerance_ok, oracle_batch, stack_kv

pytestmark = pytest.mark.gpu

N_PAGES = 400


def build(shape_name, seed, n_req, n_lo, n_hi, m_lo, m_hi, chunk_rows, n_pages=N_PAGES):
    from paper_2604_25080_amd.runtime import Session
    b = random_batch(seed, shape_name, n_req, n_lo, n_hi, m_lo, m_hi)
    refs, ws = oracle_batch(b)
    sess = Session(b.shape, ws, max_batch=n_req, max_tokens=sum(b.n_ctx) + sum(b.n_new),
                   max_positions=max(b.n_ctx) + max(b.n_new) + 16, n_pages=n_pages,
                   chunk_rows=chunk_rows, pool_fill=0xFF, staging_bytes=1 << 20)
    host = [sess.pin_host_kv(host_block(b.shape, T.kv_to_pages(b.shape, refs[i][0], b.n_ctx[i])))
            for i in range(n_req)]
    return b, refs, sess, host


def restore_and_compare(b, refs, sess, host, splits, seed, simple_only=False, pipelined=True, load_path=0,
                        dynamic=None):
    # dynamic = (cost model, plan options): scheduled at run time, checked against the splits that resulted
    sess.ctx.set_kernel_set(simple_only)
    sess.ctx.set_pipelined_join(pipelined)
    sess.ctx.set_load_path(load_path)
    sess.pool.fill_(0xFF)
    opt = PageTable(sess.n_pages)
    for op in churn_script(seed, sess.n_pages, n_ops=60, max_tokens=300):
        if op[0] == "alloc":
            sess.cache.alloc(1000 + op[1], op[2]); opt.alloc(1000 + op[1], op[2])
        else:
            sess.cache.free(1000 + op[1]); opt.release(1000 + op[1])
    reqs = []
    out = {}
    try:
        for i in range(len(b.n_ctx)):
            sess.cache.alloc(1 + i, b.n_ctx[i] + b.n_new[i])
            assert sess.cache.page_table(1 + i) == opt.alloc(1 + i, b.n_ctx[i] + b.n_new[i])
            reqs.append(dict(req_id=1 + i, ctx_tokens=b.ctx_tokens[i], new_tokens=b.new_tokens[i], host_kv=host[i]))
        if dynamic is None:
            logits, tm = sess.restore(reqs, [(0, k, c) for k, c in splits])
        else:
            logits, got, tm, st = sess.restore_dynamic(reqs, *dynamic)
            splits = [(k, c) for _, k, c in got]
            tm = dict(tm, splits=got, stats=st)
        worst_kv = worst_logit = 0.0
        for i in range(len(b.n_ctx)):
            n, m = b.n_ctx[i], b.n_new[i]
            k, v = decode_pages(b.shape, sess.read_pages(1 + i, n + m), n + m)
            rk, rv = stack_kv(b.shape, refs[i][0], refs[i][1])
            for got, ref, nm in ((k, rk, "K"), (v, rv, "V")):
                assert np.isfinite(got).all(), f"request {i}: unwritten {nm} slot"
                ok, worst, _ = kv_tolerance_ok(b.shape, got, ref)
                assert ok, f"request {i} {nm}: max abs err {worst} (splits {splits[i]})"
                worst_kv = max(worst_kv, worst)
            kk, cc = splits[i]
            hk, hv = decode_pages(b.shape, host[i].numpy()[:sess.host_kv_bytes(n)].reshape(
                b.shape.n_layers, -1, sess.page_bytes), n)
            for l in range(b.shape.n_layers):
                lo = kk if l < cc else 0
                assert np.array_equal(k[l, lo:n], hk[l, lo:n]) and np.array_equal(v[l, lo:n], hv[l, lo:n])
            err = np.abs(logits[i].cpu().numpy().astype(np.float64) - refs[i][2]).max()
            assert err <= 2e-2, f"request {i}: logits max abs err {err}"
            worst_logit = max(worst_logit, err)
            out[i] = (k, v, logits[i].cpu().numpy())
        return out, worst_kv, worst_logit, tm
    finally:
        for rid in list(opt.tables):
            sess.cache.free(rid)
        sess.ctx.set_kernel_set(False)
        sess.ctx.set_pipelined_join(True)
        sess.ctx.set_load_path(0)


@pytest.fixture(scope="module")
def mini():
    env = build("mini-bf16", 11, 4, 100, 700, 5, 150, chunk_rows=512)
    yield env
    env[2].close()


def test_mini_bf16_hybrid_splits_match_oracle(mini):
    b, refs, sess, host = mini
    L = b.shape.n_layers
    rng = np.random.default_rng(3)
    plans = [
        [(n, L) for n in b.n_ctx],                                   # all recompute
        [(0, L) for n in b.n_ctx],                                   # all load
        [((n // 2) // 16 * 16, L) for n in b.n_ctx],                 # token-wise, page aligned
        [(n, int(rng.integers(0, L + 1))) for n in b.n_ctx],         # layer-wise cuts
        [(int(rng.integers(0, n + 1)), int(rng.integers(0, L + 1))) for n in b.n_ctx],  # anything
    ]
    for p, splits in enumerate(plans):
        out_p, wkv, wlg, tm = restore_and_compare(b, refs, sess, host, splits, seed=20 + p)
        print(f"plan {p}: worst KV err {wkv:.4g}, worst logit err {wlg:.4g}")
        # the sequential join (recompute || load, wait, then the new-turn prefill) gives the same bits
        out_s, *_ = restore_and_compare(b, refs, sess, host, splits, seed=20 + p, pipelined=False)
        # ... and so does the staged load path (DMA into staging slots + scatter kernel) in place
        # of the direct load kernel, in either join mode
        out_d, *_ = restore_and_compare(b, refs, sess, host, splits, seed=20 + p, pipelined=(p % 2 == 0),
                                        load_path=1)
        for i in out_p:
            for other in (out_s, out_d):
                assert np.array_equal(out_p[i][0], other[i][0]) and np.array_equal(out_p[i][1], other[i][1])
                assert np.abs(out_p[i][2] - other[i][2]).max() <= 2e-2


def test_sampled_hidden_rows_match_the_oracle_and_feed_the_teacher_forced_checks(mini):
    """cf_ctx_capture_rows on a shape the oracle runs end to end: the residual stream of sampled
    context and new-turn rows at every layer entry (and leaving the last layer) against the
    oracle's own hidden states, then the per-layer teacher-forced checks the full-size tests use
    (K/V cells and layer output rows from the GPU's hidden rows), here on every layer."""
    from gpu_util import teacher_forced_layer_checks
    b, refs, sess, host = mini
    shape, L, B = b.shape, b.shape.n_layers, len(b.n_ctx)
    ws = WeightSource(shape, b.weight_seed, cache=True)
    off = np.concatenate([[0], np.cumsum(b.n_ctx)])
    noff = off[-1] + np.concatenate([[0], np.cumsum(b.n_new)])
    rows, rq, ps, new = [], [], [], []
    for i in range(B):
        for p in sorted({0, 1, 15, 16, 17, 63, 64, 127, 128, b.n_ctx[i] // 2, b.n_ctx[i] - 1}):
            if p < b.n_ctx[i]:
                rows.append(off[i] + p); rq.append(i); ps.append(p); new.append(False)
        for t in sorted({0, b.n_new[i] - 1}):
            rows.append(noff[i] + t); rq.append(i); ps.append(b.n_ctx[i] + t); new.append(True)
    rq, ps, new = np.array(rq), np.array(ps), np.array(new)
    hid = torch.full((2 * L + 1, len(rows), shape.d_model), float("nan"), dtype=torch.float32, device="cuda")
    reqs = []
    try:
        for i in range(B):
            sess.cache.alloc(1 + i, b.n_ctx[i] + b.n_new[i])
            reqs.append(dict(req_id=1 + i, ctx_tokens=b.ctx_tokens[i], new_tokens=b.new_tokens[i], host_kv=None))
        sess.ctx.capture_rows(np.array(rows, dtype=np.int32), hid.data_ptr())
        sess.restore(reqs, [(0, n, L) for n in b.n_ctx])
        got = hid.cpu().numpy().astype(np.float64)
        blocks = [sess.offload(1 + i, b.n_ctx[i] + b.n_new[i]) for i in range(B)]
    finally:
        for i in range(B):
            sess.cache.free(1 + i)
    for i in range(B):
        toks = np.concatenate([b.ctx_tokens[i], b.new_tokens[i]])
        _, h_final, h_in = T.prefill(shape, ws, toks, return_hidden=True)
        sel = np.nonzero(rq == i)[0]
        for l in range(L + 1):
            ref = (h_in[l] if l < L else h_final)[ps[sel]]
            g = got[2 * l, sel]
            if l < L:      # entering the MLP half: context rows have none in their last layer
                mid = got[2 * l + 1, sel]
                assert np.isfinite(mid[new[sel]]).all() and np.isnan(mid[~new[sel]]).all() == (l == L - 1)
            # context rows stop after the K/V write of their last layer: nothing leaves layer L-1
            live = np.ones(len(sel), bool) if l < L else new[sel]
            assert np.isnan(g[~live]).all()
            err = np.abs(g[live] - ref[live]).max()
            assert err <= 2e-2 * max(1.0, float(np.sqrt(np.mean(ref ** 2)))), f"request {i} layer {l}: hidden rows off by {err}"
    # the same rows through the per-layer checks (every layer's output; the last layer's only
    # exists for new-turn rows, which the helper skips by construction: out_layers below L-1)
    st = teacher_forced_layer_checks(shape, ws, sess, [n + m for n, m in zip(b.n_ctx, b.n_new)], blocks, got.astype(np.float32),
                                     rq, ps, out_layers=set(range(L)), label="mini-bf16", dtype=np.float64)
    assert st["attention_elems"] > 0 and st["mlp_elems"] > 0 and st["kv_cells"] == L * len(rows) * 2 * shape.n_kv_heads * shape.head_dim


def test_mini_bf16_mfma_kernels_agree_with_plain_kernels(mini):
    b, refs, sess, host = mini
    splits = [(n, b.shape.n_layers) for n in b.n_ctx]
    fast, *_ = restore_and_compare(b, refs, sess, host, splits, seed=31)
    slow, *_ = restore_and_compare(b, refs, sess, host, splits, seed=31, simple_only=True)
    for i in fast:
        assert np.abs(fast[i][0] - slow[i][0]).max() <= 2e-2
        assert np.abs(fast[i][2] - slow[i][2]).max() <= 2e-2


def test_mini_bf16_hybrid_equals_all_recompute_on_the_gpu(mini):
    # recomputed cells do not depend on what else is in the batch or where the split is
    b, refs, sess, host = mini
    L = b.shape.n_layers
    full, *_ = restore_and_compare(b, refs, sess, host, [(n, L) for n in b.n_ctx], seed=41)
    part, *_ = restore_and_compare(b, refs, sess, host, [((n // 3) // 16 * 16, L) for n in b.n_ctx], seed=42)
    for i in full:
        k = (b.n_ctx[i] // 3) // 16 * 16
        assert np.array_equal(full[i][0][:, :k], part[i][0][:, :k])
        assert np.array_equal(full[i][1][:, :k], part[i][1][:, :k])


def test_long_context_few_new_tokens_splits_the_key_range():
    # 3 new tokens over contexts of 2100..2900 tokens: too few query blocks to fill the GPU, so
    # the suffix attention splits each key range into slices and merges the partial results
    b, refs, sess, host = build("mini-bf16", 13, 2, 2100, 2900, 3, 9, chunk_rows=1024, n_pages=1000)
    try:
        L = b.shape.n_layers
        restore_and_compare(b, refs, sess, host, [(0, L) for n in b.n_ctx], seed=61)
        restore_and_compare(b, refs, sess, host, [(n // 2 // 16 * 16, L) for n in b.n_ctx], seed=62)
    finally:
        sess.close()


def test_head_dim_64_bf16_model():
    b, refs, sess, host = build("mini64-bf16", 12, 3, 60, 400, 3, 70, chunk_rows=256)
    try:
        L = b.shape.n_layers
        restore_and_compare(b, refs, sess, host, [(n, L) for n in b.n_ctx], seed=51)
        restore_and_compare(b, refs, sess, host, [((n // 2), 1) for n in b.n_ctx], seed=52)
    finally:
        sess.close()


@pytest.mark.parametrize("shape_name", ["mini64-gqa2-bf16", "mini128-gqa3-bf16"])
def test_remaining_head_geometries_of_the_attention_kernel(shape_name):
    """head_dim 64 with an even query group (two heads of a KV group per workgroup) and head_dim
    128 with an odd one (one head per workgroup): ragged lengths, hybrid splits, and -- few new
    tokens over contexts of 2100..2900 tokens -- split key ranges with their combine pass; all
    against the oracle, and against the plain kernels of the same library."""
    b, refs, sess, host = build(shape_name, 14, 3, 60, 700, 3, 70, chunk_rows=256)
    try:
        L = b.shape.n_layers
        fast, *_ = restore_and_compare(b, refs, sess, host, [(n, L) for n in b.n_ctx], seed=53)
        slow, *_ = restore_and_compare(b, refs, sess, host, [(n, L) for n in b.n_ctx], seed=53, simple_only=True)
        for i in fast:
            assert np.abs(fast[i][0] - slow[i][0]).max() <= 2e-2 and np.abs(fast[i][2] - slow[i][2]).max() <= 2e-2
        restore_and_compare(b, refs, sess, host, [((n // 2), 1) for n in b.n_ctx], seed=54)
        restore_and_compare(b, refs, sess, host, [(n // 3 // 16 * 16, L) for n in b.n_ctx], seed=55)
    finally:
        sess.close()
    b, refs, sess, host = build(shape_name, 15, 2, 2100, 2900, 3, 9, chunk_rows=1024, n_pages=1000)
    try:
        L = b.shape.n_layers
        restore_and_compare(b, refs, sess, host, [(0, L) for n in b.n_ctx], seed=63)
        restore_and_compare(b, refs, sess, host, [(n // 2 // 16 * 16, L) for n in b.n_ctx], seed=64)
    finally:
        sess.close()


@pytest.mark.parametrize("shape_name", ["mini-bf16", "mini64-gqa2-bf16"])
def test_small_shape_end_to_end_on_the_big_gemm_tile(shape_name):
    """The 256x256 GEMM tile (and its quartered tail) is what the full-size runs use; the small
    shapes take the 128 / 64 tiles by themselves.  Forced here (the GEMMs whose shapes allow the
    big tile: M >= 256, N >= 256, K a multiple of 128), one hybrid restore end to end against
    the oracle -- and bit for bit against the tiles the heuristic picks.  On the big tile the QKV
    projection rotates and writes Q, K and V in its own epilogue (head_dim 128 and 64: a wave
    tile of one head, and of two heads with K and V heads side by side in one block tile); on
    the small tiles a separate kernel does, so the bit comparison also holds the two against
    each other."""
    import paper_2604_25080_amd as cf
    b, refs, sess, host = build(shape_name, 16, 3, 300, 700, 40, 150, chunk_rows=2048)
    try:
        L = b.shape.n_layers
        splits = [(n // 2 // 16 * 16, L) for n in b.n_ctx]
        ref_out, *_ = restore_and_compare(b, refs, sess, host, splits, seed=71)
        for force in (256, 257):
            cf.lib.cf_debug_force_gemm_tile(force)
            try:
                out, *_ = restore_and_compare(b, refs, sess, host, splits, seed=71)
            finally:
                cf.lib.cf_debug_force_gemm_tile(0)
            for i in out:
                assert np.array_equal(out[i][0], ref_out[i][0]) and np.array_equal(out[i][1], ref_out[i][1])
                assert np.array_equal(out[i][2], ref_out[i][2])
    finally:
        sess.close()


def _token_bits(shape, raw, n_tokens):
    """raw uint8 [L, P, page_bytes] of a bf16 cache -> (K, V) uint16 [L, n_tokens, Hkv, hd]: the
    stored bits, token-major (K part [head][slot][hd], V part [head][hd][slot] in a page)."""
    L, P, _ = raw.shape
    hk, hd = shape.n_kv_heads, shape.head_dim
    vals = np.ascontiguousarray(raw).view(np.uint16).reshape(L, P, -1)
    half = hk * 16 * hd
    k = vals[:, :, :half].reshape(L, P, hk, 16, hd).transpose(0, 1, 3, 2, 4).reshape(L, P * 16, hk, hd)
    v = vals[:, :, half:].reshape(L, P, hk, hd, 16).transpose(0, 1, 4, 2, 3).reshape(L, P * 16, hk, hd)
    return k[:, :n_tokens], v[:, :n_tokens]


def test_long_loads_move_the_host_bytes_on_every_load_path():
    """Loads long enough for the DMA split of the direct path (whole pages with consecutive pool
    ids, 4 MiB or more per request and layer -- here 375 pages of 16 KiB) with everything that
    breaks a run: a ragged last page whose tail slots belong to the new turn, a split in the
    middle of a page, a pool fragmented by earlier traffic (short runs that stay with the load
    kernel), two requests per layer (two DMA queues).  The host blocks hold random bytes; what
    must come out is those bytes in every loaded cell, and the fill pattern in every slot of the
    request's pages that no token of the context owns -- on the direct path, on the load kernel
    alone and on the staged path alike."""
    from paper_2604_25080_amd.runtime import Session
    shape = SHAPES["mini-bf16"]
    L = shape.n_layers
    ws = WeightSource(shape, 77, cache=True)
    n_ctx, n_new, k_split = [6005, 4700], [40, 40], [0, 37]
    rng = np.random.default_rng(5)
    ctx_tokens = [rng.integers(0, shape.vocab, size=n).astype(np.int32) for n in n_ctx]
    new_tokens = [rng.integers(0, shape.vocab, size=m).astype(np.int32) for m in n_new]
    sess = Session(shape, ws, max_batch=2, max_tokens=1024, max_positions=max(n_ctx) + 64, n_pages=1400,
                   chunk_rows=1024, pool_fill=0xEE, staging_bytes=1 << 20)
    try:
        host = []
        for n in n_ctx:
            t = sess.pinned(sess.host_kv_bytes(n))
            t.copy_(torch.from_numpy(rng.integers(0, 256, size=t.numel(), dtype=np.uint8)))
            host.append(t)
        for fragmented in (False, True):
            for path in (0, 2, 1):
                sess.ctx.set_load_path(path)
                sess.pool.fill_(0xEE)
                held = []
                if fragmented:      # scattered small allocations, every other one freed again
                    for j in range(60):
                        sess.cache.alloc(500 + j, 16 * (1 + j % 7))
                    for j in range(0, 60, 2):
                        sess.cache.free(500 + j)
                    held = list(range(501, 560, 2))
                reqs = []
                for i in range(2):
                    sess.cache.alloc(1 + i, n_ctx[i] + n_new[i])
                    reqs.append(dict(req_id=1 + i, ctx_tokens=ctx_tokens[i], new_tokens=new_tokens[i], host_kv=host[i]))
                try:
                    tables = [sess.cache.page_table(1 + i) for i in range(2)]
                    consecutive = [all(b == a + 1 for a, b in zip(t, t[1:])) for t in tables]
                    assert all(consecutive) != fragmented      # the churn did break the runs up
                    sess.restore(reqs, [(0, k_split[i], L) for i in range(2)], want_logits=False)
                    for i in range(2):
                        n, k0 = n_ctx[i], k_split[i]
                        alloc = n + n_new[i]
                        gk, gv = _token_bits(shape, sess.read_pages(1 + i, alloc), -(-alloc // 16) * 16)
                        hk, hv = _token_bits(shape, host[i].numpy()[:sess.host_kv_bytes(n)].reshape(L, -1, sess.page_bytes), n)
                        for l in range(L):
                            assert np.array_equal(gk[l, k0:n], hk[l, k0:n]) and np.array_equal(gv[l, k0:n], hv[l, k0:n]), \
                                f"request {i} layer {l} path {path} fragmented {fragmented}: loaded cells differ from the host block"
                            # no token of the context owns these slots (the new turn did not run)
                            assert (gk[l, n:] == 0xEEEE).all() and (gv[l, n:] == 0xEEEE).all(), \
                                f"request {i} layer {l} path {path}: a slot past the context was written"
                finally:
                    for i in range(2):
                        sess.cache.free(1 + i)
                    for r in held:
                        sess.cache.free(r)
    finally:
        sess.ctx.set_load_path(0)
        sess.close()


def test_stage_restore_from_boundary_activations(mini):
    """One pipeline stage's share (Sec. 3.2): the context is restricted to layers [b, e), recompute
    starts from the oracle's hidden states entering layer b, loads cover only the stage's layers
    of the host block; layers outside the stage keep their sentinel bytes."""
    import paper_2604_25080_amd as cf
    b, refs, sess, host = mini
    L = b.shape.n_layers
    ws = WeightSource(b.shape, b.weight_seed, cache=True)
    hidden = [T.prefill(b.shape, ws, b.ctx_tokens[i], return_hidden=True)[2] for i in range(len(b.n_ctx))]
    rng = np.random.default_rng(9)
    try:
        for (lb, le) in ((1, 3), (1, 2), (2, 3), (0, 2)):
            sess.ctx.set_stage(lb, le)
            sess.pool.fill_(0xFF)
            reqs, splits = [], []
            for i, n in enumerate(b.n_ctx):
                sess.cache.alloc(1 + i, n + b.n_new[i])
                bh = torch.from_numpy(np.ascontiguousarray(hidden[i][lb], dtype=np.float32))
                if (lb, le) != (1, 2):        # pinned rows are read by a kernel, pageable ones by a DMA copy
                    bh = bh.pin_memory()
                reqs.append(dict(req_id=1 + i, ctx_tokens=b.ctx_tokens[i], new_tokens=b.new_tokens[i],
                                 host_kv=host[i], boundary_h=bh.data_ptr(), _keep=bh))
                splits.append((0, int(rng.integers(0, n + 1)), int(rng.integers(0, le - lb + 1))))
            splits[0] = (0, b.n_ctx[0], le - lb)              # one request recomputes its whole stage
            # logits need the whole model
            with pytest.raises(cf.CfError):
                sess.restore(reqs, splits, want_logits=True)
            _, tm = sess.restore(reqs, splits, want_logits=False)
            assert tm["loaded_cells"] + tm["recomputed_cells"] == sum(b.n_ctx) * (le - lb)
            for i, n in enumerate(b.n_ctx):
                raw = sess.read_pages(1 + i, n)
                k, v = decode_pages(b.shape, raw, n)
                rk, rv = stack_kv(b.shape, refs[i][0], refs[i][1])
                for l in range(L):
                    if lb <= l < le:
                        for got, ref, nm in ((k[l], rk[l, :n], "K"), (v[l], rv[l, :n], "V")):
                            ok, worst, _ = kv_tolerance_ok(b.shape, got, ref)
                            assert ok, f"stage [{lb},{le}) request {i} layer {l} {nm}: {worst} (split {splits[i]})"
                    else:
                        full_pages = n // 16
                        assert (raw[l, :full_pages] == 0xFF).all(), f"layer {l} outside the stage was written"
                sess.cache.free(1 + i)
            if lb > 0:
                # recompute in a stage above layer 0 without boundary activations is refused
                sess.cache.alloc(1, b.n_ctx[0] + b.n_new[0])
                with pytest.raises(cf.CfError):
                    sess.restore([dict(reqs[0], boundary_h=None)], [splits[0]], want_logits=False)
                sess.cache.free(1)
    finally:
        sess.ctx.set_stage(0, L)
        for i in range(len(b.n_ctx)):
            try:
                sess.cache.free(1 + i)
            except Exception:
                pass


def test_captured_boundary_reproduces_the_full_prefill_bit_for_bit(mini):
    """cf_ctx_capture_boundary during a full GPU prefill, then a stage restore that recomputes from
    the captured rows: the stage's pages are bit-identical to the full prefill's, and the captured
    rows are the oracle's hidden states entering that layer (to bf16-pipeline accuracy)."""
    b, refs, sess, host = mini
    L, d = b.shape.n_layers, b.shape.d_model
    ws = WeightSource(b.shape, b.weight_seed, cache=True)
    B = len(b.n_ctx)
    reqs = [dict(req_id=1 + i, ctx_tokens=b.ctx_tokens[i], new_tokens=b.new_tokens[i], host_kv=None)
            for i in range(B)]
    try:
        for i in range(B):
            sess.cache.alloc(1 + i, b.n_ctx[i] + b.n_new[i])
        lb = 1
        cap = torch.zeros(sum(b.n_ctx), d, dtype=torch.float32, device="cuda")
        sess.ctx.capture_boundary(lb, cap.data_ptr(), cap.shape[0])
        sess.restore(reqs, [(0, n, L) for n in b.n_ctx], want_logits=False)
        full = [sess.read_pages(1 + i, b.n_ctx[i]).copy() for i in range(B)]
        rows = cap.cpu()
        off = 0
        for i, n in enumerate(b.n_ctx):                      # packed order = call order (equal cuts)
            ref = T.prefill(b.shape, ws, b.ctx_tokens[i], return_hidden=True)[2][lb]
            got = rows[off:off + n].numpy()
            assert np.abs(got - ref).max() <= 2e-2 * max(1.0, np.abs(ref).max())
            reqs[i]["boundary_h"] = rows[off:off + n].contiguous().pin_memory()
            off += n
        sess.pool.fill_(0xFF)
        sess.ctx.set_stage(lb, L)
        sess.restore(reqs, [(0, n, L - lb) for n in b.n_ctx], want_logits=False)
        for i, n in enumerate(b.n_ctx):
            got = sess.read_pages(1 + i, n)
            k0, v0 = decode_pages(b.shape, full[i][lb:], n)
            k1, v1 = decode_pages(b.shape, got[lb:], n)
            assert np.array_equal(k0, k1) and np.array_equal(v0, v1), f"request {i}"
    finally:
        sess.ctx.set_stage(0, L)
        for i in range(B):
            sess.cache.free(1 + i)


def test_mini_bf16_run_time_scheduling(mini):
    """No split is given: the two engines claim chunks / layers while the call runs.  Whatever
    split results, the restored cache and the logits must be the oracle's."""
    import paper_2604_25080_amd as cf
    b, refs, sess, host = mini
    L = b.shape.n_layers
    kvb = b.shape.kv_bytes_per_token_layer
    tables = {
        "recompute": dict(f_c=1000, alpha=1000, beta=10, f_io=10 ** 12, gamma=10 ** 12),
        "load": dict(f_c=10 ** 12, alpha=10 ** 12, beta=10 ** 9, f_io=1000, gamma=1000),
        "race": dict(f_c=20_000_000, alpha=60_000, beta=20_000, f_io=10_000_000, gamma=30_000_000),
    }
    seed = 60
    for mode, l_delta, chunk in ((0, 0, 64), (1, 0, 64), (-1, 400, 128), (0, 0, 256)):
        for kind in ("recompute", "load", "race", "race"):
            seed += 1
            dyn = (cf.cost_model(**tables[kind]), cf.plan_opts(chunk, l_delta, L, kvb, mode, 0, 150))
            out, wkv, wlg, tm = restore_and_compare(b, refs, sess, host, None, seed=seed, dynamic=dyn)
            splits, st = tm["splits"], tm["stats"]
            print(f"mode {mode} chunk {chunk} {kind}: splits {splits} steps {st['compute_steps']} "
                  f"loads {st['io_units']} KV err {wkv:.3g}")
            assert tm["recomputed_cells"] + tm["loaded_cells"] == sum(b.n_ctx) * L
            for (m, k, c), n in zip(splits, b.n_ctx):
                assert m == (mode if mode >= 0 else (0 if n >= l_delta else 1))
                assert (c == L and (k % chunk == 0 or k == n)) if m == 0 else k == n
            if kind == "recompute":
                assert tm["loaded_cells"] == 0
            if kind == "load":
                assert tm["recomputed_cells"] == 0
