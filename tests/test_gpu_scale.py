"""GPU parity at the benchmark's full model shape (Llama-3-8B-shaped, bf16) in
the launch configuration bench.py times (configuration 2: B=8, contexts drawn
from U[2048,16384], planner splits over a hand cost table), using checks the
CPU oracle can afford:

 1. prefix exactness - by causality the first P tokens of a request do not
    depend on the rest, so the oracle prefills exactly those through all 32
    layers and every K/V cell of those tokens is compared.  The reference is
    the oracle's bf16-storage forward (cache cells are 16-bit codes, so both
    sides round where a bf16 model stores); the distance to the unrounded
    forward is printed beside it;
 2. constant-token request - if all tokens of a request are equal, every
    position has the same hidden state at every layer (attention averages
    identical values), so its whole cache follows from a ONE-token oracle
    forward plus the rotary turn of K: V[l][t] = V[l][0], K[l][t] =
    rope_t(K[l][0]).  This holds at any length and pins long-range attention
    (mask, online softmax normalisation), rotary angles at large positions and
    the page writes across all layers at 16k tokens;
 3. hybrid vs all-recompute on the GPU: recomputed cells bit-identical, loaded
    cells byte-identical to the host block;
 4. logits: the oracle's final norm + LM head on the GPU's final hidden rows.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from oracle import transformer as T
from oracle.pagetable import PageTable
from workloads import WeightSource, hand_cost_model, make_batch

from gpu_util import (bf16_noise_floor_rms, decode_pages, kv_tolerance_ok, teacher_forced_layer_checks,
                      teacher_forced_samples)

pytestmark = pytest.mark.gpu

PREFIX = 576          # tokens the oracle prefills through all layers: past a 512-token scheduling
                      # chunk, nine 64-key attention tiles, into a fifth 128-row attention work item
CONST_LEN = 16384


@pytest.fixture(scope="module")
def env():
    import paper_2604_25080_amd as cf
    from paper_2604_25080_amd.runtime import Session
    b = make_batch("cfg2")
    shape = b.shape
    # request 8: a constant-token context of the maximum length of the configuration
    b.n_ctx.append(CONST_LEN)
    b.ctx_tokens.append(np.full(CONST_LEN, 4242, dtype=np.int32))
    b.n_new.append(128)
    b.new_tokens.append(b.new_tokens[0].copy())
    B = len(b.n_ctx)
    ws = WeightSource(shape, b.weight_seed, cache=True)
    pages = sum(-(-(n + m) // 16) for n, m in zip(b.n_ctx, b.n_new)) + 64
    sess = Session(shape, WeightSource(shape, b.weight_seed), max_batch=B, max_tokens=sum(b.n_ctx),
                   max_positions=max(b.n_ctx) + 128 + 16, n_pages=pages, gen_threads=16)
    opt = PageTable(pages)
    reqs = []
    for i in range(B):
        sess.cache.alloc(1 + i, b.n_ctx[i] + b.n_new[i])
        assert sess.cache.page_table(1 + i) == opt.alloc(1 + i, b.n_ctx[i] + b.n_new[i])
        reqs.append(dict(req_id=1 + i, ctx_tokens=b.ctx_tokens[i], new_tokens=b.new_tokens[i], host_kv=None))
    L = shape.n_layers
    # hidden rows entering every layer, sampled in the longest, the shortest and the first request
    picked = sorted({0, int(np.argmax(b.n_ctx[:8])), int(np.argmin(b.n_ctx[:8]))})
    rows, rows_req, rows_pos = teacher_forced_samples(b.n_ctx, picked)
    hid = torch.full((2 * L + 1, len(rows), shape.d_model), float("nan"), dtype=torch.float32, device="cuda")
    sess.ctx.capture_rows(rows, hid.data_ptr())
    sess.restore(reqs, [(0, n, L) for n in b.n_ctx], want_logits=False)       # full prefill on the GPU
    sess.teacher = (hid.cpu().numpy(), rows_req, rows_pos)
    del hid
    for i in range(B):
        reqs[i]["host_kv"] = sess.offload(1 + i, b.n_ctx[i])
    # oracle weights for all layers, generated in parallel (float32 upcast of the bf16 weights)
    with ThreadPoolExecutor(max_workers=8) as ex:
        list(ex.map(ws.layer_f32, range(L)))
    yield b, sess, reqs, ws
    sess.close()


def host_kv_of(sess, b, reqs, i):
    n = b.n_ctx[i]
    raw = reqs[i]["host_kv"].numpy()[:sess.host_kv_bytes(n)].reshape(b.shape.n_layers, -1, sess.page_bytes)
    return decode_pages(b.shape, raw, n)


def test_prefix_exactness_of_the_gpu_prefill(env):
    """K/V of the first PREFIX tokens through all 32 layers.  Layer 0 is held to the stated
    bound against the UNROUNDED oracle (2e-2, one bf16 ulp where an ulp exceeds it).  Deeper
    layers cannot be: at width 4096 the rounding of the tensors a bf16 model stores moves
    layer-1 cells by ~5e-2 on the CPU alone (tests/test_oracle_transformer.py shows it), and
    two correct bf16 pipelines decorrelate at the ulp level.  So from layer 1 on the GPU is
    held to the noise floor the arithmetic fixes: its distance to the unrounded oracle may not
    exceed that of the oracle's own bf16-storage forward on the same cells by more than 30 %
    in RMS and 60 % in maximum."""
    b, sess, reqs, ws = env
    L = b.shape.n_layers
    rows = []
    for i, P in ((0, PREFIX), (4, 192)):
        stored, _ = T.prefill(b.shape, ws, b.ctx_tokens[i][:P], dtype=np.float32, act="bf16")
        exact, _ = T.prefill(b.shape, ws, b.ctx_tokens[i][:P], dtype=np.float32)
        k, v = host_kv_of(sess, b, reqs, i)
        for l in range(L):
            for got, st, ex, nm in ((k[l, :P], stored.k[l], exact.k[l], "K"),
                                    (v[l, :P], stored.v[l], exact.v[l], "V")):
                ex = ex.astype(np.float64)
                e_gpu, e_ref = got - ex, st - ex
                rows.append((i, l, nm, float(np.sqrt(np.mean(e_gpu ** 2))), float(np.abs(e_gpu).max()),
                             float(np.sqrt(np.mean(e_ref ** 2))), float(np.abs(e_ref).max()),
                             float(ex.std())))
                if l == 0:
                    ok, w, _ = kv_tolerance_ok(b.shape, got, ex)
                    assert ok, f"request {i} layer 0 {nm}: max abs err {w} vs the unrounded oracle"
    print("req layer  gpu_rms  gpu_max  bf16cpu_rms bf16cpu_max  std")
    for (i, l, nm, gr, gm, rr, rm, sd) in rows:
        if l in (0, 1, 2, 7, 15, 23, 31):
            print(f"{i:3d} {l:3d} {nm}  {gr:.5f}  {gm:.5f}   {rr:.5f}    {rm:.5f}   {sd:.3f}")
    for (i, l, nm, gr, gm, rr, rm, sd) in rows:
        assert gr <= 1.3 * rr + 1e-4, f"request {i} layer {l} {nm}: rms {gr} vs noise floor {rr}"
        assert gm <= 1.6 * rm + 1e-3, f"request {i} layer {l} {nm}: max {gm} vs noise floor {rm}"


def test_teacher_forced_layer_checks_at_every_layer(env):
    """Element-wise parity at full size beyond layer 0: for ~65 sampled rows of three requests
    (first and last positions, page, work-item, chunk and workspace-chunk edges) and EVERY
    layer, the K/V cells against the unrounded oracle fed with the hidden rows the GPU fed that
    layer, at 2e-2 (one ulp where |ref| >= 4); and for every layer below the last, the layer's
    output rows -- oracle attention over the GPU's K/V cells of up to 14874 earlier positions,
    O-projection, SwiGLU MLP -- against the hidden rows the GPU fed the next layer."""
    b, sess, reqs, ws = env
    hid, rows_req, rows_pos = sess.teacher
    assert len(rows_req) >= 64
    st = teacher_forced_layer_checks(b.shape, ws, sess, b.n_ctx, [r["host_kv"] for r in reqs], hid, rows_req,
                                     rows_pos, out_layers=set(range(b.shape.n_layers)), label="cfg2")
    assert st["kv_cells"] == 32 * len(rows_req) * 2 * 8 * 128
    assert st["attention_elems"] == st["mlp_elems"] == 31 * len(rows_req) * 4096


def test_constant_token_request_matches_the_one_token_oracle(env):
    """A 16384-token context of one repeated token: V[l][t] = V[l][0] and K[l][t] = rope_t(K[l][0])
    at every layer, with K[l][0], V[l][0] from a ONE-token oracle forward.  Layer 0 to the stated
    bound; deeper layers to the bf16 noise floor (1.5x in RMS, 8x the RMS floor in maximum): a
    wrong mask, softmax normalisation, rotary angle or page slot shows up as an O(1) error."""
    b, sess, reqs, ws = env
    i = len(b.n_ctx) - 1
    kv1, _ = T.prefill(b.shape, ws, b.ctx_tokens[i][:1], dtype=np.float64)
    k, v = host_kv_of(sess, b, reqs, i)
    pos = np.array([0, 1, 15, 16, 255, 4095, 4096, 9999, 12345, CONST_LEN - 1])
    for l in range(b.shape.n_layers):
        k_ref = T.rope(np.repeat(kv1.k[l], len(pos), axis=0), pos, b.shape.rope_base)
        v_ref = np.repeat(kv1.v[l], len(pos), axis=0)
        floor = bf16_noise_floor_rms(l)
        for got, ref, nm in ((k[l, pos], k_ref, "K"), (v[l, pos], v_ref, "V")):
            err = got - ref
            if l == 0:
                ok, w, _ = kv_tolerance_ok(b.shape, got, ref)
                assert ok, f"layer 0 {nm}: max abs err {w}"
            rms, mx = float(np.sqrt(np.mean(err ** 2))), float(np.abs(err).max())
            assert rms <= 1.5 * floor and mx <= 8 * floor, f"layer {l} {nm}: rms {rms} max {mx} floor {floor}"
    # all positions carry the same V (up to the noise floor) on a dense sample of the last layer
    sample = np.arange(0, CONST_LEN, 97)
    assert np.abs(v[-1, sample] - v[-1, :1]).max() <= 8 * bf16_noise_floor_rms(b.shape.n_layers - 1)


def test_planner_hybrid_restore_matches_all_recompute_and_logits_match_oracle_head(env):
    import paper_2604_25080_amd as cf
    b, sess, reqs, ws = env
    shape, L, B = b.shape, b.shape.n_layers, len(b.n_ctx)
    cm = cf.cost_model(**hand_cost_model("startup"))
    opts = cf.plan_opts(b.chunk_tokens, 0, L, shape.kv_bytes_per_token_layer, cf.CF_TOKEN_WISE)
    splits, stats, _ = cf.restore_plan(cm, opts, b.n_ctx)
    assert any(0 < s[1] < n for s, n in zip(splits, b.n_ctx))
    sess.pool.fill_(0xFF)
    logits, tm = sess.restore(reqs, splits)
    for i in range(B):
        n = b.n_ctx[i]
        k, v = decode_pages(shape, sess.read_pages(1 + i, n), n)
        hk, hv = host_kv_of(sess, b, reqs, i)
        # loaded cells byte-identical; recomputed cells bit-identical to the all-recompute pass
        assert np.array_equal(k, hk) and np.array_equal(v, hv), f"request {i}"
    # logits: oracle final norm + LM head applied to the GPU's final hidden rows
    hid = sess.ctx.read_final_hidden(B)
    got = logits.cpu().numpy()
    for i in (0, B - 1):
        ref = T.logits_last(shape, ws, hid[i].astype(np.float64), act="bf16")
        err = np.abs(got[i] - ref).max()
        assert err <= 2e-2, f"request {i}: logits max abs err {err}"
    assert tm["loaded_cells"] + tm["recomputed_cells"] == sum(b.n_ctx) * L


def test_run_time_scheduled_restore_at_full_size(env):
    """cf_restore_dynamic on the same batch: whatever split results, loaded cells are the host
    block's bytes, recomputed cells (chunk by chunk, in steps) agree with the single-pass prefill
    that made the host block to within the bf16 noise floor of their layer (layer 0, which no
    attention feeds, to the stated bound), and the logits are the oracle head's on the final hidden rows."""
    import paper_2604_25080_amd as cf
    b, sess, reqs, ws = env
    shape, L, B = b.shape, b.shape.n_layers, len(b.n_ctx)
    cm = cf.cost_model(**hand_cost_model("startup"))
    opts = cf.plan_opts(b.chunk_tokens, 0, L, shape.kv_bytes_per_token_layer, cf.CF_TOKEN_WISE)
    static_splits, _, _ = cf.restore_plan(cm, opts, b.n_ctx)
    ref_logits = sess.restore(reqs, static_splits)[0].cpu().numpy().copy()
    sess.pool.fill_(0xFF)
    logits, splits, tm, st = sess.restore_dynamic(reqs, cm, opts)
    print("run-time splits", [s[1] for s in splits], "static", [s[1] for s in static_splits], st)
    assert tm["loaded_cells"] + tm["recomputed_cells"] == sum(b.n_ctx) * L
    assert any(s[1] > 0 for s in splits) and any(s[1] < n for s, n in zip(splits, b.n_ctx))
    for i in range(B):
        n, (mode, kk, cc) = b.n_ctx[i], splits[i]
        assert mode == cf.CF_TOKEN_WISE and cc == L and (kk % b.chunk_tokens == 0 or kk == n)
        k, v = decode_pages(shape, sess.read_pages(1 + i, n), n)
        hk, hv = host_kv_of(sess, b, reqs, i)
        assert np.isfinite(k).all() and np.isfinite(v).all(), f"request {i}: unwritten slot"
        assert np.array_equal(k[:, kk:], hk[:, kk:]) and np.array_equal(v[:, kk:], hv[:, kk:]), f"request {i}"
        if kk == 0:
            continue
        for got, ref, nm in ((k[:, :kk], hk[:, :kk], "K"), (v[:, :kk], hv[:, :kk], "V")):
            ok, w, _ = kv_tolerance_ok(shape, got[0], ref[0])
            assert ok, f"request {i} layer 0 {nm}: {w}"
            for l in range(1, L):
                rms = float(np.sqrt(np.mean((got[l] - ref[l]) ** 2)))
                assert rms <= 2.0 * bf16_noise_floor_rms(l), f"request {i} layer {l} {nm}: rms {rms}"
    # logits: the oracle's final norm + LM head on the final hidden rows this call left behind.
    # (Against the planned restore's logits only a noise-floor statement could be made: the two
    # recompute different token sets in different summation orders.)
    hid = sess.ctx.read_final_hidden(B)
    out = logits.cpu().numpy()
    for i in (0, B - 1):
        ref = T.logits_last(shape, ws, hid[i].astype(np.float64), act="bf16")
        err = np.abs(out[i] - ref).max()
        assert err <= 2e-2, f"request {i}: logits max abs err {err}"
    print("logits: max abs difference to the planned restore (not asserted)", np.abs(out - ref_logits).max())
