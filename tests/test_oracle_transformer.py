"""Pins for oracle/transformer.py: closed forms, invariants the method fixes
(Sec. 1 (i)-(ii), Sec. 3.1), and a library cross-check.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import transformer as T
from workloads import SHAPES, ModelShape, WeightSource, make_batch

TINY = SHAPES["tiny"]


def small_shape(**kw):
    base = dict(name="s", n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2,
                head_dim=8, d_ffn=48, vocab=50, rope_base=10000.0,
                rms_eps=1e-5, dtype="f32")
    base.update(kw)
    return ModelShape(**base)


# ---------------------------------------------------------------- closed forms
def test_rmsnorm_constant_vector():
    c, d, eps = 3.0, 16, 1e-5
    x = np.full((2, d), c)
    g = np.linspace(0.5, 2.0, d)
    out = T.rmsnorm(x, g, eps)
    np.testing.assert_allclose(out, np.broadcast_to(c / np.sqrt(c * c + eps) * g, (2, d)),
                               rtol=1e-14)


def test_rmsnorm_is_scale_invariant_and_unit_rms():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(5, 64))
    a = T.rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.sqrt(np.mean(a * a, -1)), 1.0, rtol=1e-13)
    np.testing.assert_allclose(T.rmsnorm(7.0 * x, np.ones(64), 0.0), a, rtol=1e-13)


def test_rope_position_zero_is_identity():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(1, 3, 8))
    np.testing.assert_array_equal(T.rope(x, [0], 10000.0), x)


def test_rope_hand_values_fix_pairing_and_sign():
    # head_dim 4: pairs (0,2) with theta=1 and (1,3) with theta=base^(-1/2).
    base, p = 100.0, 3
    x = np.array([[[1.0, 0.0, 0.0, 2.0]]])
    y = T.rope(x, [p], base)[0, 0]
    th1 = p * base ** -0.5
    # (x0,x2)=(1,0) -> (cos p, sin p); (x1,x3)=(0,2) -> (-2 sin th1, 2 cos th1)
    np.testing.assert_allclose(y, [np.cos(p), -2 * np.sin(th1), np.sin(p), 2 * np.cos(th1)],
                               rtol=1e-14)


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(2)
    q = rng.normal(size=(1, 1, 16))
    k = rng.normal(size=(1, 1, 16))
    ref = None
    for m, n in ((5, 2), (105, 102), (131071, 131068)):
        s = np.sum(T.rope(q, [m], 500000.0) * T.rope(k, [n], 500000.0))
        ref = s if ref is None else ref
        np.testing.assert_allclose(s, ref, rtol=1e-9)
    # and it is not position-independent
    assert abs(np.sum(T.rope(q, [5], 500000.0) * T.rope(k, [4], 500000.0)) - ref) > 1e-6


def test_silu_closed_forms():
    x = np.array([-3.0, -1.0, 0.0, 0.5, 4.0])
    np.testing.assert_allclose(T.silu(x) - T.silu(-x), x, rtol=1e-14, atol=1e-15)
    assert T.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(T.silu(np.array([1.0]))[0], 1.0 / (1.0 + np.exp(-1.0)))


def test_attention_zero_query_gives_running_mean_and_gqa_mapping():
    rng = np.random.default_rng(3)
    tq, hq, hkv, hd = 6, 4, 2, 8
    q = np.zeros((tq, hq, hd))
    k = rng.normal(size=(tq, hkv, hd))
    v = rng.normal(size=(tq, hkv, hd))
    out = T.causal_attention(q, k, v, np.arange(tq))
    for t in range(tq):
        for h in range(hq):
            np.testing.assert_allclose(out[t, h], v[:t + 1, h // 2].mean(0), rtol=1e-13)


def test_attention_peaked_scores_select_one_key():
    # huge aligned query picks the matching *visible* key: pins mask direction and scale sign
    hd = 4
    k = np.eye(4)[:, None, :]                       # key t = e_t
    v = np.arange(16.0).reshape(4, 1, 4)
    q = 1e4 * np.eye(4)[[3, 1, 2, 0]][:, None, :]   # query t wants key [3,1,2,0][t]
    out = T.causal_attention(q, k, v, np.arange(4))
    # t=0 wants key 3 (invisible): only key 0 visible -> v[0]
    np.testing.assert_allclose(out[0, 0], v[0, 0])
    np.testing.assert_allclose(out[1, 0], v[1, 0])
    np.testing.assert_allclose(out[2, 0], v[2, 0])
    np.testing.assert_allclose(out[3, 0], v[0, 0])


def test_attention_matches_torch_sdpa():
    rng = np.random.default_rng(4)
    tq, hq, hkv, hd = 33, 8, 2, 16
    q = rng.normal(size=(tq, hq, hd))
    k = rng.normal(size=(tq, hkv, hd))
    v = rng.normal(size=(tq, hkv, hd))
    ours = T.causal_attention(q, k, v, np.arange(tq))
    tq_, tk_, tv_ = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    tk_ = tk_.repeat_interleave(hq // hkv, dim=1)
    tv_ = tv_.repeat_interleave(hq // hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq_, tk_, tv_, is_causal=True)
    np.testing.assert_allclose(ours, ref[0].permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


def test_kv_size_formula_matches_the_paper_example():
    # Sec. 2: 2*L*H*d*N elements; the paper states the resulting size for a named model
    # (tests/golden/kv_size_examples.txt); the formula must land on it to the stated digits.
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "kv_size_examples.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert rows
    for name, layers, kvh, hd, eb, toks, gb in rows:
        n_bytes = 2 * int(layers) * int(kvh) * int(hd) * int(toks) * int(eb)
        # "GB" read as 10^9 or 2^30 bytes, whichever the authors meant
        assert min(abs(n_bytes / 1e9 - float(gb)), abs(n_bytes / 2 ** 30 - float(gb))) <= 0.1, (name, n_bytes)
    s = SHAPES["8b"]
    assert s.kv_bytes_per_token_layer * s.n_layers == 2 * s.n_layers * s.n_kv_heads * s.head_dim * 2


# ---------------------------------------------------- independent formulations
def torch_forward(shape, ws, tokens):
    """Same model written with torch library ops and complex-number RoPE."""
    s = shape
    dt = torch.float64
    h = torch.from_numpy(ws.f32("embed")).to(dt)[torch.as_tensor(np.asarray(tokens, dtype=np.int64))]
    t = h.shape[0]
    pos = torch.arange(t, dtype=dt)
    theta = torch.tensor(s.rope_base, dtype=dt) ** (-torch.arange(0, s.head_dim, 2, dtype=dt) / s.head_dim)
    rot = torch.polar(torch.ones(t, s.head_dim // 2, dtype=dt), pos[:, None] * theta[None])

    def rope_c(x):  # x [T,H,hd]; pairs (j, j+hd/2)
        half = s.head_dim // 2
        z = torch.complex(x[..., :half], x[..., half:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    ks, vs = [], []
    for l in range(s.n_layers):
        lw = {n: torch.from_numpy(w).to(dt) for n, w in ws.layer_f32(l).items()}
        a = torch.nn.functional.rms_norm(h, (s.d_model,), eps=s.rms_eps)
        qkv = torch.nn.functional.linear(a, lw["wqkv"])
        nq, nk = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
        q = rope_c(qkv[:, :nq].reshape(t, s.n_q_heads, s.head_dim))
        k = rope_c(qkv[:, nq:nq + nk].reshape(t, s.n_kv_heads, s.head_dim))
        v = qkv[:, nq + nk:].reshape(t, s.n_kv_heads, s.head_dim)
        ks.append(k.numpy()); vs.append(v.numpy())
        g = s.n_q_heads // s.n_kv_heads
        o = torch.nn.functional.scaled_dot_product_attention(
            q.permute(1, 0, 2)[None], k.permute(1, 0, 2).repeat_interleave(g, 0)[None],
            v.permute(1, 0, 2).repeat_interleave(g, 0)[None], is_causal=True)[0]
        h = h + torch.nn.functional.linear(o.permute(1, 0, 2).reshape(t, nq), lw["wo"])
        u = torch.nn.functional.rms_norm(h, (s.d_model,), eps=s.rms_eps)
        h = h + torch.nn.functional.linear(
            torch.nn.functional.silu(torch.nn.functional.linear(u, lw["w_gate"])) *
            torch.nn.functional.linear(u, lw["w_up"]), lw["w_down"])
    a = torch.nn.functional.rms_norm(h[-1:], (s.d_model,), eps=s.rms_eps)
    logits = torch.nn.functional.linear(a, torch.from_numpy(ws.f32("lm_head")).to(dt))[0]
    return ks, vs, logits.numpy()


@pytest.mark.parametrize("shape", [small_shape(), small_shape(n_kv_heads=4), TINY])
def test_forward_matches_torch_library_formulation(shape):
    ws = WeightSource(shape, 11, cache=True)
    rng = np.random.default_rng(5)
    toks = rng.integers(0, shape.vocab, size=37)
    kv, h = T.prefill(shape, ws, toks)
    logits = T.logits_last(shape, ws, h[-1])
    ks, vs, ref_logits = torch_forward(shape, ws, toks)
    for l in range(shape.n_layers):
        np.testing.assert_allclose(kv.k[l], ks[l], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(kv.v[l], vs[l], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(logits, ref_logits, rtol=1e-9, atol=1e-11)


def test_token_by_token_decode_equals_batched_prefill():
    shape = small_shape()
    ws = WeightSource(shape, 12, cache=True)
    toks = np.random.default_rng(6).integers(0, shape.vocab, size=19)
    kv_b, h_b = T.prefill(shape, ws, toks)
    cache = T.KVCache(shape.n_layers)
    for l in range(shape.n_layers):
        cache.k[l] = np.zeros((0, shape.n_kv_heads, shape.head_dim))
        cache.v[l] = np.zeros((0, shape.n_kv_heads, shape.head_dim))
    for t in range(len(toks)):
        kv1, h1 = T.prefill(shape, ws, toks[t:t + 1], past=cache)
        for l in range(shape.n_layers):
            cache.k[l] = np.concatenate([cache.k[l], kv1.k[l]])
            cache.v[l] = np.concatenate([cache.v[l], kv1.v[l]])
    for l in range(shape.n_layers):
        np.testing.assert_allclose(cache.k[l], kv_b.k[l], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(cache.v[l], kv_b.v[l], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(h1[0], h_b[-1], rtol=1e-10, atol=1e-12)


# ------------------------------------------- invariants of hybrid restoration
def test_I1_restore_equals_full_prefill_for_every_split_and_cut():
    shape = small_shape(n_layers=3)
    ws = WeightSource(shape, 13, cache=True)
    toks = np.random.default_rng(7).integers(0, shape.vocab, size=21)
    kv_full, _ = T.prefill(shape, ws, toks)
    for k in range(len(toks) + 1):
        for c in range(shape.n_layers + 1):
            r = T.restore(shape, ws, toks, kv_full, k, c)
            for l in range(shape.n_layers):
                np.testing.assert_allclose(r.k[l], kv_full.k[l], rtol=1e-10, atol=1e-12)
                np.testing.assert_allclose(r.v[l], kv_full.v[l], rtol=1e-10, atol=1e-12)


def test_I1_special_cases_all_load_is_a_copy_and_all_recompute_is_prefill():
    shape = small_shape()
    ws = WeightSource(shape, 14, cache=True)
    toks = np.random.default_rng(8).integers(0, shape.vocab, size=20)
    kv_full, _ = T.prefill(shape, ws, toks)
    # k=0: pure copy, even of garbage (nothing is recomputed)
    junk = kv_full.copy()
    for l in range(shape.n_layers):
        junk.k[l] = junk.k[l] + 100.0
    r = T.restore(shape, ws, toks, junk, 0, shape.n_layers)
    for l in range(shape.n_layers):
        np.testing.assert_array_equal(r.k[l], junk.k[l])
    # k=n, c=L: nothing is read from the store
    r = T.restore(shape, ws, toks, junk, len(toks), shape.n_layers)
    for l in range(shape.n_layers):
        np.testing.assert_allclose(r.k[l], kv_full.k[l], rtol=1e-10, atol=1e-12)


def test_I2_recomputed_prefix_never_reads_tokens_past_the_split():
    shape = small_shape()
    ws = WeightSource(shape, 15, cache=True)
    rng = np.random.default_rng(9)
    toks = rng.integers(0, shape.vocab, size=24)
    k = 10
    kv_a, _ = T.prefill(shape, ws, toks)
    poisoned = toks.copy()
    poisoned[k:] = (poisoned[k:] + 17) % shape.vocab
    kv_b, _ = T.prefill(shape, ws, poisoned)
    for l in range(shape.n_layers):
        np.testing.assert_array_equal(kv_a.k[l][:k], kv_b.k[l][:k])
        np.testing.assert_array_equal(kv_a.v[l][:k], kv_b.v[l][:k])
        if l > 0:       # layer 0 K/V of a token depend on that token alone
            assert not np.allclose(kv_a.k[l][k:], kv_b.k[l][k:])


def test_I3_logits_after_restore_equal_full_prefill_logits_cfg1():
    b = make_batch("cfg1")
    shape = b.shape
    ws = WeightSource(shape, b.weight_seed, cache=True)
    for i in range(len(b.n_ctx)):
        kv_ctx, kv_new, logits = T.full_reference(shape, ws, b.ctx_tokens[i], b.new_tokens[i])
        whole, h = T.prefill(shape, ws, np.concatenate([b.ctx_tokens[i], b.new_tokens[i]]))
        np.testing.assert_allclose(T.logits_last(shape, ws, h[-1]), logits, rtol=1e-9, atol=1e-11)
        k, c = b.forced_splits[i]
        r = T.restore(shape, ws, b.ctx_tokens[i], kv_ctx, k, c)
        lg, _ = T.first_token_logits(shape, ws, r, b.new_tokens[i])
        np.testing.assert_allclose(lg, logits, rtol=1e-9, atol=1e-11)


def test_float32_mode_tracks_float64():
    b = make_batch("cfg1")
    ws = WeightSource(b.shape, b.weight_seed, cache=True)
    kv64, _ = T.prefill(b.shape, ws, b.ctx_tokens[1])
    kv32, _ = T.prefill(b.shape, ws, b.ctx_tokens[1], dtype=np.float32)
    assert kv32.k[1].dtype == np.float32
    np.testing.assert_allclose(kv32.k[1], kv64.k[1], atol=2e-5)


def test_teacher_forced_rows_match_full_layer():
    shape = small_shape()
    ws = WeightSource(shape, 16, cache=True)
    toks = np.random.default_rng(10).integers(0, shape.vocab, size=18)
    kv, h_out, h_in = T.prefill(shape, ws, toks, return_hidden=True)
    rows = np.array([0, 7, 17])
    l = 1
    kr, vr, hr = T.layer_rows_teacher_forced(shape, ws.layer_f32(l), ws.norm_gain(),
                                             h_in[l][rows], rows, kv.k[l], kv.v[l])
    np.testing.assert_allclose(kr, kv.k[l][rows], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(vr, kv.v[l][rows], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(hr, h_out[rows], rtol=1e-10, atol=1e-12)
    # the two halves on their own: with a zero down-projection a layer's output IS the residual
    # stream after its attention half, and the MLP half of that stream is what the full layer adds
    lw0 = dict(ws.layer_f32(l))
    lw0["w_down"] = np.zeros_like(lw0["w_down"])
    h_mid_full, _, _ = T.layer_forward(shape, lw0, ws.norm_gain(), h_in[l], np.arange(len(toks)), None, None)
    _, _, h_mid = T.attention_rows_teacher_forced(shape, ws.layer_f32(l), ws.norm_gain(), h_in[l][rows], rows,
                                                  kv.k[l], kv.v[l])
    np.testing.assert_allclose(h_mid, h_mid_full[rows], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(T.mlp_rows(shape, ws.layer_f32(l), ws.norm_gain(), h_mid_full[rows]), h_out[rows],
                               rtol=1e-10, atol=1e-12)
    assert np.abs(h_mid - h_out[rows]).max() > 1e-3          # the MLP half is not a no-op here
    # the K/V-only form agrees with the full prefill at every layer (not with itself: the
    # prefill computes the cells inside layer_forward, batched over all tokens)
    for l in range(shape.n_layers):
        k2, v2 = T.kv_rows_teacher_forced(shape, ws.layer_f32(l), ws.norm_gain(), h_in[l][rows], rows)
        np.testing.assert_allclose(k2, kv.k[l][rows], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(v2, kv.v[l][rows], rtol=1e-10, atol=1e-12)


def test_kv_to_pages_layout():
    shape = small_shape()
    n = 37
    cache = T.KVCache(shape.n_layers)
    for l in range(shape.n_layers):
        idx = np.arange(n)[:, None, None] * 1000 + np.arange(shape.n_kv_heads)[None, :, None] * 10 \
            + np.arange(shape.head_dim)[None, None, :] * 0.01 + l * 100000
        cache.k[l] = idx.astype(np.float64)
        cache.v[l] = -idx.astype(np.float64)
    pages = T.kv_to_pages(shape, cache, n)
    hk, hd = shape.n_kv_heads, shape.head_dim
    assert pages.shape == (shape.n_layers, 3, 2 * hk * 16 * hd)
    for (l, t, g, j) in ((0, 0, 0, 0), (1, 17, 1, 3), (1, 36, 0, 7)):
        pg, sl = t // 16, t % 16
        assert pages[l, pg, (g * 16 + sl) * hd + j] == np.float32(cache.k[l][t, g, j])
        assert pages[l, pg, hk * 16 * hd + (g * hd + j) * 16 + sl] == np.float32(cache.v[l][t, g, j])
    kpart = pages[:, 2, :hk * 16 * hd].reshape(shape.n_layers, hk, 16, hd)
    vpart = pages[:, 2, hk * 16 * hd:].reshape(shape.n_layers, hk, hd, 16)
    assert np.all(kpart[:, :, 5:, :] == 0) and np.all(vpart[:, :, :, 5:] == 0)


# ----------------------------------------------------------- bf16 storage mode
def test_round_bf16_is_nearest_even_on_hand_values():
    # bf16 keeps 8 significand bits: spacing 2^-7 in [1,2)
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -7, -2.5 - 2.0 ** -7, 3.14159])
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -2.5, 3.140625])
    np.testing.assert_array_equal(T.round_bf16(x), want)
    rng = np.random.default_rng(11)
    y = rng.normal(size=1000) * 5
    r = T.round_bf16(y)
    assert np.all(np.abs(r - y) <= np.abs(y) * 2.0 ** -8)           # half an ulp at most
    np.testing.assert_array_equal(T.round_bf16(r), r)               # idempotent
    np.testing.assert_array_equal(r, torch.from_numpy(y).to(torch.bfloat16).to(torch.float64).numpy())


def test_bf16_storage_mode_keeps_the_restore_invariant_and_stays_near_exact():
    shape = small_shape(n_layers=3)
    ws = WeightSource(shape, 17, cache=True)
    toks = np.random.default_rng(12).integers(0, shape.vocab, size=20)
    kv_full, _ = T.prefill(shape, ws, toks, act="bf16")
    for l in range(shape.n_layers):       # cache cells are bf16 codes
        np.testing.assert_array_equal(T.round_bf16(kv_full.k[l]), kv_full.k[l])
        np.testing.assert_array_equal(T.round_bf16(kv_full.v[l]), kv_full.v[l])
    for k, c in ((0, 3), (7, 3), (20, 2), (13, 1)):
        r = T.restore(shape, ws, toks, kv_full, k, c, act="bf16")
        for l in range(shape.n_layers):
            np.testing.assert_array_equal(r.k[l], kv_full.k[l])     # same rounding, same codes
            np.testing.assert_array_equal(r.v[l], kv_full.v[l])
    exact, _ = T.prefill(shape, ws, toks)
    assert np.abs(exact.k[2] - kv_full.k[2]).max() < 0.05 * np.abs(exact.k[2]).max()


def test_bf16_storage_alone_moves_kv_by_more_than_2e_2_at_width_4096():
    # Why the bf16 configurations are compared with the bf16-storage forward: at d_model 4096
    # with N(0, 0.02) weights the K/V entries have std ~1.3, and rounding the tensors a bf16
    # model stores (no kernel involved, pure CPU) already shifts layer-1 cells by more than
    # the 2e-2 the unrounded forward would have to be matched to.
    shape = ModelShape("wide", 2, 4096, 8, 2, 128, 1024, 64, 500000.0, 1e-5, "bf16")
    ws = WeightSource(shape, 18, cache=True)
    toks = np.random.default_rng(13).integers(0, shape.vocab, size=32)
    exact, _ = T.prefill(shape, ws, toks, dtype=np.float32)
    stored, _ = T.prefill(shape, ws, toks, dtype=np.float32, act="bf16")
    assert 1.0 < exact.k[1].std() < 1.6
    assert np.abs(stored.k[1] - exact.k[1]).max() > 2e-2
    assert np.abs(stored.k[1] - exact.k[1]).max() < 0.2          # ... but it is rounding, not a bug


def test_stage_restore_from_boundary_activations_equals_full_prefill():
    """Sec. 3.2: a pipeline stage restores its own layers from the hidden states entering its
    first layer, with nothing from the stages below.  For every stage of a 3-layer model and
    every (k, cut) the stage's cells equal the full prefill; stage [0, L) from the embeddings is
    plain restore; the stages together tile the model (Eq. 2 divides the work by S)."""
    shape = SHAPES["mini-bf16"].with_layers(3).with_vocab(300)
    ws = WeightSource(shape, 77, cache=True)
    rng = np.random.default_rng(5)
    toks = rng.integers(0, 300, size=40).astype(np.int32)
    full, _, hidden_in = T.prefill(shape, ws, toks, return_hidden=True)
    assert np.array_equal(hidden_in[0], T.embed(ws, toks))
    for b, e in ((0, 3), (0, 1), (1, 3), (1, 2), (2, 3)):
        for k in (0, 1, 17, 40):
            for cut in range(0, e - b + 1):
                # poison what a correct stage restore must overwrite
                stored = full.copy()
                for l in range(b, b + cut):
                    stored.k[l][:k] = np.nan
                    stored.v[l][:k] = np.nan
                got = T.restore_stage(shape, ws, hidden_in[b], stored, k, cut, b, e, len(toks))
                for l in range(shape.n_layers):
                    if b <= l < e:
                        assert np.abs(got.k[l] - full.k[l]).max() <= 1e-10
                        assert np.abs(got.v[l] - full.v[l]).max() <= 1e-10
                    else:
                        assert got.k[l] is None and got.v[l] is None
    plain = T.restore(shape, ws, toks, full, 17, 2)
    staged = T.restore_stage(shape, ws, T.embed(ws, toks), full, 17, 2, 0, 3, len(toks))
    for l in range(3):
        assert np.array_equal(plain.k[l], staged.k[l]) and np.array_equal(plain.v[l], staged.v[l])
