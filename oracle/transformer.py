"""Oracle: decoder-only transformer forward and hybrid-restore semantics.

TEST INFRASTRUCTURE ONLY (see package docstring).

The method is exact: a KV cache restored partly by recomputation and partly by
loading must equal the cache a full prefill produces, because token t's state
depends only on tokens <= t (causal dependency) and layer l's only on layers
< l (feed-forward dependency) -- Sec. 1 items (i)-(ii), Sec. 3.1.  The oracle
is therefore the plain definition of the forward pass, written out with numpy
matmuls and no blocking or fusion.

Model family (Sec. 4.1 names Llama-3.1-8B / Qwen3-8B; widths come from the
benchmark configurations): pre-norm decoder, RMSNorm with unit-initialised
gain, rotary position embedding in the rotate-half pairing (j, j + hd/2) with
theta_j = base^(-2j/hd) and absolute positions, grouped-query attention where
Q head j reads KV head j // (Hq/Hkv), SwiGLU MLP, no biases, untied LM head.

All arithmetic runs in `dtype` (float64 by default; float32 on request for the
timed baseline).  Rotary angles are always formed in float64.

Storage precision.  With act="exact" (default) nothing is rounded: this is the
reference the method's exactness is stated against.  With act="bf16" the
forward is that of a bf16 MODEL: every tensor such a model stores in 16 bits
is rounded to bf16 (nearest-even) where it is stored -- the normalised
activations fed to the projections, Q, K and V after the rotary turn (K and V
are the cache cells), the attention probabilities fed to the value product,
the attention output and the MLP activation -- while the residual stream,
norms, softmax and all accumulation stay in `dtype`.  A cache cell is a 16-bit
code; comparing codes needs both sides to round at the same places.
"""
import numpy as np


def round_bf16(x):
    """Nearest-even rounding to bf16, returned in x's float type."""
    x = np.asarray(x)
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = (u + (((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(x.dtype if x.dtype.kind == "f" else np.float64)


def _store(x, act):
    return round_bf16(x) if act == "bf16" else x


def rmsnorm(x, gain, eps, dtype=np.float64):
    """x * rsqrt(mean(x^2) + eps) * gain, row-wise."""
    x = np.asarray(x, dtype=dtype)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + dtype(eps)) * np.asarray(gain, dtype=dtype)


def rope_angles(positions, head_dim, base):
    """cos, sin of pos * base^(-2j/hd), j in [0, hd/2); float64."""
    j = np.arange(head_dim // 2, dtype=np.float64)
    theta = np.float64(base) ** (-2.0 * j / np.float64(head_dim))
    ang = np.asarray(positions, dtype=np.float64)[:, None] * theta[None, :]
    return np.cos(ang), np.sin(ang)


def rope(x, positions, base, dtype=np.float64):
    """Rotate x[T, H, hd]: pair (j, j+hd/2) turns by angle pos*theta_j."""
    x = np.asarray(x, dtype=dtype)
    hd = x.shape[-1]
    half = hd // 2
    cos, sin = rope_angles(positions, hd, base)
    cos = cos.astype(dtype)[:, None, :]
    sin = sin.astype(dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def causal_attention(q, k, v, q_pos, dtype=np.float64, act="exact"):
    """q[Tq,Hq,hd] at absolute positions q_pos[Tq]; k, v [Tk,Hkv,hd] hold
    positions 0..Tk-1.  Query at position p sees keys 0..p."""
    q = np.asarray(q, dtype=dtype)
    k = np.asarray(k, dtype=dtype)
    v = np.asarray(v, dtype=dtype)
    tq, hq, hd = q.shape
    tk, hkv, _ = k.shape
    group = hq // hkv
    scale = dtype(1.0) / np.sqrt(dtype(hd))
    visible = np.arange(tk)[None, :] <= np.asarray(q_pos)[:, None]
    out = np.empty((tq, hq, hd), dtype=dtype)
    for h in range(hq):
        g = h // group
        s = (q[:, h, :] @ k[:, g, :].T) * scale
        s = np.where(visible, s, -np.inf)
        s = s - np.max(s, axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / np.sum(p, axis=-1, keepdims=True)
        out[:, h, :] = _store(p, act) @ v[:, g, :]
    return out


class KVCache:
    """Per-layer K and V, [n_layers][T, Hkv, hd], unrounded."""

    def __init__(self, n_layers):
        self.k = [None] * n_layers
        self.v = [None] * n_layers

    def copy(self):
        c = KVCache(len(self.k))
        c.k = [None if a is None else a.copy() for a in self.k]
        c.v = [None if a is None else a.copy() for a in self.v]
        return c

    def n_tokens(self, layer=0):
        return 0 if self.k[layer] is None else self.k[layer].shape[0]


def embed(weights, tokens, dtype=np.float64):
    e = weights.f32("embed")
    return e[np.asarray(tokens, dtype=np.int64)].astype(dtype)


def layer_forward(shape, lw, gain, h, positions, k_past, v_past,
                  dtype=np.float64, act="exact"):
    """One decoder layer over rows h[T, d] at `positions`, attending to the
    given past K/V (positions 0..P-1, contiguous, P == positions[0]) followed
    by the rows' own K/V.  Returns (h_out, k_new, v_new)."""
    s = shape
    t = h.shape[0]
    a = _store(rmsnorm(h, gain, s.rms_eps, dtype), act)
    qkv = a @ lw["wqkv"].astype(dtype).T
    nq = s.n_q_heads * s.head_dim
    nk = s.n_kv_heads * s.head_dim
    q = qkv[:, :nq].reshape(t, s.n_q_heads, s.head_dim)
    k = qkv[:, nq:nq + nk].reshape(t, s.n_kv_heads, s.head_dim)
    v = _store(qkv[:, nq + nk:].reshape(t, s.n_kv_heads, s.head_dim), act)
    q = _store(rope(q, positions, s.rope_base, dtype), act)
    k = _store(rope(k, positions, s.rope_base, dtype), act)
    if k_past is not None and k_past.shape[0] > 0:
        k_all = np.concatenate([np.asarray(k_past, dtype=dtype), k], axis=0)
        v_all = np.concatenate([np.asarray(v_past, dtype=dtype), v], axis=0)
    else:
        k_all, v_all = k, v
    o = _store(causal_attention(q, k_all, v_all, positions, dtype, act), act)
    h = h + o.reshape(t, nq) @ lw["wo"].astype(dtype).T
    u = _store(rmsnorm(h, gain, s.rms_eps, dtype), act)
    gate = u @ lw["w_gate"].astype(dtype).T
    up = u @ lw["w_up"].astype(dtype).T
    h = h + _store(silu(gate) * up, act) @ lw["w_down"].astype(dtype).T
    return h, k, v


def prefill(shape, weights, tokens, past=None, n_layers=None,
            dtype=np.float64, return_hidden=False, act="exact"):
    """Run `tokens` (positions P..P+T-1 where P = tokens already in `past`)
    through layers [0, n_layers).  Returns (KVCache of the new rows' K/V for
    those layers, final hidden rows h[T, d])."""
    n_layers = shape.n_layers if n_layers is None else n_layers
    t = len(tokens)
    p0 = 0 if past is None else past.n_tokens(0)
    positions = np.arange(p0, p0 + t)
    gain = weights.norm_gain()
    h = embed(weights, tokens, dtype)
    out = KVCache(shape.n_layers)
    hidden_in = []
    for l in range(n_layers):
        if return_hidden:
            hidden_in.append(h.copy())
        lw = weights.layer_f32(l)
        kp = None if past is None else past.k[l]
        vp = None if past is None else past.v[l]
        h, k, v = layer_forward(shape, lw, gain, h, positions, kp, vp, dtype, act)
        out.k[l], out.v[l] = k, v
    if return_hidden:
        return out, h, hidden_in
    return out, h


def logits_last(shape, weights, h_last, dtype=np.float64, act="exact"):
    """Final RMSNorm and LM head on one hidden row."""
    a = _store(rmsnorm(h_last[None, :], weights.norm_gain(), shape.rms_eps, dtype), act)
    return (a @ weights.f32("lm_head").astype(dtype).T)[0]


def restore(shape, weights, ctx_tokens, kv_full, k_tokens, layer_cut,
            dtype=np.float64, act="exact"):
    """Hybrid restoration of one request (Sec. 3.1): cells (token < k_tokens,
    layer < layer_cut) are recomputed from the first k_tokens tokens alone;
    every other cell is taken from the stored cache `kv_full`."""
    n = len(ctx_tokens)
    assert 0 <= k_tokens <= n and 0 <= layer_cut <= shape.n_layers
    cache = KVCache(shape.n_layers)
    for l in range(shape.n_layers):
        cache.k[l] = np.array(kv_full.k[l][:n], dtype=dtype, copy=True)
        cache.v[l] = np.array(kv_full.v[l][:n], dtype=dtype, copy=True)
    if k_tokens > 0 and layer_cut > 0:
        rec, _ = prefill(shape, weights, ctx_tokens[:k_tokens],
                         n_layers=layer_cut, dtype=dtype, act=act)
        for l in range(layer_cut):
            cache.k[l][:k_tokens] = rec.k[l]
            cache.v[l][:k_tokens] = rec.v[l]
    return cache


def restore_stage(shape, weights, boundary_h, kv_full, k_tokens, layer_cut,
                  layer_begin, layer_end, n_tokens, dtype=np.float64, act="exact"):
    """Restoration of ONE pipeline stage's layers [layer_begin, layer_end) of a
    request (Sec. 3.2): the stage holds the hidden states entering its first
    layer ("boundary activations", boundary_h[n, d]) and recomputes cells
    (token < k_tokens, layer_begin <= layer < layer_begin + layer_cut) from the
    first k_tokens rows of them, with no input from any other stage; every
    other cell of the stage is taken from the stored cache.  Layers outside
    the stage are left as None.  layer_begin = 0 with boundary_h = the token
    embeddings is plain `restore`."""
    assert 0 <= layer_begin < layer_end <= shape.n_layers
    assert 0 <= k_tokens <= n_tokens and 0 <= layer_cut <= layer_end - layer_begin
    cache = KVCache(shape.n_layers)
    for l in range(layer_begin, layer_end):
        cache.k[l] = np.array(kv_full.k[l][:n_tokens], dtype=dtype, copy=True)
        cache.v[l] = np.array(kv_full.v[l][:n_tokens], dtype=dtype, copy=True)
    if k_tokens > 0 and layer_cut > 0:
        h = np.asarray(boundary_h[:k_tokens], dtype=dtype)
        positions = np.arange(k_tokens)
        gain = weights.norm_gain()
        for l in range(layer_begin, layer_begin + layer_cut):
            h, k, v = layer_forward(shape, weights.layer_f32(l), gain, h, positions, None, None, dtype, act)
            cache.k[l][:k_tokens] = k
            cache.v[l][:k_tokens] = v
    return cache


def first_token_logits(shape, weights, cache, new_tokens, dtype=np.float64, act="exact"):
    """Prefill the new-turn tokens over a restored cache; return (logits at
    the last new token, KVCache of the new tokens' own K/V)."""
    kv_new, h = prefill(shape, weights, new_tokens, past=cache, dtype=dtype, act=act)
    return logits_last(shape, weights, h[-1], dtype, act), kv_new


def full_reference(shape, weights, ctx_tokens, new_tokens, dtype=np.float64, act="exact"):
    """Full prefill of context then new tokens: (kv_ctx, kv_new, logits)."""
    kv_ctx, _ = prefill(shape, weights, ctx_tokens, dtype=dtype, act=act)
    logits, kv_new = first_token_logits(shape, weights, kv_ctx, new_tokens, dtype, act)
    return kv_ctx, kv_new, logits


def attention_rows_teacher_forced(shape, lw, gain, h_rows, positions, k_cache,
                                  v_cache, dtype=np.float64):
    """Attention half of one layer on a few sampled rows: given the rows' input
    hidden states and the layer's K/V cache for positions 0..max(positions)
    (which must already include the rows' own K/V), return (k_rows, v_rows,
    h_mid_rows) with h_mid = h + attention(h) W_o, the residual stream that
    enters the MLP half."""
    s = shape
    t = h_rows.shape[0]
    a = rmsnorm(h_rows, gain, s.rms_eps, dtype)
    qkv = a @ lw["wqkv"].astype(dtype).T
    nq = s.n_q_heads * s.head_dim
    nk = s.n_kv_heads * s.head_dim
    q = rope(qkv[:, :nq].reshape(t, s.n_q_heads, s.head_dim), positions,
             s.rope_base, dtype)
    k = rope(qkv[:, nq:nq + nk].reshape(t, s.n_kv_heads, s.head_dim), positions,
             s.rope_base, dtype)
    v = qkv[:, nq + nk:].reshape(t, s.n_kv_heads, s.head_dim)
    o = causal_attention(q, k_cache, v_cache, positions, dtype)
    h = np.asarray(h_rows, dtype=dtype) + o.reshape(t, nq) @ lw["wo"].astype(dtype).T
    return k, v, h


def mlp_rows(shape, lw, gain, h_mid_rows, dtype=np.float64):
    """MLP half of one layer on a few rows: h_mid + SwiGLU(RMSNorm(h_mid))."""
    h = np.asarray(h_mid_rows, dtype=dtype)
    u = rmsnorm(h, gain, shape.rms_eps, dtype)
    return h + (silu(u @ lw["w_gate"].astype(dtype).T) *
                (u @ lw["w_up"].astype(dtype).T)) @ lw["w_down"].astype(dtype).T


def layer_rows_teacher_forced(shape, lw, gain, h_rows, positions, k_cache,
                              v_cache, dtype=np.float64):
    """Teacher-forced check of one layer on a few sampled rows: the attention
    half followed by the MLP half.  Returns (k_rows, v_rows, h_out_rows)."""
    k, v, h_mid = attention_rows_teacher_forced(shape, lw, gain, h_rows, positions,
                                                k_cache, v_cache, dtype)
    return k, v, mlp_rows(shape, lw, gain, h_mid, dtype)


def kv_rows_teacher_forced(shape, lw, gain, h_rows, positions, dtype=np.float64):
    """The K/V half of the teacher-forced check: the cache cells of one layer
    for a few sampled rows, from the rows' input hidden states alone (K and V
    of a token depend on nothing but its own hidden state and position):
    RMSNorm, K/V projection, rotary turn of K.  Returns (k_rows, v_rows)."""
    s = shape
    t = h_rows.shape[0]
    a = rmsnorm(h_rows, gain, s.rms_eps, dtype)
    nq = s.n_q_heads * s.head_dim
    nk = s.n_kv_heads * s.head_dim
    kv = a @ lw["wqkv"][nq:].astype(dtype).T
    k = rope(kv[:, :nk].reshape(t, s.n_kv_heads, s.head_dim), positions, s.rope_base, dtype)
    v = kv[:, nk:].reshape(t, s.n_kv_heads, s.head_dim)
    return k, v


def kv_to_pages(shape, cache, n_tokens, page_tokens=16):
    """Lay a request's cache out as the host KV block of the boundary:
    [layer][page] with each page = K part [kv_head][slot][hd] followed by the
    V part stored transposed, [kv_head][hd][slot].  Returned as float32
    [L, n_pages, 2*Hkv*page_tokens*hd] (callers round for 16-bit models).
    Unused slots of the last page are zero."""
    s = shape
    n_pages = -(-n_tokens // page_tokens)
    half = s.n_kv_heads * page_tokens * s.head_dim
    out = np.zeros((s.n_layers, n_pages, 2 * half), dtype=np.float32)
    for l in range(s.n_layers):
        kpad = np.zeros((n_pages * page_tokens, s.n_kv_heads, s.head_dim), dtype=np.float32)
        vpad = np.zeros_like(kpad)
        kpad[:n_tokens] = cache.k[l][:n_tokens]
        vpad[:n_tokens] = cache.v[l][:n_tokens]
        kp = kpad.reshape(n_pages, page_tokens, s.n_kv_heads, s.head_dim)
        vp = vpad.reshape(n_pages, page_tokens, s.n_kv_heads, s.head_dim)
        out[l, :, :half] = kp.transpose(0, 2, 1, 3).reshape(n_pages, half)   # [g][slot][hd]
        out[l, :, half:] = vp.transpose(0, 2, 3, 1).reshape(n_pages, half)   # [g][hd][slot]
    return out
