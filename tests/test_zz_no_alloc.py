"""cf_offload_static -- the entry point for callers that cannot allocate -- against
cf_offload on the same pages: two calls in a row on one GPU's static scratch, the
second with a smaller input, so that what the first call left behind in the
scratch (a longer page table, a fuller staging slot) must not leak into the
second's result.  Bytes must be identical to cf_offload's (integer/byte work:
bit-exact), on the float32 tiny shape and on a bf16 shape whose request spans
needs one staging piece per layer, and on a one-layer model of the 8B shape's
page size (64 KiB) whose 5000-token request needs two pieces per layer."""
import numpy as np
import pytest
import torch

from workloads import SHAPES, WeightSource

pytestmark = pytest.mark.gpu


class _Batch:
    pass


def _session(shape_name, seed, n_ctx_list):
    from paper_2604_25080_amd.runtime import Session
    b = _Batch()
    b.shape = SHAPES["8b"].with_layers(1).with_vocab(1000) if shape_name == "8b-1layer" else SHAPES[shape_name]
    rng = np.random.default_rng(seed)
    b.n_ctx = list(n_ctx_list)
    b.n_new = [3] * len(b.n_ctx)
    b.ctx_tokens = [rng.integers(0, b.shape.vocab, size=n).astype(np.int32) for n in b.n_ctx]
    b.new_tokens = [rng.integers(0, b.shape.vocab, size=m).astype(np.int32) for m in b.n_new]
    ws = WeightSource(b.shape, 9000 + seed, cache=True)
    pages = sum(-(-(n + m) // 16) for n, m in zip(b.n_ctx, b.n_new)) + 8
    sess = Session(b.shape, ws, max_batch=len(b.n_ctx), max_tokens=sum(b.n_ctx) + sum(b.n_new),
                   max_positions=max(b.n_ctx) + 32, n_pages=pages, pool_fill=0x5A)
    return b, sess


@pytest.mark.parametrize("shape_name,lengths", [("tiny", (203, 64)), ("mini-bf16", (1000, 333)),
                                                ("8b-1layer", (5000, 300))])
def test_static_scratch_offload_equals_offload_on_two_calls_in_a_row(shape_name, lengths):
    import paper_2604_25080_amd as cf
    b, sess = _session(shape_name, 77, lengths)
    try:
        reqs = []
        for i, n in enumerate(b.n_ctx):
            sess.cache.alloc(1 + i, n + b.n_new[i])
            reqs.append(dict(req_id=1 + i, ctx_tokens=b.ctx_tokens[i], new_tokens=b.new_tokens[i], host_kv=None))
        sess.restore(reqs, [(0, n, b.shape.n_layers) for n in b.n_ctx], want_logits=False)
        assert b.n_ctx[1] < b.n_ctx[0]
        for i, n in enumerate(b.n_ctx):               # first call: the larger request, then the smaller
            nbytes = sess.host_kv_bytes(n)
            out = sess.pinned(nbytes)
            out.fill_(0xEE)
            sess.ctx.offload_static(sess.cache, 1 + i, n, out.data_ptr())
            sess.ctx.set_load_path(1)
            staged = sess.offload(1 + i, n).numpy()[:nbytes].copy()
            sess.ctx.set_load_path(0)
            direct = sess.offload(1 + i, n).numpy()[:nbytes].copy()
            got = out.numpy()[:nbytes]
            assert np.array_equal(got, staged), f"request {i}: differs from cf_offload's staged path"
            assert np.array_equal(got, direct), f"request {i}: differs from cf_offload's direct path"
        # limits and preconditions are errors, not faults
        with pytest.raises(cf.CfError) as e:
            sess.ctx.offload_static(sess.cache, 1, b.n_ctx[0], torch.zeros(sess.host_kv_bytes(b.n_ctx[0]),
                                                                        dtype=torch.uint8).data_ptr())
        assert e.value.status == cf.CF_ERR_INVALID_ARG          # pageable destination
        with pytest.raises(cf.CfError) as e:
            sess.ctx.offload_static(sess.cache, 99, 16, sess.pinned(1 << 16).data_ptr())
        assert e.value.status == cf.CF_ERR_UNKNOWN_REQUEST
        assert cf.lib.cf_offload_static_max_tokens() == 16320 * 16
    finally:
        sess.close()
