"""GPU kernel parity: the MFMA GEMM (all fused epilogues) and the plain FMA
GEMM against the definition (a float64 matmul of the same bf16 inputs), at
sizes that span several tiles with ragged tails."""
import numpy as np
import pytest
import torch

from workloads import SHAPES, WeightSource, bf16_bits, bits_to_f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sess():
    from paper_2604_25080_amd.runtime import Session
    shape = SHAPES["mini-bf16"].with_layers(1)
    s = Session(shape, WeightSource(shape, 5), max_batch=2, max_tokens=256, max_positions=256, n_pages=8)
    real = s.ctx
    s.ctx = _Synced(real)
    yield s
    s.ctx = real
    s.close()


class _Synced:
    """The library launches on its own streams, which do not order against torch's: operands and
    output buffers made by torch kernels (fills, slices) must be complete before a library call."""

    def __init__(self, ctx):
        self._ctx = ctx

    def op_gemm(self, *a, **k):
        torch.cuda.synchronize()
        return self._ctx.op_gemm(*a, **k)


def dev_bf16(x):
    return torch.from_numpy(bf16_bits(x).view(np.int16)).cuda().view(torch.bfloat16)


def from_bf16(t):
    return bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1)).reshape(t.shape)


SHAPES_MNK = [(256, 256, 64), (300, 544, 512), (1000, 1408, 512), (129, 96, 1408), (2, 2000, 512),
              (2048, 1280, 1024)]


@pytest.mark.parametrize("impl", [3, 4, 5, 1, 6])
@pytest.mark.parametrize("mnk", SHAPES_MNK + [(4400, 4096, 128)])
def test_gemm_epilogues_match_float64_matmul(sess, impl, mnk):
    import paper_2604_25080_amd as cf
    M, N, K = mnk
    rng = np.random.default_rng(M * 7 + N)
    a = bits_to_f32(bf16_bits(rng.normal(size=(M, K)).astype(np.float32)))
    w = bits_to_f32(bf16_bits((rng.normal(size=(N, K)) * 0.05).astype(np.float32)))
    w2 = bits_to_f32(bf16_bits((rng.normal(size=(N, K)) * 0.05).astype(np.float32)))
    ref = a.astype(np.float64) @ w.astype(np.float64).T
    ref2 = a.astype(np.float64) @ w2.astype(np.float64).T
    A, W, W2 = dev_bf16(a), dev_bf16(w), dev_bf16(w2)
    Cf = torch.zeros(M, N, dtype=torch.float32, device="cuda")
    Dt = torch.zeros(M, N, dtype=torch.bfloat16, device="cuda")
    tol = 1e-4 * np.sqrt(K / 512)

    sess.ctx.op_gemm(A.data_ptr(), W.data_ptr(), 0, Cf.data_ptr(), 0, M, N, K, cf.EPI_STORE_F32, impl)
    assert np.abs(Cf.cpu().numpy() - ref).max() <= tol
    base = torch.from_numpy(rng.normal(size=(M, N)).astype(np.float32)).cuda()
    Cf.copy_(base)
    sess.ctx.op_gemm(A.data_ptr(), W.data_ptr(), 0, Cf.data_ptr(), 0, M, N, K, cf.EPI_ADD_F32, impl)
    assert np.abs(Cf.cpu().numpy() - (ref + base.cpu().numpy())).max() <= tol
    sess.ctx.op_gemm(A.data_ptr(), W.data_ptr(), 0, 0, Dt.data_ptr(), M, N, K, cf.EPI_STORE_T, impl)
    got = from_bf16(Dt)
    assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + tol)      # one bf16 rounding
    sess.ctx.op_gemm(A.data_ptr(), W.data_ptr(), W2.data_ptr(), 0, Dt.data_ptr(), M, N, K, cf.EPI_SILU_MUL, impl)
    want = ref / (1.0 + np.exp(-ref)) * ref2
    got = from_bf16(Dt)
    assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -8 + 4 * tol)


# (4352, 4096): 17 x 16 = 272 big tiles = one round of 256 and 16 more: the mixed launch covers a
# 1 x 16 rectangle with 128x128 tiles; (4400, 4104): ragged edges, 18 x 17 = 306 tiles, tail 50
# rounded up to 2 x 25 > 17 columns, so the plain launch; (4660, 4360): 19 x 18 = 342, tail 86 =
# 3 rows x 29 > 18: plain; (8192, 2100): 32 x 9 = 288, tail 32 = 8 rows x 4 columns, ragged N
@pytest.mark.parametrize("mnk", [(300, 544, 512), (129, 4096, 1024), (16, 1280, 8192), (2048, 1280, 1024),
                                 (600, 768, 1408), (4352, 4096, 256), (4400, 4104, 256), (8192, 2100, 128),
                                 (4500, 4096, 128)])
def test_gemm_bits_do_not_depend_on_the_tile_shape(sess, mnk):
    """Every output element is accumulated in the same order along K whatever the block tile
    (256x256, 128x128, 64x64 with its deeper operand pipeline) and whatever else is in the
    launch: hybrid == all-recompute == chunk-by-chunk restores rest on this."""
    import paper_2604_25080_amd as cf
    M, N, K = mnk
    rng = np.random.default_rng(M + N + K)
    A = dev_bf16(rng.normal(size=(M, K)).astype(np.float32))
    W = dev_bf16((rng.normal(size=(N, K)) * 0.05).astype(np.float32))
    outs, impls = [], []
    for impl in (3, 6, 4, 5, 0):
        if impl in (3, 6) and (M < 256 or N < 256 or K % 128):
            continue
        Cf = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        sess.ctx.op_gemm(A.data_ptr(), W.data_ptr(), 0, Cf.data_ptr(), 0, M, N, K, cf.EPI_STORE_F32, impl)
        outs.append(Cf)
        impls.append(impl)
    # a sub-range of the rows on its own gives the same bits for those rows
    lo = M // 3
    Cs = torch.full((M - lo, N), float("nan"), dtype=torch.float32, device="cuda")
    sess.ctx.op_gemm(A[lo:].contiguous().data_ptr(), W.data_ptr(), 0, Cs.data_ptr(), 0, M - lo, N, K,
                     cf.EPI_STORE_F32, 0)
    for o, impl in zip(outs[1:], impls[1:]):
        if not torch.equal(outs[0], o):
            bad = torch.nonzero((outs[0] != o) | torch.isnan(o))
            raise AssertionError(f"impl {impl} differs from impl {impls[0]} in {len(bad)} elements, first at "
                                 f"{bad[0].tolist()}, last at {bad[-1].tolist()}; NaN left: {int(torch.isnan(o).sum())}")
    assert torch.equal(outs[0][lo:], Cs)


def test_gemm_mfma_refuses_what_it_cannot_tile(sess):
    import paper_2604_25080_amd as cf
    A = torch.zeros(64, 40, dtype=torch.bfloat16, device="cuda")
    Cf = torch.zeros(64, 64, dtype=torch.float32, device="cuda")
    with pytest.raises(cf.CfError) as e:
        sess.ctx.op_gemm(A.data_ptr(), A.data_ptr(), 0, Cf.data_ptr(), 0, 64, 64, 40, cf.EPI_STORE_F32, 2)
    assert e.value.status == cf.CF_ERR_UNSUPPORTED
    sess.ctx.op_gemm(A.data_ptr(), A.data_ptr(), 0, Cf.data_ptr(), 0, 64, 64, 40, cf.EPI_STORE_F32, 0)
