"""GPU parity for shapes with a ragged K (not a multiple of 64) or N (not a multiple of 4): packing,
unpacking, the quantiser, the decode and prefill products and the streamed table against the CPU
oracle.  Bytes, beta, int8, int32 and scale bit patterns bit-exact; fp32 outputs to 1e-6 relative."""
import numpy as np
import pytest

import oracle
import synth
from helpers import Case, assert_y_close, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
DEV = "cuda:0"

SHAPES = [(1, 1), (3, 17), (5, 63), (7, 65), (6, 128), (129, 200), (258, 2561), (1001, 333), (64, 100), (30, 4097)]


@pytest.fixture(scope="module")
def bl():
    from paper_2504_12285_amd import binding
    binding.load()
    return binding


@pytest.fixture
def force_path(bl):
    yield lambda p: bl._check(bl.load().bl_debug_force_path(p), "bl_debug_force_path")
    bl.load().bl_debug_force_path(0)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("N,K", SHAPES)
def test_pack_unpack_ragged(bl, N, K, layout):
    c = Case(900 + N + K, 1, N, K, full=False)
    want = oracle.pack_padded(c.Wt, layout)
    assert bl.bl_packed_bytes(N, K, layout) == want.size
    packed, beta = bl.bl_pack_ternary(to_dev(c.W), layout)
    assert np.array_equal(beta.cpu().numpy().view(np.uint32), np.array([c.beta], dtype=np.float32).view(np.uint32))
    assert np.array_equal(packed.cpu().numpy(), want)
    packed8, _ = bl.bl_pack_ternary(to_dev(c.Wt), layout, beta=float(c.beta))       # already-ternary input
    assert np.array_equal(packed8.cpu().numpy(), want)
    Wt, bad = bl.bl_unpack_ternary(packed, N, K, layout)
    assert int(bad.item()) == 0
    assert np.array_equal(Wt.cpu().numpy(), c.Wt)


@pytest.mark.parametrize("M,K", [(1, 1), (3, 17), (2, 63), (5, 65), (4, 200), (3, 2561), (130, 333), (2, 8195)])
def test_quant_ragged(bl, M, K):
    X = synth.activations_bf16(77 + K, M, K)
    q_o, s_o, r_o = oracle.quant_act(X)
    q, s, r = bl.bl_quant_act_int8(to_dev(X))
    assert tuple(q.shape) == (M, oracle.padded_k(K))
    assert np.array_equal(q.cpu().numpy(), oracle.pad_q(q_o))
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_o.view(np.uint32))
    assert np.array_equal(r.cpu().numpy(), r_o)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("path", [0, 1, 2, 3])
@pytest.mark.parametrize("M", [1, 2, 5, 17, 64])
def test_decode_product_ragged(bl, force_path, M, path, layout):
    """Every decode kernel (default choice, dot4, row-resident matrix-core, streaming panel) on ragged
    shapes, with and without the caller's row sums."""
    force_path(path)
    for i, (N, K) in enumerate(SHAPES):
        c = Case(1300 + 7 * i + M, M, N, K)
        packed = to_dev(oracle.pack_padded(c.Wt, layout))
        beta = to_dev(np.array([c.beta], dtype=np.float32))
        q = to_dev(oracle.pad_q(c.q))
        rowsum = to_dev(c.rowsum) if i % 2 else None
        acc, y = bl.bl_gemv_w158a8(packed, beta, layout, q, to_dev(c.scale), rowsum, N, K=K)
        torch.cuda.synchronize()
        assert np.array_equal(acc.cpu().numpy(), c.acc), (N, K)
        assert_y_close(y.cpu().numpy(), c.y)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("M", [1, 100, 300])
def test_prefill_product_ragged(bl, M, layout):
    for i, (N, K) in enumerate(SHAPES + [(515, 1000), (130, 8256)]):
        c = Case(1700 + 5 * i + M, M, N, K)
        packed = to_dev(oracle.pack_padded(c.Wt, layout))
        beta = to_dev(np.array([c.beta], dtype=np.float32))
        q = to_dev(oracle.pad_q(c.q))
        rowsum = to_dev(c.rowsum) if i % 2 else None
        acc, y = bl.bl_gemm_w158a8(packed, beta, layout, q, to_dev(c.scale), rowsum, N, K=K)
        torch.cuda.synchronize()
        assert np.array_equal(acc.cpu().numpy(), c.acc), (N, K)
        assert_y_close(y.cpu().numpy(), c.y)


def test_quantiser_feeds_product_on_ragged_shape(bl):
    """bf16 -> bl_quant_act_int8 -> bl_gemv_w158a8 / bl_gemm_w158a8 end to end on one ragged shape."""
    M, N, K = 9, 203, 1111
    c = Case(31, M, N, K)
    packed, beta = bl.bl_pack_ternary(to_dev(c.W), 1)
    q, s, r = bl.bl_quant_act_int8(to_dev(c.X))
    for fn in (bl.bl_gemv_w158a8, bl.bl_gemm_w158a8):
        acc, y = fn(packed, beta, 1, q, s, r, N, K=K)
        assert np.array_equal(acc.cpu().numpy(), c.acc)
        assert_y_close(y.cpu().numpy(), c.y)


@pytest.mark.parametrize("layout", [0, 1])
def test_stream_table_ragged(bl, layout):
    """The streamed table with int8 inputs of ragged shapes, with and without row sums and residuals."""
    rng = np.random.default_rng(5)
    items, cases, residuals = [], [], []
    for i, (N, K) in enumerate(SHAPES + [(2561, 2561), (77, 6913)]):
        c = Case(2100 + i, 1, N, K)
        res = rng.standard_normal((1, N)).astype(np.float32) if i % 3 == 0 else None
        it = dict(packed=to_dev(oracle.pack_padded(c.Wt, layout)), beta=to_dev(np.array([c.beta], dtype=np.float32)),
                  N=N, K=K, q=to_dev(oracle.pad_q(c.q)), scale=to_dev(c.scale),
                  acc=torch.full((1, N), -9, dtype=torch.int32, device=DEV),
                  y=torch.full((1, N), float("nan"), dtype=torch.float32, device=DEV))
        if i % 2:
            it["rowsum"] = to_dev(c.rowsum)
        if res is not None:
            it["residual"] = to_dev(res)
        items.append(it)
        cases.append(c)
        residuals.append(res)
    st = bl.Stack(items, layout, 1, DEV)
    st.run()
    torch.cuda.synchronize()
    for it, c, res in zip(items, cases, residuals):
        assert np.array_equal(it["acc"].cpu().numpy(), c.acc), (c.N, c.K)
        got = it["y"].cpu().numpy()
        if res is None:
            assert_y_close(got, c.y)
        else:
            assert np.array_equal(got.view(np.uint32), (res + c.y).view(np.uint32))


def test_grouped_decode_ragged_and_rejects(bl):
    """One grouped launch over ragged int8 products; bf16 inputs inside a product kernel need K % 64 == 0."""
    M = 3
    items, cases = [], []
    for i, (N, K) in enumerate([(129, 200), (7, 65), (258, 2561), (1001, 333)]):
        c = Case(2500 + i, M, N, K)
        items.append(dict(packed=to_dev(oracle.pack_padded(c.Wt, 1)), beta=to_dev(np.array([c.beta], dtype=np.float32)),
                          N=N, K=K, q=to_dev(oracle.pad_q(c.q)), scale=to_dev(c.scale),
                          acc=torch.empty((M, N), dtype=torch.int32, device=DEV),
                          y=torch.empty((M, N), dtype=torch.float32, device=DEV)))
        cases.append(c)
    bl.bl_bitlinear_decode_group(bl.make_decode_descs(items), 1, M)
    torch.cuda.synchronize()
    for it, c in zip(items, cases):
        assert np.array_equal(it["acc"].cpu().numpy(), c.acc)
        assert_y_close(it["y"].cpu().numpy(), c.y)
    c = cases[0]
    bad = dict(items[0])
    del bad["q"]
    bad["X"] = to_dev(c.X)
    with pytest.raises(bl.BitLinearError) as e:
        bl.bl_bitlinear_decode_group(bl.make_decode_descs([bad]), 1, M)
    assert e.value.status == 2
    with pytest.raises(bl.BitLinearError) as e:
        bl.Stack([dict(bad, X=to_dev(c.X[:1]))], 1, 1, DEV)
    assert e.value.status == 2
