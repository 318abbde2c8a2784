"""GPU parity of the batched form of the persistent streaming decode (bl_stack_build with
2 <= M <= 64 tokens per product): a table of independent products walked by one launch on the
matrix cores, each product compared with the CPU oracle.  int32 accumulators bit-exact; fp32
outputs to 1e-6 relative, and bit-exact where the residual add makes the comparison a single
fp32 operation.  The cases cover token groups (M > 32), k parts met through integer atomics
(long k with many tokens), ragged N and K, and tables whose entries differ in all of these."""
import numpy as np
import pytest

import oracle
import synth
from helpers import Case, assert_y_close, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
DEV = "cuda:0"


@pytest.fixture(scope="module")
def bl():
    from paper_2504_12285_amd import binding
    binding.load()
    return binding


def _item(c, want_acc=True, want_y=True, residual=None):
    Kp = (c.K + 63) // 64 * 64
    q = np.zeros((c.M, Kp), dtype=np.int8)
    q[:, :c.K] = c.q
    it = dict(packed=to_dev(c.packed(1)), beta=to_dev(np.array([c.beta], dtype=np.float32)), N=c.N, K=c.K,
              q=to_dev(q), scale=to_dev(c.scale), rowsum=to_dev(c.rowsum))
    if want_y:
        it["y"] = torch.full((c.M, c.N), float("nan"), dtype=torch.float32, device=DEV)
    if want_acc:
        it["acc"] = torch.full((c.M, c.N), -99, dtype=torch.int32, device=DEV)
    if residual is not None:
        it["residual"] = to_dev(residual)
    return it


def _check(it, c, residual=None):
    if "acc" in it:
        assert np.array_equal(it["acc"].cpu().numpy(), c.acc)
    if "y" in it:
        got = it["y"].cpu().numpy()
        if residual is None:
            assert_y_close(got, c.y)
        else:
            want = residual + c.y
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("M", [8, 32, 64])
def test_batched_stream_layer_shapes(bl, M):
    """Config 2: the four 2B-style shapes of a layer, every output compared.  At M = 32 the long-k
    product is split along k (partial sums through atomics + finishing kernel); at M = 64 every
    product is two token groups."""
    cases, items = [], []
    for name in ["qkv", "o", "gate_up", "down"]:
        N, K = synth.LAYER_SHAPES[name]
        c = Case(0, M, N, K, layer=1, matrix=name, relu2=(name == "down"))
        cases.append(c)
        items.append(_item(c))
    st = bl.Stack(items, 1, M, DEV)
    assert st.plan.packed_bytes == 17367040 and st.plan.tokens == M
    assert st.plan.entries >= 4
    for _ in range(2):                    # the second run finds the partial sums cleared by the first
        for it in items:
            it["y"].fill_(float("nan"))
            it["acc"].fill_(-99)
        st.run()
        torch.cuda.synchronize()
        for it, c in zip(items, cases):
            _check(it, c)


@pytest.mark.parametrize("M", [2, 3, 17, 31, 33, 48, 63])
def test_batched_stream_token_counts(bl, M):
    """Every kind of token count (below, at and above a matrix-core tile) on ragged shapes."""
    shapes = [(100, 2560), (259, 6912), (2563, 1000), (64, 64), (33, 4608)]
    cases, items, ress = [], [], []
    for i, (N, K) in enumerate(shapes):
        c = Case(11 + M, M, N, K, layer=i, matrix=i % 4)
        res = None
        if i % 2 == 1:
            res = synth.latent_weights(5, M, N, layer=i, matrix=9).astype(np.float32) * 50.0
        cases.append(c)
        ress.append(res)
        items.append(_item(c, want_acc=(i != 2), want_y=(i != 3), residual=res))
    st = bl.Stack(items, 1, M, DEV)
    st.run()
    torch.cuda.synchronize()
    for it, c, res in zip(items, cases, ress):
        _check(it, c, res)


@pytest.mark.parametrize("M", [49, 56, 64])
def test_batched_stream_tile_route(bl, M):
    """More than 48 tokens with every row padded to a multiple of 128: the table is walked by the
    matrix-core tile kernel (plan.norm == 3).  Ragged N (a part-filled last tile, a single
    part-filled tile), K = 128 (one k step) to K = 6912, residuals, y alone, acc alone; two runs."""
    shapes = [(100, 2560), (259, 6912), (2563, 1000), (129, 128), (33, 4608), (1280, 1152)]
    cases, items, ress = [], [], []
    for i, (N, K) in enumerate(shapes):
        c = Case(40 + M, M, N, K, layer=i, matrix=i % 4)
        res = None
        if i % 2 == 1:
            res = synth.latent_weights(6, M, N, layer=i, matrix=9).astype(np.float32) * 50.0
        cases.append(c)
        ress.append(res)
        items.append(_item(c, want_acc=(i != 2), want_y=(i != 3), residual=res))
    st = bl.Stack(items, 1, M, DEV)
    assert st.plan.norm == 3 and st.plan.tokens == M and st.plan.prep_count == 0
    assert st.plan.red_ints == sum((N + 127) // 128 for N, _ in shapes)
    for _ in range(2):
        for it in items:
            if "y" in it:
                it["y"].fill_(float("nan"))
            if "acc" in it:
                it["acc"].fill_(-99)
        st.run()
        torch.cuda.synchronize()
        for it, c, res in zip(items, cases, ress):
            _check(it, c, res)


def test_batched_stream_tile_route_extreme_values_and_fallback(bl):
    """|acc| = 127 * K on every output through the tile route; and a table that holds one row
    length that is not a multiple of 128 stays on the LDS-resident kernel with the same results."""
    M, N, K = 64, 200, 6912
    c = Case(0, M, N, K, full=False)
    c.Wt = np.ones((N, K), dtype=np.int8)
    c.Wt[1::2] = -1
    c.q = np.full((M, K), 127, dtype=np.int8)
    c.q[1::2] = -127
    c.rowsum = c.q.astype(np.int32).sum(1).astype(np.int32)
    c.acc = oracle.matmul_i32(c.q, c.Wt)
    c.y = oracle.rescale(c.acc, c.beta, c.scale)
    assert abs(int(c.acc[0, 0])) == 127 * K
    it = _item(c)
    st = bl.Stack([it], 1, M, DEV)
    assert st.plan.norm == 3
    st.run()
    torch.cuda.synchronize()
    _check(it, c)
    c2 = Case(1, M, 96, 192)                      # 192 = 64 * 3: not a multiple of 128
    it1, it2 = _item(c), _item(c2)
    st = bl.Stack([it1, it2], 1, M, DEV)
    assert st.plan.norm != 3
    st.run()
    torch.cuda.synchronize()
    _check(it1, c)
    _check(it2, c2)


def test_batched_stream_extreme_values(bl):
    """|acc| = 127 * K on every output: all weights +1 or -1 against saturated activations."""
    M, N, K = 16, 96, 6912
    c = Case(0, M, N, K, full=False)
    c.Wt = np.ones((N, K), dtype=np.int8)
    c.Wt[1::2] = -1
    c.q = np.full((M, K), 127, dtype=np.int8)
    c.q[1::2] = -127
    c.rowsum = c.q.astype(np.int32).sum(1).astype(np.int32)
    c.acc = oracle.matmul_i32(c.q, c.Wt)
    c.y = oracle.rescale(c.acc, c.beta, c.scale)
    assert abs(int(c.acc[0, 0])) == 127 * K
    it = _item(c)
    st = bl.Stack([it], 1, M, DEV)
    st.run()
    torch.cuda.synchronize()
    _check(it, c)


def test_batched_stream_many_products_repeatable(bl):
    """A longer table (more entries than workgroups meet one by one) run three times: identical
    bits every time, and equal to the decode entry point on the same inputs."""
    M = 24
    cases, items = [], []
    for i in range(12):
        N, K = [(640, 2560), (384, 6912), (1024, 1536)][i % 3]
        c = Case(3, M, N, K, layer=i, matrix=i % 4, full=False)
        cases.append(c)
        items.append(_item(c))
    st = bl.Stack(items, 1, M, DEV)
    outs = []
    for _ in range(3):
        st.run()
        torch.cuda.synchronize()
        outs.append([(it["acc"].clone(), it["y"].clone()) for it in items])
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    for a, b in zip(outs[0], outs[2]):
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    for it, c, o in zip(items, cases, outs[0]):
        acc, y = bl.bl_gemv_w158a8(it["packed"], it["beta"], 1, it["q"], it["scale"], it["rowsum"], c.N, K=c.K)
        assert torch.equal(acc, o[0]) and torch.equal(y, o[1])
        assert np.array_equal(acc.cpu().numpy(), oracle.matmul_i32(c.q, c.Wt))


def test_batched_stream_rejects(bl):
    """Argument errors of the batched form, found on the host."""
    c = Case(0, 4, 64, 128)
    it = _item(c)
    with pytest.raises(bl.BitLinearError) as e:
        bl.Stack([it], 0, 4, DEV)                      # layout 0 is not taken
    assert e.value.status == 3
    bad = dict(it)
    del bad["rowsum"]
    with pytest.raises(bl.BitLinearError) as e:
        bl.Stack([bad], 1, 4, DEV)
    assert e.value.status == 1
    with pytest.raises(bl.BitLinearError):
        bl.Stack([it], 1, 65, DEV)                     # beyond BL_STACK_MAX_TOKENS
