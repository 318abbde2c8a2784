"""GPU parity of the persistent streaming decode (bl_stack_build / bl_stack_run): a table of
independent products walked by one launch, each product compared with the CPU oracle.
int32 accumulators, quantised inputs and scales bit-exact; fp32 outputs to 1e-6 relative
(and bit-exact where the residual add makes the comparison a single fp32 operation)."""
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


def _item(c, layout, mode, want_acc=True, residual=None, rowsum=True, emit=False):
    it = dict(packed=to_dev(c.packed(layout)), beta=to_dev(np.array([c.beta], dtype=np.float32)), N=c.N, K=c.K,
              y=torch.full((1, c.N), float("nan"), dtype=torch.float32, device=DEV))
    if want_acc:
        it["acc"] = torch.full((1, c.N), -99, dtype=torch.int32, device=DEV)
    if mode == "x":
        it["X"] = to_dev(c.X)
        if emit:
            it["q_out"] = torch.empty((1, c.K), dtype=torch.int8, device=DEV)
            it["scale_out"] = torch.empty(1, dtype=torch.float32, device=DEV)
    else:
        it.update(q=to_dev(c.q), scale=to_dev(c.scale))
        if rowsum:
            it["rowsum"] = to_dev(c.rowsum)
    if residual is not None:
        it["residual"] = to_dev(residual)
    return it


def _check(it, c, residual=None):
    if "acc" in it:
        assert np.array_equal(it["acc"].cpu().numpy(), c.acc)
    got = it["y"].cpu().numpy()
    if residual is None:
        assert_y_close(got, c.y)
    else:
        # y = residual + t with t = float(acc)*(beta*scale): t is bit-identical on both sides
        # (two fp32 multiplies), so the single fp32 add can be compared bit for bit
        want = residual + c.y
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    if "q_out" in it:
        assert np.array_equal(it["q_out"].cpu().numpy(), c.q)
        assert np.array_equal(it["scale_out"].cpu().numpy().view(np.uint32), c.scale.view(np.uint32))


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("mode", ["x", "q"])
def test_stream_one_layer_shapes(bl, layout, mode):
    """The four 2B-style shapes of a layer as one table (lane splits 8 and 32 per row)."""
    cases, items = [], []
    for name in ["qkv", "o", "gate_up", "down"]:
        N, K = synth.LAYER_SHAPES[name]
        c = Case(0, 1, N, K, layer=2, matrix=name, relu2=(name == "down"))
        cases.append(c)
        items.append(_item(c, layout, mode, emit=True))
    st = bl.Stack(items, layout, 1, DEV)
    assert st.plan.packed_bytes == 17367040
    st.run()
    torch.cuda.synchronize()
    for it, c in zip(items, cases):
        _check(it, c)
    assert st.plan.inline_count == (4 if mode == "x" else 0)


@pytest.mark.parametrize("seed", list(range(8)))
def test_stream_seeded_shape_mix(bl, seed):
    """Seeded tables: 1..9 products with ragged N (not a multiple of the row group), K from 64
    to 20480 (every lane split: 8, 16, 32, 64 lanes per row), either layout, bf16 or int8 inputs,
    optional row sums, residuals, int32 outputs; run twice (the second run must not depend on
    what the first left behind)."""
    rng = np.random.default_rng(3000 + seed)
    layout = int(rng.integers(0, 2))
    count = int(rng.integers(1, 10))
    ks = [64, 448, 2560, 6912, 5184, 10240, 20480, 1088, 3136]
    items, cases, residuals = [], [], []
    for i in range(count):
        K = ks[(seed + i) % len(ks)] if i < 3 else 64 * int(rng.integers(1, 60))
        N = 4 * int(rng.integers(1, 120 if K <= 4096 else 30))
        c = Case(4000 + 20 * seed + i, 1, N, K, relu2=bool(rng.integers(0, 2)))
        res = rng.standard_normal((1, N)).astype(np.float32) if rng.integers(0, 3) == 0 else None
        items.append(_item(c, layout, "x" if rng.integers(0, 2) else "q", want_acc=bool(rng.integers(0, 2)),
                           residual=res, rowsum=bool(rng.integers(0, 2)), emit=bool(rng.integers(0, 2))))
        cases.append(c)
        residuals.append(res)
    st = bl.Stack(items, layout, 1, DEV)
    for rep in range(2):
        st.run()
        torch.cuda.synchronize()
        for it, c, res in zip(items, cases, residuals):
            _check(it, c, res)
            it["y"].fill_(float("nan"))
            if "acc" in it:
                it["acc"].fill_(-5)


def test_stream_many_products_cross_slice_boundaries(bl):
    """Sixty small products (more products than a workgroup's slice is long): every workgroup
    meets several products and restages its activations each time."""
    items, cases = [], []
    for i in range(60):
        c = Case(5000 + i, 1, 4 * (3 + i % 11), 64 * (1 + (7 * i) % 23))
        cases.append(c)
        items.append(_item(c, 1, "x" if i % 2 else "q", rowsum=bool(i % 3)))
    st = bl.Stack(items, 1, 1, DEV)
    for rep in range(3):                     # replays: the ready flags of one run must not leak into the next
        for it in items:
            it["y"].fill_(float("nan"))
        st.run()
        torch.cuda.synchronize()
        for it, c in zip(items, cases):
            _check(it, c)


@pytest.mark.timeout(900)
def test_stream_whole_tables_as_benchmarked(bl):
    """The benchmark's streamed launches at their full size: the 120 BitLinears of 30 layers of
    the 2B shapes (521 MB of packed weights, packed on the GPU from the seeded latent weights) in
    ONE bl_stack_run each: M = 1 with bf16 inputs quantised inside the launch (config 1, the
    headline), M = 8 and M = 64 with int8 inputs (config 2).  Every int32 accumulator and every
    fp32 output of every product against the oracle."""
    names = list(synth.LAYER_SHAPES)
    Ms = (1, 8, 64)
    X = {(n, M): synth.activations_bf16(0, M, synth.LAYER_SHAPES[n][1], layer=0, matrix=n, relu2=(n == "down"))
         for n in names for M in Ms}
    quant = {k: oracle.quant_act(x) for k, x in X.items()}
    Xd = {n: to_dev(X[(n, 1)]) for n in names}
    qd = {k: tuple(to_dev(a) for a in v) for k, v in quant.items() if k[1] > 1}
    items = {M: [] for M in Ms}
    want = {M: [] for M in Ms}
    for l in range(synth.N_LAYERS):
        for n in names:
            N, K = synth.LAYER_SHAPES[n]
            W = synth.latent_weights(0, N, K, layer=l, matrix=n)
            beta, mean64 = oracle.absmean_beta(W, return_mean64=True)
            assert oracle.beta_guard_ok(mean64)
            Wt = oracle.ternarize(W, beta)
            packed, b = bl.bl_pack_ternary(to_dev(W), 1)
            assert b.item() == float(beta)
            del W
            for M in Ms:
                q, scale, _ = quant[(n, M)]
                acc = oracle.matmul_i32(q, Wt)
                want[M].append((acc, oracle.rescale(acc, beta, scale)))
                it = dict(packed=packed, beta=b, N=N, K=K,
                          y=torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV),
                          acc=torch.full((M, N), -99, dtype=torch.int32, device=DEV))
                if M == 1:
                    it["X"] = Xd[n]
                else:
                    it.update(q=qd[(n, M)][0], scale=qd[(n, M)][1], rowsum=qd[(n, M)][2])
                items[M].append(it)
            del Wt
    for M in Ms:
        st = bl.Stack(items[M], 1, M, DEV)
        assert st.plan.count == 120 and (M > 1 or st.plan.prep_count == 0)
        assert st.plan.packed_bytes == 30 * sum(N * K // 4 for N, K in synth.LAYER_SHAPES.values())
        st.run()
        torch.cuda.synchronize()
        for it, (acc, y) in zip(items[M], want[M]):
            assert np.array_equal(it["acc"].cpu().numpy(), acc)
            assert_y_close(it["y"].cpu().numpy(), y)


def test_stream_replay_with_changed_inputs(bl):
    """The same table run again after its bf16 inputs changed in place: the quantisation inside
    the launch must be redone and waited for (a stale ready flag would give the old result)."""
    N, K = 3840, 2560
    c1 = Case(61, 1, N, K)
    c2 = Case(62, 1, N, K)
    c2.Wt, c2.beta = c1.Wt, c1.beta           # same weights, new token
    c2.acc = oracle.matmul_i32(c2.q, c1.Wt)
    c2.y = oracle.rescale(c2.acc, c1.beta, c2.scale)
    it = _item(c1, 1, "x", emit=True)
    st = bl.Stack([it], 1, 1, DEV)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        st.run()
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            st.run()
    for c in (c1, c2, c1, c2):
        it["X"].copy_(to_dev(c.X))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        _check(it, c)


def test_stream_producers_and_normalisation(bl):
    """Fused producers (fp32 input, ReLU^2 gate, residual sum with its by-product) and the RMS
    normalisation in front of the quantiser, inside the streaming kernel."""
    rng = np.random.default_rng(21)
    x = (rng.standard_normal((1, 2560)) * 3).astype(np.float32)
    o = rng.standard_normal((1, 2560)).astype(np.float32)
    gu = rng.standard_normal((1, 13824)).astype(np.float32)
    gain = (1.0 + 0.05 * rng.standard_normal(2560)).astype(np.float32)
    keep = dict(x=to_dev(x), o=to_dev(o), gu=to_dev(gu), gain=to_dev(gain),
                h1=torch.empty((1, 2560), dtype=torch.float32, device=DEV))
    prods = [
        (bl.make_producer(bl.BL_PROD_F32, keep["x"]), 2560, oracle.f32_to_bf16(x)),
        (bl.make_producer(bl.BL_PROD_RELU2_GATE, keep["gu"]), 6912, oracle.chain_relu2_gate(gu)),
        (bl.make_producer(bl.BL_PROD_RESIDUAL, keep["x"], keep["o"], keep["h1"]), 2560,
         oracle.f32_to_bf16(oracle.chain_residual(x, o))),
        (bl.make_producer(bl.BL_PROD_F32, keep["x"], norm=True, gain=keep["gain"], eps=1e-5), 2560,
         oracle.rmsnorm_rows(x, gain, 1e-5)),
        (bl.make_producer(bl.BL_PROD_RELU2_GATE, keep["gu"], norm=True, eps=1e-5), 6912,
         oracle.rmsnorm_rows(oracle.chain_relu2_gate_f32(gu), None, 1e-5)),
    ]
    items, refs = [], []
    for i, (prod, K, xbits) in enumerate(prods):
        N = 200 + 4 * i
        Wt = synth.uniform_i8(70 + i, (N, K), -1, 1)
        refs.append(oracle.bitlinear(xbits, Wt, np.float32(0.5)))
        items.append(dict(packed=to_dev(oracle.pack(Wt, 1)), beta=to_dev(np.array([0.5], dtype=np.float32)), N=N, K=K,
                          prod=prod, acc=torch.empty((1, N), dtype=torch.int32, device=DEV),
                          y=torch.empty((1, N), dtype=torch.float32, device=DEV),
                          q_out=torch.empty((1, K), dtype=torch.int8, device=DEV),
                          scale_out=torch.empty(1, dtype=torch.float32, device=DEV)))
    st = bl.Stack(items, 1, 1, DEV)
    assert st.plan.norm == 1
    st.run()
    torch.cuda.synchronize()
    for it, ref in zip(items, refs):
        assert np.array_equal(it["q_out"].cpu().numpy(), ref["q"])
        assert np.array_equal(it["scale_out"].cpu().numpy().view(np.uint32), ref["scale"].view(np.uint32))
        assert np.array_equal(it["acc"].cpu().numpy(), ref["acc"])
        assert_y_close(it["y"].cpu().numpy(), ref["y"])
    assert np.array_equal(keep["h1"].cpu().numpy().view(np.uint32), oracle.chain_residual(x, o).view(np.uint32))


def test_stream_rejects_bad_tables(bl):
    c = Case(1, 1, 8, 64)
    it = _item(c, 1, "q")
    with pytest.raises(bl.BitLinearError) as e:
        bl.Stack([it], 1, 65, DEV)         # M beyond the batched form (tests/test_gpu_stream_batched.py)
    assert e.value.status == 2
    big = dict(it)
    big["K"] = 20480 + 64
    with pytest.raises(bl.BitLinearError) as e:
        bl.Stack([big], 1, 1, DEV)
    assert e.value.status == 2
    bad = dict(it)
    del bad["q"]
    with pytest.raises(bl.BitLinearError) as e:
        bl.Stack([bad], 1, 1, DEV)
    assert e.value.status == 1
