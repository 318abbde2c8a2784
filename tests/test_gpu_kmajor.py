"""GPU parity of the k-major form (layout 3), the one that leaves out the weights of zero activations:
packing and unpacking against the oracle's bytes, and the streamed M = 1 decode over tables in that form
against the oracle's products at activation densities from all-zero to dense (int32, int8 and scale bit
patterns bit-exact, fp32 to 1e-6 relative, residual sums bit-exact)."""
import numpy as np
import pytest

import oracle
import synth
from helpers import Case, assert_y_close, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
DEV = "cuda:0"
KM = 3


@pytest.fixture(scope="module")
def bl():
    from paper_2504_12285_amd import binding
    binding.load()
    return binding


@pytest.mark.parametrize("N,K", [(1, 1), (3, 17), (64, 64), (70, 9), (257, 333), (2560, 6912)])
def test_pack_unpack_kmajor(bl, N, K):
    c = Case(600 + N + K, 1, N, K, full=False)
    want = oracle.pack_kmajor(c.Wt)
    assert bl.bl_packed_bytes(N, K, KM) == want.size
    packed, beta = bl.bl_pack_ternary(to_dev(c.W), KM)
    assert np.array_equal(beta.cpu().numpy().view(np.uint32), np.array([c.beta], dtype=np.float32).view(np.uint32))
    assert np.array_equal(packed.cpu().numpy(), want)
    packed8, _ = bl.bl_pack_ternary(to_dev(c.Wt), KM, beta=float(c.beta))
    assert np.array_equal(packed8.cpu().numpy(), want)
    Wt, bad = bl.bl_unpack_ternary(packed, N, K, KM)
    assert int(bad.item()) == 0 and np.array_equal(Wt.cpu().numpy(), c.Wt)


class SparseCase(Case):
    """A Case whose bf16 activations are zero with probability 1 - density (whole elements, as squared
    ReLU produces them)."""

    def __init__(self, seed, N, K, density, **kw):
        super().__init__(seed, 1, N, K, full=False, **kw)
        rng = np.random.default_rng(seed + 99)
        keep = rng.random((1, K)) < density
        self.X = np.where(keep, self.X, np.uint16(0)).astype(np.uint16)
        self.q, self.scale, self.rowsum = oracle.quant_act(self.X)
        self.acc = oracle.matmul_i32(self.q, self.Wt)
        self.y = oracle.rescale(self.acc, self.beta, self.scale)


def _item(c, mode, want_acc=True, residual=None, rowsum=True, emit=False):
    it = dict(packed=to_dev(c.packed(KM)), beta=to_dev(np.array([c.beta], dtype=np.float32)), N=c.N, K=c.K,
              y=torch.full((1, c.N), float("nan"), dtype=torch.float32, device=DEV))
    if want_acc:
        it["acc"] = torch.full((1, c.N), -99, dtype=torch.int32, device=DEV)
    if mode == "x":
        it["X"] = to_dev(c.X)
        if emit:
            it["q_out"] = torch.empty((1, c.K), dtype=torch.int8, device=DEV)
            it["scale_out"] = torch.empty(1, dtype=torch.float32, device=DEV)
    else:
        it.update(q=to_dev(oracle.pad_q(c.q)), scale=to_dev(c.scale))
        if rowsum:
            it["rowsum"] = to_dev(c.rowsum)
    if residual is not None:
        it["residual"] = to_dev(residual)
    return it


def _check(it, c, residual=None):
    if "acc" in it:
        assert np.array_equal(it["acc"].cpu().numpy(), c.acc), (c.N, c.K)
    got = it["y"].cpu().numpy()
    if residual is None:
        assert_y_close(got, c.y)
    else:
        assert np.array_equal(got.view(np.uint32), (residual + c.y).view(np.uint32))
    if "q_out" in it:
        assert np.array_equal(it["q_out"].cpu().numpy(), c.q)
        assert np.array_equal(it["scale_out"].cpu().numpy().view(np.uint32), c.scale.view(np.uint32))


@pytest.mark.parametrize("mode", ["x", "q"])
@pytest.mark.parametrize("density", [0.0, 0.02, 0.5, 1.0])
def test_stream_kmajor_down_projection(bl, mode, density):
    """Eight down projections (2560 x 6912) of different layers in one table; run three times (the
    partial-sum arrays must be left at zero by every run)."""
    N, K = synth.LAYER_SHAPES["down"]
    cases = [SparseCase(40 + l, N, K, density, layer=l, matrix="down", relu2=True) for l in range(8)]
    rng = np.random.default_rng(2)
    residuals = [rng.standard_normal((1, N)).astype(np.float32) if l % 2 else None for l in range(8)]
    items = [_item(c, mode, residual=r, emit=True) for c, r in zip(cases, residuals)]
    st = bl.Stack(items, KM, 1, DEV)
    assert st.plan.packed_bytes == 8 * 6912 * 2560 // 4
    for rep in range(3):
        for it in items:
            it["y"].fill_(float("nan"))
            it["acc"].fill_(-7)
        st.run()
        torch.cuda.synchronize()
        for it, c, r in zip(items, cases, residuals):
            _check(it, c, r)


def test_stream_kmajor_relu2_inputs_as_generated(bl):
    """The synthetic squared-ReLU activations as they come: half of them exactly zero before the
    quantiser, and, because squaring stretches the outliers that set the absmax, most of the rest
    quantise to zero as well."""
    N, K = synth.LAYER_SHAPES["down"]
    c = Case(3, 1, N, K, layer=5, matrix="down", relu2=True)
    assert 0.4 < np.count_nonzero(c.X == 0) / c.X.size < 0.6
    assert np.count_nonzero(c.q == 0) / c.q.size > 0.9 and np.count_nonzero(c.q) >= 8
    it = _item(c, "x")
    st = bl.Stack([it], KM, 1, DEV)
    st.run()
    torch.cuda.synchronize()
    _check(it, c)


@pytest.mark.parametrize("seed", list(range(6)))
def test_stream_kmajor_seeded_mix(bl, seed):
    """Seeded tables: ragged N (1 .. 3072: one, two or three column blocks) and K, bf16 or int8 inputs,
    optional row sums, residuals, int32 outputs, densities from sparse to dense; run twice."""
    rng = np.random.default_rng(9000 + seed)
    count = int(rng.integers(1, 8))
    items, cases, residuals = [], [], []
    for i in range(count):
        K = [64, 65, 448, 2560, 6912, 20480, 1088, 333][(seed + i) % 8] if i < 3 else int(rng.integers(1, 3000))
        N = [1, 16, 17, 1024, 1025, 2049, 3072, 2560][(seed * 3 + i) % 8] if i < 4 else int(rng.integers(1, 3073))
        if K > 8000:
            N = min(N, 600)
        c = SparseCase(9100 + 20 * seed + i, N, K, float(rng.choice([0.05, 0.3, 0.5, 0.9, 1.0])))
        res = rng.standard_normal((1, N)).astype(np.float32) if rng.integers(0, 3) == 0 else None
        mode = "x" if (K % 64 == 0 and rng.integers(0, 2)) else "q"
        items.append(_item(c, mode, want_acc=bool(rng.integers(0, 2)), residual=res,
                           rowsum=bool(rng.integers(0, 2)), emit=bool(rng.integers(0, 2))))
        cases.append(c)
        residuals.append(res)
    st = bl.Stack(items, KM, 1, DEV)
    for rep in range(2):
        st.run()
        torch.cuda.synchronize()
        for it, c, res in zip(items, cases, residuals):
            _check(it, c, res)
            it["y"].fill_(float("nan"))
            if "acc" in it:
                it["acc"].fill_(-5)


def test_kmajor_limits_and_rejects(bl):
    c = Case(1, 1, 8, 64)
    it = _item(c, "q")
    wide = dict(it, N=3073)
    with pytest.raises(bl.BitLinearError) as e:
        bl.Stack([wide], KM, 1, DEV)
    assert e.value.status == 2
    packed, beta = it["packed"], it["beta"]
    for fn in (bl.bl_gemv_w158a8, bl.bl_gemm_w158a8):
        with pytest.raises(bl.BitLinearError) as e:
            fn(packed, beta, KM, to_dev(c.q), to_dev(c.scale), to_dev(c.rowsum), 8)
        assert e.value.status == 3
