"""GPU parity: every C-ABI call against the CPU oracle on the same seeded
inputs.  Integers, bytes and bit patterns must match exactly; rescaled fp32
outputs to 1e-6 relative (the stated bar; both sides use the same two fp32
multiplies so they are normally bit-identical)."""
import numpy as np
import pytest

import oracle
import synth
from helpers import Case, assert_y_close, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def bl():
    from paper_2504_12285_amd import binding
    binding.load()
    return binding


def _sync():
    torch.cuda.synchronize()


PATHS = {"rows": 1, "mma": 2, "panel": 3}


@pytest.fixture
def force_path(bl):
    """Routes the decode entry points to one kernel through the library's test hook and puts the
    default back afterwards."""
    def set_path(name):
        assert bl.load().bl_debug_force_path(PATHS[name]) == 0
    yield set_path
    assert bl.load().bl_debug_force_path(0) == 0


# ------------------------------------------------------------------- packing
@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("shape", [(4, 64), (48, 320), (2560, 2560), (2560, 6912)])
def test_pack_bytes_and_beta_bit_exact(bl, layout, shape):
    N, K = shape
    c = Case(10 + N % 7, 1, N, K, full=False)
    packed, beta = bl.bl_pack_ternary(to_dev(c.W), layout)
    _sync()
    assert beta.item() == float(c.beta)
    assert np.array_equal(packed.cpu().numpy(), c.packed(layout))
    Wt, bad = bl.bl_unpack_ternary(packed, N, K, layout)
    _sync()
    assert bad.item() == 0 and np.array_equal(Wt.cpu().numpy(), c.Wt)
    # already-ternary input gives the same bytes
    p2, _ = bl.bl_pack_ternary(to_dev(c.Wt), layout, beta=float(c.beta))
    _sync()
    assert np.array_equal(p2.cpu().numpy(), c.packed(layout))


def test_pack_ties_and_zero_matrix(bl):
    # exact ties of W/(beta+1e-5): beta chosen so the divisor is 2^-6
    eps = np.float32(1e-5)
    W = np.zeros((4, 64), dtype=np.float32)
    r = np.array([0.5, -0.5, 1.5, -1.5, 2.5, 0.51, -0.51, 0.49, 100, -100], dtype=np.float32)
    W[0, : r.size] = r * np.float32(2.0 ** -6)
    beta_o = oracle.absmean_beta(W)
    Wt_o = oracle.ternarize(W, beta_o)
    packed, beta = bl.bl_pack_ternary(to_dev(W), 0)
    _sync()
    assert beta.item() == float(beta_o)
    assert np.array_equal(packed.cpu().numpy(), oracle.pack(Wt_o, 0))
    Z = np.zeros((8, 128), dtype=np.float32)
    packed, beta = bl.bl_pack_ternary(to_dev(Z), 1)
    _sync()
    assert beta.item() == 0.0 and np.all(packed.cpu().numpy() == 0x55)


def test_unpack_counts_invalid_codes(bl):
    p = np.arange(256, dtype=np.uint8).repeat(4)  # N*K/4 = 1024 bytes -> N=16, K=256
    Wt_o, bad_o = oracle.unpack(p, 16, 256, 0)
    Wt, bad = bl.bl_unpack_ternary(to_dev(p), 16, 256, 0)
    _sync()
    assert bad.item() == bad_o and np.array_equal(Wt.cpu().numpy(), Wt_o)


# --------------------------------------------------------------- quantiser
@pytest.mark.parametrize("M,K,relu2", [(1, 64, False), (4, 2560, False), (33, 6912, True), (3, 320, False),
                                       (64, 2560, False)])
def test_quant_bit_exact(bl, M, K, relu2):
    X = synth.activations_bf16(21, M, K, matrix=3 if relu2 else 0, relu2=relu2)
    q_o, s_o, r_o = oracle.quant_act(X)
    q, s, r = bl.bl_quant_act_int8(to_dev(X))
    _sync()
    assert np.array_equal(q.cpu().numpy(), q_o)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_o.view(np.uint32))
    assert np.array_equal(r.cpu().numpy(), r_o)


def test_quant_edge_rows(bl):
    K = 128
    rows = np.zeros((5, K), dtype=np.float32)
    rows[0, :8] = [127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 63]       # ties at inv = 1
    rows[1, :7] = [2, 1, 0.5, -1, -2, 0, 0.25]                      # ties at inv = 63.5
    rows[3, :7] = [254, 1, 3, 5, -7, 0, -254]
    rows[4, :] = 3.0e-6                                             # below the 1e-5 clamp
    X = oracle.f32_to_bf16(rows)
    q_o, s_o, r_o = oracle.quant_act(X)
    q, s, r = bl.bl_quant_act_int8(to_dev(X))
    _sync()
    assert np.array_equal(q.cpu().numpy(), q_o)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_o.view(np.uint32))
    assert np.array_equal(r.cpu().numpy(), r_o)
    q2, s2, r2 = bl.bl_quant_act_int8(to_dev(X), want_rowsum=False)
    _sync()
    assert r2 is None and np.array_equal(q2.cpu().numpy(), q_o)


# ------------------------------------------------------------------ products
def _run_product(bl, fn, c, layout, use_rowsum=True):
    packed = to_dev(c.packed(layout))
    beta = to_dev(np.array([c.beta], dtype=np.float32))
    q, scale = to_dev(c.q), to_dev(c.scale)
    rowsum = to_dev(c.rowsum) if use_rowsum else None
    acc, y = fn(packed, beta, layout, q, scale, rowsum, c.N)
    _sync()
    return acc.cpu().numpy(), y.cpu().numpy()


GEMV_SHAPES = [(4, 64), (20, 64), (52, 320), (2560, 2560), (2564, 1024)]


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("M", [1, 2, 3, 4])
@pytest.mark.parametrize("shape", GEMV_SHAPES)
def test_gemv_small_m(bl, layout, M, shape):
    N, K = shape
    c = Case(31, M, N, K)
    acc, y = _run_product(bl, bl.bl_gemv_w158a8, c, layout, use_rowsum=False)
    assert np.array_equal(acc, c.acc)
    assert_y_close(y, c.y)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("M", [5, 8, 17, 32, 64])
def test_gemv_batched(bl, layout, M):
    c = Case(32, M, 2560, 2560)
    acc, y = _run_product(bl, bl.bl_gemv_w158a8, c, layout, use_rowsum=(M % 2 == 0))
    assert np.array_equal(acc, c.acc)
    assert_y_close(y, c.y)


@pytest.mark.parametrize("M,N,K", [(9, 2564, 1024), (16, 52, 320), (33, 2560, 6912), (48, 200, 8192), (64, 20, 64),
                                   (40, 132, 320), (24, 100, 1088), (20, 36, 192), (57, 264, 2624)])
def test_gemv_batched_phases_and_tails(bl, M, N, K):
    """Staging phases with a short last phase, ragged row groups, K at the limit."""
    c = Case(35, M, N, K)
    for layout in (0, 1):
        acc, y = _run_product(bl, bl.bl_gemv_w158a8, c, layout, use_rowsum=(layout == 1))
        assert np.array_equal(acc, c.acc)
        assert_y_close(y, c.y)


@pytest.mark.parametrize("path", ["rows", "mma"])
@pytest.mark.parametrize("M", [1, 2, 3, 4])
def test_both_small_m_decode_kernels(bl, force_path, path, M):
    """1..4 tokens: the dot4 kernel and the matrix-core kernel, int8 and fused inputs."""
    force_path(path)
    c = Case(39, M, 264, 1088)
    for layout in (0, 1):
        acc, y = _run_product(bl, bl.bl_gemv_w158a8, c, layout, use_rowsum=(layout == 0))
        assert np.array_equal(acc, c.acc)
        assert_y_close(y, c.y)
    packed = to_dev(c.packed(1))
    beta = to_dev(np.array([c.beta], dtype=np.float32))
    acc, y, q, scale = bl.bl_bitlinear_decode(packed, beta, 1, to_dev(c.X), c.N, want_acc=True, want_q=True)
    _sync()
    assert np.array_equal(q.cpu().numpy(), c.q) and np.array_equal(scale.cpu().numpy(), c.scale)
    assert np.array_equal(acc.cpu().numpy(), c.acc)
    assert_y_close(y.cpu().numpy(), c.y)


@pytest.mark.parametrize("path", ["mma", "panel"])
@pytest.mark.parametrize("M,N,K", [(5, 264, 1088), (12, 2560, 2560), (17, 2560, 2560), (32, 264, 2624),
                                   (40, 100, 1088), (64, 2560, 6912), (64, 36, 192), (9, 20, 64)])
def test_both_batched_decode_kernels_at_every_m(bl, force_path, path, M, N, K):
    """The library picks one of two matrix-core kernels by measured speed; the test hook forces
    either, and both must give the oracle's numbers on every shape."""
    force_path(path)
    c = Case(37, M, N, K)
    for layout in (0, 1):
        acc, y = _run_product(bl, bl.bl_gemv_w158a8, c, layout, use_rowsum=(layout == 0))
        assert np.array_equal(acc, c.acc)
        assert_y_close(y, c.y)


@pytest.mark.parametrize("M", [2, 12, 28, 48])
def test_decode_single_outputs(bl, M):
    """acc alone (no scales at all) and y alone, on each decode kernel."""
    c = Case(38, M, 136, 832)
    packed = to_dev(c.packed(1))
    beta = to_dev(np.array([c.beta], dtype=np.float32))
    q, scale, rowsum = to_dev(c.q), to_dev(c.scale), to_dev(c.rowsum)
    acc, y = bl.bl_gemv_w158a8(packed, beta, 1, q, None, rowsum, c.N, want_acc=True, want_y=False)
    _sync()
    assert y is None and np.array_equal(acc.cpu().numpy(), c.acc)
    acc, y = bl.bl_gemv_w158a8(packed, beta, 1, q, scale, None, c.N, want_acc=False, want_y=True)
    _sync()
    assert acc is None
    assert_y_close(y.cpu().numpy(), c.y)


@pytest.mark.parametrize("M", [1, 3, 40])
def test_long_rows_beyond_the_decode_kernels(bl, M):
    """K above 8192: the decode entry point hands over to the prefill kernel; the int32 sums
    reach 16,384 terms.  Both layouts (layout 0 takes the register-staged kernel)."""
    c = Case(36, M, 68, 16384)
    for layout in (0, 1):
        for fn in (bl.bl_gemv_w158a8, bl.bl_gemm_w158a8):
            acc, y = _run_product(bl, fn, c, layout, use_rowsum=(layout == 0))
            assert np.array_equal(acc, c.acc)
            assert_y_close(y, c.y)


@pytest.mark.parametrize("name", ["qkv", "o", "gate_up", "down"])
@pytest.mark.parametrize("M", [1, 4, 8, 32, 64])
def test_gemv_layer_shapes(bl, name, M):
    """Configs 1 and 2: every layer shape as a single product at M = 1, 4, 8, 32 and 64."""
    N, K = synth.LAYER_SHAPES[name]
    c = Case(0, M, N, K, layer=0, matrix=name, relu2=(name == "down"))
    for layout in (0, 1):
        acc, y = _run_product(bl, bl.bl_gemv_w158a8, c, layout)
        assert np.array_equal(acc, c.acc)
        assert_y_close(y, c.y)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("M,N,K", [(1, 4, 64), (7, 20, 64), (100, 132, 320), (128, 128, 128), (300, 2560, 2560),
                                   (129, 260, 6912)])
def test_gemm_ragged(bl, layout, M, N, K):
    c = Case(33, M, N, K)
    acc, y = _run_product(bl, bl.bl_gemm_w158a8, c, layout, use_rowsum=(M % 2 == 1))
    assert np.array_equal(acc, c.acc)
    assert_y_close(y, c.y)


@pytest.mark.parametrize("name", ["qkv", "o", "gate_up", "down"])
def test_gemm_prefill_2048_full(bl, name):
    N, K = synth.LAYER_SHAPES[name]
    c = Case(0, 2048, N, K, layer=0, matrix=name, relu2=(name == "down"))
    acc, y = _run_product(bl, bl.bl_gemm_w158a8, c, 1)
    assert np.array_equal(acc, c.acc)
    assert_y_close(y, c.y)


def test_weights_read_back_through_the_product(bl):
    """x = 127 * e_k gives acc[m][n] = 127 * Wt[n][k]: one token per k reads the
    whole matrix back through pack + product (catches any layout/index slip)."""
    N, K = 64, 256
    Wt = synth.uniform_i8(40, (N, K), -1, 1)
    q = np.zeros((K, K), dtype=np.int8)
    q[np.arange(K), np.arange(K)] = 127
    scale = np.ones(K, dtype=np.float32)
    beta = to_dev(np.array([1.0], dtype=np.float32))
    for layout in (0, 1):
        packed = to_dev(oracle.pack(Wt, layout))
        acc, _ = bl.bl_gemm_w158a8(packed, beta, layout, to_dev(q), to_dev(scale), None, N)
        _sync()
        assert np.array_equal(acc.cpu().numpy(), 127 * Wt.T.astype(np.int32))
        for k0 in (0, 64, 192):
            acc, _ = bl.bl_gemv_w158a8(packed, beta, layout, to_dev(q[k0:k0 + 4]), to_dev(scale[:4]), None, N)
            _sync()
            assert np.array_equal(acc.cpu().numpy(), 127 * Wt.T[k0:k0 + 4].astype(np.int32))


def test_extreme_values_and_zero_input(bl):
    N, K = 128, 6912
    ones = np.ones((N, K), dtype=np.int8)
    q = np.full((2, K), 127, dtype=np.int8)
    q[1] = -127
    beta = to_dev(np.array([1.0], dtype=np.float32))
    scale = to_dev(np.ones(2, dtype=np.float32))
    packed = to_dev(oracle.pack(ones, 1))
    for fn in (bl.bl_gemv_w158a8, bl.bl_gemm_w158a8):
        acc, y = fn(packed, beta, 1, to_dev(q), scale, None, N)
        _sync()
        a = acc.cpu().numpy()
        assert np.all(a[0] == 127 * K) and np.all(a[1] == -127 * K)   # |acc| bound 877,824 reached
        acc, y = fn(packed, beta, 1, to_dev(np.zeros((2, K), np.int8)), scale, None, N)
        _sync()
        assert not acc.cpu().numpy().any()
        yz = y.cpu().numpy()
        assert np.all(yz == 0) and not np.signbit(yz).any()


def test_repeatable_and_token_independent(bl):
    c = Case(34, 4, 2560, 2560)
    first = _run_product(bl, bl.bl_gemv_w158a8, c, 1)[0]
    for _ in range(3):
        assert np.array_equal(_run_product(bl, bl.bl_gemv_w158a8, c, 1)[0], first)
    packed = to_dev(c.packed(1))
    beta = to_dev(np.array([c.beta], dtype=np.float32))
    for m in range(4):
        acc, _ = bl.bl_gemv_w158a8(packed, beta, 1, to_dev(c.q[m:m + 1]), to_dev(c.scale[m:m + 1]), None, c.N)
        _sync()
        assert np.array_equal(acc.cpu().numpy()[0], first[m])


def test_whole_layer_through_the_abi(bl):
    """Config-0 style end to end: latent weights and bf16 activations in, every
    intermediate compared (packed, beta, q, scale, acc, y)."""
    c = Case(0, 4, 2560, 2560)
    packed, beta = bl.bl_pack_ternary(to_dev(c.W), 1)
    q, scale, rowsum = bl.bl_quant_act_int8(to_dev(c.X))
    acc, y = bl.bl_gemv_w158a8(packed, beta, 1, q, scale, rowsum, c.N)
    _sync()
    assert np.array_equal(packed.cpu().numpy(), c.packed(1)) and beta.item() == float(c.beta)
    assert np.array_equal(q.cpu().numpy(), c.q) and np.array_equal(scale.cpu().numpy(), c.scale)
    assert np.array_equal(acc.cpu().numpy(), c.acc)
    assert_y_close(y.cpu().numpy(), c.y)


# ------------------------------------------------ fused and grouped decode
@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("M", [1, 3, 4])
@pytest.mark.parametrize("name", ["o", "down", "small"])
def test_fused_decode_matches_oracle(bl, layout, M, name):
    N, K = (52, 320) if name == "small" else synth.LAYER_SHAPES[name]
    c = Case(51, M, N, K, matrix=3 if name == "down" else 1, relu2=(name == "down"))
    packed = to_dev(c.packed(layout))
    beta = to_dev(np.array([c.beta], dtype=np.float32))
    acc, y, q, scale = bl.bl_bitlinear_decode(packed, beta, layout, to_dev(c.X), N, want_acc=True, want_q=True)
    _sync()
    assert np.array_equal(q.cpu().numpy(), c.q)
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), c.scale.view(np.uint32))
    assert np.array_equal(acc.cpu().numpy(), c.acc)
    assert_y_close(y.cpu().numpy(), c.y)


def test_fused_decode_zero_and_tiny_rows(bl):
    N, K = 64, 256
    Wt = synth.uniform_i8(52, (N, K), -1, 1)
    rows = np.zeros((3, K), dtype=np.float32)
    rows[1, :] = 3.0e-6
    rows[2, :5] = [2, 1, 0.5, -1, 0.25]
    X = oracle.f32_to_bf16(rows)
    ref = oracle.bitlinear(X, Wt, np.float32(0.5))
    packed = to_dev(oracle.pack(Wt, 1))
    beta = to_dev(np.array([0.5], dtype=np.float32))
    acc, y, q, scale = bl.bl_bitlinear_decode(packed, beta, 1, to_dev(X), N, want_acc=True, want_q=True)
    _sync()
    assert np.array_equal(q.cpu().numpy(), ref["q"]) and np.array_equal(scale.cpu().numpy(), ref["scale"])
    assert np.array_equal(acc.cpu().numpy(), ref["acc"])
    assert_y_close(y.cpu().numpy(), ref["y"])


@pytest.mark.parametrize("M,fused", [(1, False), (1, True), (2, False), (2, True), (4, False), (4, True), (8, False), (8, True),
                                     (8, "mixed"), (24, False), (32, False), (40, False), (64, False)])
def test_grouped_decode_whole_layer(bl, M, fused):
    """The four shapes of one layer in ONE launch equal four oracle products."""
    cases, items, keep = [], [], []
    mixed = fused == "mixed"
    for name in ["qkv", "o", "gate_up", "down"]:
        if mixed:
            fused = name in ("o", "down")
        N, K = synth.LAYER_SHAPES[name]
        c = Case(0, M, N, K, layer=1, matrix=name, relu2=(name == "down"))
        it = dict(packed=to_dev(c.packed(1)), beta=to_dev(np.array([c.beta], dtype=np.float32)), N=N, K=K,
                  acc=torch.empty((M, N), dtype=torch.int32, device="cuda:0"),
                  y=torch.empty((M, N), dtype=torch.float32, device="cuda:0"))
        if fused:
            it["X"] = to_dev(c.X)
        else:
            it.update(q=to_dev(c.q), scale=to_dev(c.scale), rowsum=to_dev(c.rowsum))
        cases.append(c)
        items.append(it)
    descs = bl.make_decode_descs(items)
    bl.bl_bitlinear_decode_group(descs, 1, M)
    _sync()
    for c, it in zip(cases, items):
        assert np.array_equal(it["acc"].cpu().numpy(), c.acc)
        assert_y_close(it["y"].cpu().numpy(), c.y)


@pytest.mark.parametrize("M", [3, 12, 40, 64])
def test_grouped_decode_residual_epilogue(bl, M):
    """y = residual + float(acc) * (beta * scale): the fp32 add of the epilogue, every decode kernel."""
    rng = np.random.default_rng(7)
    c = Case(54, M, 264, 1088)
    res = rng.standard_normal((M, c.N)).astype(np.float32)
    it = dict(packed=to_dev(c.packed(1)), beta=to_dev(np.array([c.beta], dtype=np.float32)), N=c.N, K=c.K,
              q=to_dev(c.q), scale=to_dev(c.scale), rowsum=to_dev(c.rowsum), residual=to_dev(res),
              y=torch.empty((M, c.N), dtype=torch.float32, device="cuda:0"))
    bl.bl_bitlinear_decode_group(bl.make_decode_descs([it]), 1, M)
    _sync()
    # y = residual + t, t = float(acc)*(beta*scale): t is the same two fp32 multiplies on both
    # sides, so the one fp32 add is compared bit for bit
    want = res + c.y
    got = it["y"].cpu().numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("M", [6, 24, 56])
def test_grouped_decode_two_products_one_with_residual(bl, M):
    """Two products of different shape in one launch, the second with a residual and without
    row sums: the group then takes the variant that accumulates sum_k q itself."""
    rng = np.random.default_rng(11)
    ca, cb = Case(55, M, 200, 1088), Case(56, M, 132, 4160)
    res = rng.standard_normal((M, cb.N)).astype(np.float32)
    items = []
    for c, extra in ((ca, {}), (cb, dict(residual=to_dev(res)))):
        it = dict(packed=to_dev(c.packed(1)), beta=to_dev(np.array([c.beta], dtype=np.float32)), N=c.N, K=c.K,
                  q=to_dev(c.q), scale=to_dev(c.scale), acc=torch.empty((M, c.N), dtype=torch.int32, device="cuda:0"),
                  y=torch.empty((M, c.N), dtype=torch.float32, device="cuda:0"))
        if c is ca:
            it["rowsum"] = to_dev(c.rowsum)
        it.update(extra)
        items.append(it)
    bl.bl_bitlinear_decode_group(bl.make_decode_descs(items), 1, M)
    _sync()
    assert np.array_equal(items[0]["acc"].cpu().numpy(), ca.acc)
    assert np.array_equal(items[1]["acc"].cpu().numpy(), cb.acc)
    assert_y_close(items[0]["y"].cpu().numpy(), ca.y)
    want = res + cb.y
    assert np.array_equal(items[1]["y"].cpu().numpy().view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("seed", list(range(12)))
def test_grouped_decode_seeded_shape_mix(bl, seed):
    """Seeded mixes of valid shapes through the grouped entry point: 1..4 int8 products with
    ragged N, K not a multiple of the kernels' k steps, either layout, optional row sums,
    residuals and int32 outputs; every token count from 2 to 64 comes up over the seeds."""
    rng = np.random.default_rng(1000 + seed)
    M = int(rng.integers(2, 65))
    layout = int(rng.integers(0, 2))
    count = int(rng.integers(1, 5))
    items, cases, residuals = [], [], []
    for i in range(count):
        N = 4 * int(rng.integers(1, 150))
        K = 64 * int(rng.integers(1, 70))
        c = Case(2000 + 10 * seed + i, M, N, K)
        it = dict(packed=to_dev(c.packed(layout)), beta=to_dev(np.array([c.beta], dtype=np.float32)), N=N, K=K,
                  q=to_dev(c.q), scale=to_dev(c.scale),
                  y=torch.empty((M, N), dtype=torch.float32, device="cuda:0"))
        if rng.integers(0, 2):
            it["rowsum"] = to_dev(c.rowsum)
        if rng.integers(0, 2):
            it["acc"] = torch.empty((M, N), dtype=torch.int32, device="cuda:0")
        res = None
        if rng.integers(0, 3) == 0:
            res = rng.standard_normal((M, N)).astype(np.float32)
            it["residual"] = to_dev(res)
        items.append(it); cases.append(c); residuals.append(res)
    bl.bl_bitlinear_decode_group(bl.make_decode_descs(items), layout, M)
    _sync()
    for it, c, res in zip(items, cases, residuals):
        if "acc" in it:
            assert np.array_equal(it["acc"].cpu().numpy(), c.acc)
        got = it["y"].cpu().numpy()
        if res is None:
            assert_y_close(got, c.y)
        else:
            want = res + c.y
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_fused_fixed_scale(bl):
    c = Case(53, 2, 128, 256)
    it = dict(packed=to_dev(c.packed(1)), beta=to_dev(np.array([c.beta], dtype=np.float32)), N=c.N, K=c.K,
              X=to_dev(c.X), y=torch.empty((2, c.N), dtype=torch.float32, device="cuda:0"),
              fixed_scale=float(np.float32(1.0) / np.float32(127.0)))
    bl.bl_bitlinear_decode_group(bl.make_decode_descs([it]), 1, 2)
    _sync()
    unit = np.full(2, np.float32(1.0) / np.float32(127.0), dtype=np.float32)
    assert_y_close(it["y"].cpu().numpy(), oracle.rescale(c.acc, c.beta, unit))


@pytest.mark.parametrize("M,N,K", [(2048, 13824, 2560), (2100, 4200, 640), (1024, 8320, 128), (1100, 8200, 1152)])
def test_gemm_prefill_fp32_output_alone_defers_its_stores(bl, M, N, K):
    """With only the fp32 output asked for, the 128x128 prefill kernel keeps a tile's results in
    registers and stores them during the workgroup's next tile.  More tiles than resident
    workgroups (so tiles are deferred), edges in M and N (stored at once), fewer k steps than
    store groups (flushed behind the k loop), one k step: bit-identical to the call that also
    returns the accumulators, and within 1e-6 of the oracle on sampled rows."""
    rng = np.random.default_rng(M + N + K)
    Wt = rng.integers(-1, 2, size=(N, K), dtype=np.int8)
    q = rng.integers(-127, 128, size=(M, K), dtype=np.int8)
    scale = (rng.random(M, dtype=np.float32) + np.float32(0.5)) / np.float32(127.0)
    beta = np.float32(0.0173)
    rowsum = q.astype(np.int32).sum(1).astype(np.int32)
    packed = to_dev(oracle.pack(Wt, 1))
    b = to_dev(np.array([beta], dtype=np.float32))
    qd, sd, rd = to_dev(q), to_dev(scale), to_dev(rowsum)
    acc, y_both = bl.bl_gemm_w158a8(packed, b, 1, qd, sd, rd, N)
    y_only = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
    for _ in range(2):
        y_only.fill_(float("nan"))
        bl.bl_gemm_w158a8(packed, b, 1, qd, sd, rd, N, want_acc=False, y=y_only)
        torch.cuda.synchronize()
        assert torch.equal(y_only, y_both)
    rows = np.unique(np.concatenate([np.arange(0, M, 97), [M - 1]]))
    want_acc = oracle.matmul_i32(q[rows], Wt)
    assert np.array_equal(acc.cpu().numpy()[rows], want_acc)
    assert_y_close(y_only.cpu().numpy()[rows], oracle.rescale(want_acc, beta, scale[rows]))
