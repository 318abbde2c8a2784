"""Pins of the CPU oracle against things other than itself: values worked by
hand (tests/golden), closed forms for Gaussian inputs, exactly-rounded library
routines (math.fsum, int64 matmul, torch's bf16 cast), brute force in fp64 and
structural invariants.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

import oracle
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


# ----------------------------------------------------------------- packing
def test_pack_golden_bytes():
    for ln in _rows("pack_bytes.txt"):
        *w, byte = [int(t) for t in ln.split()]
        Wt = np.zeros((4, 64), dtype=np.int8)
        Wt[0, :4] = w
        p = oracle.pack(Wt, 0)
        assert p[0] == byte, (w, p[0], byte)


def test_pack_all_81_tuples_bijective_and_roundtrip():
    tuples = list(itertools.product((-1, 0, 1), repeat=4))
    assert len(tuples) == 81
    # lay the 81 tuples along k of one matrix: K = 81*4 = 324 -> pad to 384
    Wt = np.zeros((4, 384), dtype=np.int8)
    Wt[0, :324] = np.array(tuples, dtype=np.int8).reshape(-1)
    p = oracle.pack(Wt, 0)
    first = p[:81]
    assert len(set(first.tolist())) == 81
    back, bad = oracle.unpack(p, 4, 384, 0)
    assert bad == 0 and np.array_equal(back, Wt)


def test_unpack_all_256_bytes_rejects_175():
    # every byte value once; 81 are valid, 175 contain at least one code 3
    N, K = 4, 256
    p = np.arange(256, dtype=np.uint8)
    Wt, bad_fields = oracle.unpack(p, N, K, 0)
    fields = np.stack([(p >> (2 * j)) & 3 for j in range(4)], axis=1)
    n_bad_bytes = int((fields == 3).any(axis=1).sum())
    assert n_bad_bytes == 175
    assert bad_fields == int((fields == 3).sum())
    # weight k of byte b decodes to field-1
    assert np.array_equal(Wt.reshape(-1, 4), fields.astype(np.int8) - 1)


@pytest.mark.parametrize("layout", [0, 1])
def test_pack_one_hot_positions(layout):
    """A single +1 among zeros: exactly one 2-bit field differs from code 1, at
    the byte/bit the layout formula in include/bitlinear.h states."""
    N, K = 32, 256
    rng = np.random.default_rng(1)
    for _ in range(40):
        n, k = int(rng.integers(N)), int(rng.integers(K))
        Wt = np.zeros((N, K), dtype=np.int8)
        Wt[n, k] = 1
        p = oracle.pack(Wt, layout)
        diff = np.nonzero(p != 0x55)[0]
        assert diff.size == 1
        if layout == 0:
            byte = n * (K // 4) + k // 4
            shift = 2 * (k % 4)
        else:
            i = k % 16
            byte = n * (K // 4) + (k // 16) * 4 + i % 4
            shift = 2 * (i // 4)
        assert diff[0] == byte
        assert p[byte] == (0x55 + (1 << shift))


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("shape", [(16, 64), (48, 320), (2560, 2560)])
def test_pack_roundtrip_random(layout, shape):
    N, K = shape
    Wt = synth.uniform_i8(3, (N, K), -1, 1, stream=N + K)
    p = oracle.pack(Wt, layout)
    assert p.size == N * K // 4  # four per byte (Section 5.1)
    back, bad = oracle.unpack(p, N, K, layout)
    assert bad == 0 and np.array_equal(back, Wt)


def test_layout1_word_digit_swap():
    """Layout 1 keeps each 16-weight word in place and swaps (byte, bit-pair)
    digits inside it: word1.byte[b].pair[s] == word0.byte[s].pair[b]."""
    N, K = 8, 128
    Wt = synth.uniform_i8(5, (N, K), -1, 1)
    p0 = oracle.pack(Wt, 0).reshape(-1, 4)
    p1 = oracle.pack(Wt, 1).reshape(-1, 4)
    f0 = np.stack([(p0 >> (2 * s)) & 3 for s in range(4)], axis=2)  # [word][byte][pair]
    f1 = np.stack([(p1 >> (2 * s)) & 3 for s in range(4)], axis=2)
    assert np.array_equal(f1, f0.transpose(0, 2, 1))
    # natural order: pair s of byte b of layout 1 is weight 4s+b of the word
    w = (Wt.reshape(-1, 16) + 1).astype(np.uint8)
    for s_ in range(4):
        for b in range(4):
            assert np.array_equal(f1[:, b, s_], w[:, 4 * s_ + b])


def test_pack_rejects_non_ternary():
    Wt = np.zeros((4, 64), dtype=np.int8)
    Wt[1, 3] = 2
    with pytest.raises(ValueError):
        oracle.pack(Wt, 0)


# --------------------------------------------------------- weight quantiser
def test_beta_equals_exact_mean_fsum():
    W = synth.latent_weights(11, 256, 320)
    beta, mean64 = oracle.absmean_beta(W, return_mean64=True)
    exact = math.fsum(abs(float(v)) for v in W.reshape(-1)) / W.size
    assert abs(mean64 - exact) <= 4e-16 * exact
    assert beta == np.float32(exact)
    assert oracle.beta_guard_ok(mean64)


def test_beta_closed_form_gaussian():
    W = synth.latent_weights(0, 2560, 2560)
    beta = oracle.absmean_beta(W)
    # E|N(0,s^2)| = s*sqrt(2/pi); sampling sd of the mean ~ s*0.6/sqrt(NK)
    assert abs(float(beta) - 0.02 * math.sqrt(2 / math.pi)) < 5 * 0.02 * 0.6 / math.sqrt(W.size)


def test_beta_pathological_sum_needs_fp64():
    # 1 followed by many tiny terms: a float32 running sum would drop them all
    W = np.full((64, 1024), 1e-8, dtype=np.float32)
    W[0, 0] = 1.0
    beta = oracle.absmean_beta(W)
    exact = math.fsum(float(v) for v in W.reshape(-1)) / W.size
    assert beta == np.float32(exact)


def _beta_with_pow2_divisor(target):
    """A beta whose fp32 (beta + 1e-5f) is exactly `target` (a power of two)."""
    eps = np.float32(1e-5)
    b = np.float32(target) - eps
    for _ in range(64):
        d = np.float32(b + eps)
        if d == np.float32(target):
            return b
        b = np.nextafter(b, np.float32(np.inf) if d < target else np.float32(-np.inf))
    raise AssertionError("no beta found")


def test_ternarize_golden_ties():
    d = 2.0 ** -6
    beta = _beta_with_pow2_divisor(d)
    rows = [ln.split() for ln in _rows("ternary_ties.txt")]
    r = np.array([float(a) for a, _ in rows], dtype=np.float32)
    want = np.array([int(b) for _, b in rows], dtype=np.int8)
    W = np.zeros((4, 64), dtype=np.float32)
    W[0, : r.size] = r * np.float32(d)  # exact: power-of-two scaling
    Wt = oracle.ternarize(W, beta)
    assert np.array_equal(Wt[0, : r.size], want), (Wt[0, : r.size], want)
    assert not Wt[1:].any()


def test_ternarize_all_zero_matrix():
    W = np.zeros((8, 64), dtype=np.float32)
    beta = oracle.absmean_beta(W)
    assert beta == 0.0
    assert not oracle.ternarize(W, beta).any()


def test_ternarize_invariants_and_zero_fraction():
    W = synth.latent_weights(0, 2560, 2560)
    beta = oracle.absmean_beta(W)
    Wt = oracle.ternarize(W, beta)
    assert set(np.unique(Wt).tolist()) == {-1, 0, 1}  # Section 2: ternary values
    nz = Wt != 0
    assert np.array_equal(np.sign(W[nz]).astype(np.int8), Wt[nz])  # sign preserved
    # threshold structure: everything below the largest zeroed |W| ... monotone
    a = np.abs(W)
    assert a[~nz].max() <= a[nz].min()
    # the threshold is |W| = d/2
    d = float(np.float32(beta) + np.float32(1e-5))
    assert abs(a[~nz].max() - d / 2) < 1e-6 and abs(a[nz].min() - d / 2) < 1e-6
    # closed form for N(0, 0.02^2): P(|W| < d/2) = erf(d/(2*sigma*sqrt 2))
    p0 = math.erf(d / (2 * 0.02 * math.sqrt(2)))
    assert abs(p0 - 0.3102) < 2e-3
    frac0 = 1.0 - nz.mean()
    assert abs(frac0 - p0) < 5 * math.sqrt(p0 * (1 - p0) / W.size)
    assert abs((Wt == 1).mean() - (Wt == -1).mean()) < 5 / math.sqrt(W.size)


def test_ternarize_matches_numpy_float32_division():
    W = synth.latent_weights(2, 128, 256)
    beta = oracle.absmean_beta(W)
    d = np.float32(beta) + np.float32(1e-5)
    want = np.clip(np.rint(W / d), -1, 1).astype(np.int8)
    assert np.array_equal(oracle.ternarize(W, beta), want)


# ----------------------------------------------------- activation quantiser
def test_bf16_narrowing_matches_torch_cast():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 7,
                        np.array([1.00390625, 1.01171875, -1.00390625, 0.0, 3.140625, 65280.0], dtype=np.float32),
                        # exact ties between two bf16 neighbours, both parities
                        (np.arange(256, 512, dtype=np.uint32) << 16 | 0x8000).view(np.float32)])
    got = oracle.f32_to_bf16(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    assert np.array_equal(synth.bf16_bits_to_f32(got), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_quant_golden_rows():
    for ln in _rows("quant_rows.txt"):
        xs, qs = ln.split("|")
        x = np.array([float(t) for t in xs.split()], dtype=np.float32)
        want = np.array([int(t) for t in qs.split()], dtype=np.int8)
        K = 64
        xp = np.zeros((1, K), dtype=np.float32)
        xp[0, : x.size] = x
        bits = oracle.f32_to_bf16(xp)
        assert np.array_equal(synth.bf16_bits_to_f32(bits), xp)  # inputs exact in bf16
        q, scale, rowsum = oracle.quant_act(bits)
        assert np.array_equal(q[0, : x.size], want), (q[0, : x.size], want)
        assert not q[0, x.size:].any()
        assert rowsum[0] == int(want.astype(np.int32).sum())
        g = max(float(np.abs(x).max()), float(np.float32(1e-5)))
        assert scale[0] == np.float32(np.float32(g) / np.float32(127.0))


def test_quant_invariants_config_inputs():
    X = synth.activations_bf16(0, 16, 2560)
    x = synth.bf16_bits_to_f32(X)
    q, scale, rowsum = oracle.quant_act(X)
    assert q.dtype == np.int8 and np.abs(q.astype(np.int32)).max() <= 127
    am = np.abs(x).argmax(axis=1)
    assert np.all(np.abs(q[np.arange(16), am].astype(np.int32)) == 127)  # absmax hits 127
    nzq = q != 0
    assert np.array_equal(np.sign(x[nzq]).astype(np.int8), np.sign(q[nzq]))
    assert np.array_equal(rowsum, q.astype(np.int64).sum(axis=1).astype(np.int32))
    assert np.array_equal(scale, (np.abs(x).max(axis=1) / np.float32(127)).astype(np.float32))
    # monotone within a row
    for m in range(4):
        o = np.argsort(x[m], kind="stable")
        assert np.all(np.diff(q[m][o].astype(np.int32)) >= 0)
    # outlier channels dominate: most entries are small
    assert np.percentile(np.abs(q.astype(np.int32)), 90) <= 8
    # dequantisation error bound: |q*scale - x| <= scale/2 (+ rounding slack)
    err = np.abs(q.astype(np.float64) * scale[:, None].astype(np.float64) - x.astype(np.float64))
    assert np.all(err <= 0.5 * scale[:, None] * (1 + 1e-5))


def test_quant_matches_numpy_float32_ops():
    X = synth.activations_bf16(4, 8, 6912, matrix="down", relu2=True)
    x = synth.bf16_bits_to_f32(X)
    q, scale, _ = oracle.quant_act(X)
    g = np.maximum(np.abs(x).max(axis=1), np.float32(1e-5)).astype(np.float32)
    inv = (np.float32(127.0) / g).astype(np.float32)
    want = np.clip(np.rint(x * inv[:, None]), -127, 127).astype(np.int8)
    assert np.array_equal(q, want)
    assert q.min() >= 0  # ReLU^2 inputs are non-negative
    assert (q == 0).mean() > 0.45


def test_quant_power_of_two_equivariance_and_row_independence():
    X = synth.activations_bf16(7, 6, 256)
    x = synth.bf16_bits_to_f32(X)
    q, scale, _ = oracle.quant_act(X)
    X4 = oracle.f32_to_bf16(x * np.float32(4.0))
    q4, scale4, _ = oracle.quant_act(X4)
    assert np.array_equal(q, q4) and np.array_equal(scale4, scale * np.float32(4.0))
    perm = np.array([3, 0, 5, 1, 4, 2])
    qp, sp, _ = oracle.quant_act(X[perm])
    assert np.array_equal(qp, q[perm]) and np.array_equal(sp, scale[perm])


def test_quant_zero_row_gives_zero_and_no_nan():
    X = np.zeros((2, 128), dtype=np.uint16)
    q, scale, rowsum = oracle.quant_act(X)
    assert not q.any() and not rowsum.any()
    assert np.all(scale == np.float32(np.float32(1e-5) / np.float32(127.0)))


# --------------------------------------------------------------- contraction
def _small_case(seed, M, N, K):
    q = synth.uniform_i8(seed, (M, K), -127, 127, stream=1)
    Wt = synth.uniform_i8(seed, (N, K), -1, 1, stream=2)
    return q, Wt


def test_matmul_equals_int64_library_matmul():
    q, Wt = _small_case(1, 5, 48, 320)
    acc = oracle.matmul_i32(q, Wt)
    want = torch.from_numpy(q).long() @ torch.from_numpy(Wt).long().T
    assert np.array_equal(acc.astype(np.int64), want.numpy())
    # transposed-operand mistake would fail on this non-square case
    assert acc.shape == (5, 48)


def test_matmul_special_cases():
    M, N, K = 3, 8, 128
    q, _ = _small_case(2, M, N, K)
    ones = np.ones((N, K), dtype=np.int8)
    assert np.array_equal(oracle.matmul_i32(q, ones), np.repeat(q.astype(np.int32).sum(1)[:, None], N, 1))
    assert np.array_equal(oracle.matmul_i32(q, -ones), -oracle.matmul_i32(q, ones))
    # one-hot weight rows select one activation
    sel = np.array([5, 0, 127, 64, 3, 3, 99, 1])
    Wt = np.zeros((N, K), dtype=np.int8)
    Wt[np.arange(N), sel] = 1
    assert np.array_equal(oracle.matmul_i32(q, Wt), q[:, sel].astype(np.int32))
    # x = gamma * e_k reads back column k of the weights times 127
    _, Wr = _small_case(3, 1, 16, K)
    for k in (0, 17, 127):
        e = np.zeros((1, K), dtype=np.int8)
        e[0, k] = 127
        assert np.array_equal(oracle.matmul_i32(e, Wr)[0], 127 * Wr[:, k].astype(np.int32))
    assert not oracle.matmul_i32(np.zeros((2, K), np.int8), Wr).any()


def test_matmul_linearity_bound_and_token_independence():
    M, N, K = 4, 32, 256
    q1 = synth.uniform_i8(4, (M, K), -60, 60, stream=1)
    q2 = synth.uniform_i8(4, (M, K), -60, 60, stream=2)
    _, Wt = _small_case(4, M, N, K)
    a1, a2 = oracle.matmul_i32(q1, Wt), oracle.matmul_i32(q2, Wt)
    assert np.array_equal(oracle.matmul_i32((q1 + q2).astype(np.int8), Wt), a1 + a2)
    assert np.abs(a1).max() <= 127 * K
    for m in range(M):
        assert np.array_equal(oracle.matmul_i32(q1[m:m + 1], Wt)[0], a1[m])
    ms = np.array([0, 3, 2, 1]); ns = np.array([31, 0, 7, 16])
    assert np.array_equal(oracle.matmul_i32_sampled(q1, Wt, ms, ns), a1[ms, ns])


def test_layer_against_fp64_brute_force_of_dequantised_operands():
    """y must equal sum_k (beta*Wt)(q*scale) computed in fp64, to 1e-6 relative."""
    M, N, K = 4, 24, 192
    W = synth.latent_weights(9, N, K)
    X = synth.activations_bf16(9, M, K)
    beta = oracle.absmean_beta(W)
    Wt = oracle.ternarize(W, beta)
    r = oracle.bitlinear(X, Wt, beta)
    Wd = float(beta) * Wt.astype(np.float64)
    xd = r["q"].astype(np.float64) * r["scale"].astype(np.float64)[:, None]
    want = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            s = 0.0
            for k in range(K):
                s += Wd[n, k] * xd[m, k]
            want[m, n] = s
    nz = want != 0
    assert np.all(np.abs(r["y"][nz] - want[nz]) <= 1e-6 * np.abs(want[nz]))
    assert np.all(r["y"][~nz] == 0)
    # and the layer approximates the unquantised product x @ W^T (sanity, loose)
    ref = synth.bf16_bits_to_f32(X).astype(np.float64) @ W.astype(np.float64).T
    assert np.corrcoef(ref.reshape(-1), r["y"].reshape(-1))[0, 1] > 0.8


def test_rescale_against_fp64():
    acc = np.array([[0, 1, -1, 877824, -877824, 12345]], dtype=np.int32)
    beta = np.float32(0.0159577)
    scale = np.array([39.25 / 127], dtype=np.float32)
    y = oracle.rescale(acc, beta, scale)
    want = acc.astype(np.float64) * float(beta) * float(scale[0])
    assert y[0, 0] == 0.0 and not np.signbit(y[0, 0])
    nz = want != 0
    assert np.all(np.abs(y[nz] - want[nz]) <= 1e-6 * np.abs(want[nz]))
    # the order is (beta*scale) first: one rounding, then one more
    c = np.float32(beta * scale[0])
    assert np.array_equal(y[0], acc[0].astype(np.float32) * c)


# ---------------------------------------------------------------- chain glue
def test_chain_glue_against_torch():
    rng = np.random.default_rng(5)
    M = 3
    qkv = rng.standard_normal((M, 3840)).astype(np.float32)
    a = oracle.chain_attn_stub(qkv)
    v = torch.from_numpy(qkv)[:, 3200:].reshape(M, 5, 1, 128).expand(M, 5, 4, 128).reshape(M, 2560)
    assert np.array_equal(a, v.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    gu = rng.standard_normal((M, 2 * 6912)).astype(np.float32)
    f = oracle.chain_relu2_gate(gu)
    g, u = torch.from_numpy(gu[:, :6912]), torch.from_numpy(gu[:, 6912:])
    r = torch.relu(g)
    want = ((r * r) * u).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(f, want)
    x, y = qkv[:, :2560], qkv[:, 100:2660]
    assert np.array_equal(oracle.chain_residual(x, y), x + y)
    # the fp32 forms used in front of the normalisation: the same maps without the narrowing
    assert np.array_equal(oracle.chain_attn_f32(qkv).view(np.uint32), v.contiguous().numpy().view(np.uint32))
    assert np.array_equal(oracle.chain_relu2_gate_f32(gu).view(np.uint32), ((r * r) * u).numpy().view(np.uint32))
    # a wrong head mapping or operand order would show: V of kv head 1 feeds q heads 4..7 only
    probe = np.zeros((1, 3840), np.float32)
    probe[0, 3200 + 128 + 5] = 2.5
    a32 = oracle.chain_attn_f32(probe)
    assert sorted(np.nonzero(a32[0])[0].tolist()) == [h * 128 + 5 for h in range(4, 8)]
    gate = np.zeros((1, 8), np.float32)
    gate[0, :4] = [-3.0, 2.0, 0.5, 0.0]
    gate[0, 4:] = [7.0, -1.5, 4.0, 9.0]
    assert oracle.chain_relu2_gate_f32(gate)[0].tolist() == [0.0, -6.0, 1.0, 0.0]


def test_chain_layer_stays_bounded_and_is_token_independent():
    H, F = 256, 512  # reduced widths; head layout 4 q heads, 1 kv head, dim 64
    shapes = {"qkv": (H + 2 * 64, H), "o": (H, H), "gate_up": (2 * F, H), "down": (H, F)}

    def layer_weights(layer):
        out = {}
        for name, (N, K) in shapes.items():
            W = synth.latent_weights(1, N, K, layer=layer, matrix=name)
            beta = oracle.absmean_beta(W)
            out[name] = (oracle.ternarize(W, beta), beta)
        return out

    # monkey-free small-geometry variant of chain_layer
    def run(x, layers):
        for wts in layers:
            def bl(name, xb):
                Wt, beta = wts[name]
                return oracle.bitlinear(xb, Wt, beta, unit_scale=True)["y"]
            qkv = bl("qkv", oracle.f32_to_bf16(x))
            o = bl("o", oracle.chain_attn_stub(qkv, n_q=4, n_kv=1, hd=64))
            h1 = oracle.chain_residual(x, o)
            gu = bl("gate_up", oracle.f32_to_bf16(h1))
            x = oracle.chain_residual(h1, bl("down", oracle.chain_relu2_gate(gu)))
        return x

    layers = [layer_weights(l) for l in range(6)]
    x0 = synth.bf16_bits_to_f32(synth.activations_bf16(1, 4, H))
    out = run(x0, layers)
    assert np.all(np.isfinite(out)) and np.abs(out).max() < 1e4
    one = run(x0[2:3], layers)
    assert np.array_equal(one[0], out[2])


def test_chain_layer_wiring_and_products_at_full_geometry():
    """chain_layer at the 2B geometry, two tokens, checked from outside: the input of every
    BitLinear it records must be what plain numpy index arithmetic makes of the recorded outputs
    before it (V of KV head h // 4 for query head h, fp32 sums in the stated operand order, gate
    and up halves), and every product, teacher-forced on the recorded input, must agree with an
    fp64 contraction of the operands scaled afterwards, (Wt . q) * beta / 127."""
    import torch

    def bf16(a):            # round-to-nearest-even narrowing by the library cast (pinned elsewhere against the oracle's own)
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)

    wts = {}
    for name, (N, K) in synth.LAYER_SHAPES.items():
        W = synth.latent_weights(3, N, K, layer=7, matrix=name)
        beta = oracle.absmean_beta(W)
        wts[name] = (oracle.ternarize(W, beta), beta)
    x = synth.bf16_bits_to_f32(synth.activations_bf16(3, 2, 2560, layer=7))
    tr = []
    out = oracle.chain_layer(x, wts, trace=tr)
    assert [t["name"] for t in tr] == ["qkv", "o", "gate_up", "down"]
    qkv, o, gu, dn = (t["y"] for t in tr)
    # wiring
    assert np.array_equal(tr[0]["x_bf16"], bf16(x))
    heads = np.arange(20)
    v = qkv[:, 3200:].reshape(2, 5, 128)[:, heads // 4, :].reshape(2, 2560)      # [Q 20x128 | K 5x128 | V 5x128]
    assert np.array_equal(tr[1]["x_bf16"], bf16(v))
    h1 = x + o
    assert np.array_equal(tr[2]["x_bf16"], bf16(h1))
    g, u = gu[:, :6912], gu[:, 6912:]
    r = np.maximum(g, np.float32(0.0))
    assert np.array_equal(tr[3]["x_bf16"], bf16((r * r) * u))
    assert np.array_equal(out.view(np.uint32), (h1 + dn).view(np.uint32))
    # products, teacher-forced, in another formulation: fp64 over dequantised operands
    for t in tr:
        Wt, beta = wts[t["name"]]
        xb = synth.bf16_bits_to_f32(t["x_bf16"]).astype(np.float64)
        gamma = np.maximum(np.abs(xb).max(axis=1, keepdims=True), 1e-5)
        q = np.clip(np.rint(xb * (np.float64(np.float32(127.0) / gamma.astype(np.float32)))), -127, 127)
        assert np.array_equal(q.astype(np.int8), t["q"])
        want = (q @ Wt.astype(np.float64).T) * (np.float64(beta) / 127.0)     # integer-valued sums are exact in fp64
        nz = want != 0
        assert np.all(np.abs(t["y"][nz] - want[nz]) <= 1e-6 * np.abs(want[nz]))
        assert np.all(t["y"][~nz] == 0)


# --------------------------------------------------------------- RMS normalisation
def _bf16_to_f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def test_rmsnorm_closed_forms():
    """Rows whose mean square is known exactly (Section 2 names the normalisation; the
    formula pinned here is the bias-free RMS form)."""
    K = 512
    # constant row c: ss = K*c^2 exactly in fp64, r = 1/sqrt(c^2 + eps)
    for c in (1.0, -2.0, 0.5, 3.0):
        t = np.full((1, K), c, dtype=np.float32)
        r = np.float32(1.0 / np.sqrt(np.float64(c) * np.float64(c) + np.float64(np.float32(1e-5))))
        want = oracle.f32_to_bf16(np.full((1, K), np.float32(c) * r, dtype=np.float32))
        assert np.array_equal(oracle.rmsnorm_rows(t, None, 1e-5), want)
    # zero row: r = 1/sqrt(eps) is finite, output exactly +0
    z = oracle.rmsnorm_rows(np.zeros((1, K), np.float32), None, 1e-5)
    assert not z.any()
    # a single spike s at k=3: ss/K = s^2/K; the output there is s*r, elsewhere 0
    t = np.zeros((1, K), np.float32)
    t[0, 3] = 16.0
    r = np.float32(1.0 / np.sqrt(256.0 / K + np.float64(np.float32(1e-5))))
    out = _bf16_to_f32(oracle.rmsnorm_rows(t, None, 1e-5))
    assert out[0, 3] == _bf16_to_f32(oracle.f32_to_bf16(np.array([np.float32(16.0) * r])))[0]
    assert not np.delete(out[0], 3).any()
    # eps sits inside the root, added to the MEAN (not the sum): with eps = 3 and a unit row, r = 1/2
    t = np.ones((2, 64), np.float32)
    assert np.all(_bf16_to_f32(oracle.rmsnorm_rows(t, None, 3.0)) == 0.5)


def test_rmsnorm_against_fp64_formula_and_gains():
    rng = np.random.default_rng(5)
    for K in (64, 2560, 6912):
        t = (rng.standard_normal((5, K)) * rng.uniform(0.1, 30.0, size=(5, 1))).astype(np.float32)
        t[:, 1] *= 50.0
        g = (1.0 + 0.3 * rng.standard_normal(K)).astype(np.float32)
        ref = t.astype(np.float64) / np.sqrt((t.astype(np.float64) ** 2).mean(axis=1, keepdims=True) + 1e-5)
        for gain, refg in ((None, ref), (g, ref * g.astype(np.float64))):
            out = _bf16_to_f32(oracle.rmsnorm_rows(t, gain, 1e-5)).astype(np.float64)
            # bf16 keeps 8 significant bits: half an ulp is at most 2^-8 relative; the fp32 steps add ~1e-7
            assert np.all(np.abs(out - refg) <= np.abs(refg) * (2.0 ** -8 + 1e-6) + 1e-30)
            assert np.mean(np.abs(out - refg) <= np.abs(refg) * 2.0 ** -9) > 0.6   # and usually half of that
        # rows are independent and the gain is elementwise
        one = oracle.rmsnorm_rows(t[2:3], g, 1e-5)
        assert np.array_equal(one, oracle.rmsnorm_rows(t, g, 1e-5)[2:3])
    # the sum of squares is the exactly rounded one: math.fsum of the exact fp64 squares
    import math
    for K in (64, 2560, 6912):
        t = (rng.standard_normal((4, K)) * 1e3).astype(np.float32)
        _, r64 = oracle.rmsnorm_rows(t, None, 1e-5, return_r64=True)
        for m in range(4):
            ss = math.fsum(float(v) * float(v) for v in t[m])
            want = 1.0 / math.sqrt(ss / K + float(np.float32(1e-5)))
            assert abs(r64[m] - want) <= 4e-16 * want
    # the guard trips exactly when the factor sits at an fp32 rounding midpoint
    f = np.float32(0.3)
    mid = (float(f) + float(np.nextafter(f, np.float32(1)))) / 2.0
    assert not oracle.fp32_rounding_guard_ok(mid) and not oracle.fp32_rounding_guard_ok(mid * (1 + 5e-12))
    assert oracle.fp32_rounding_guard_ok(mid * (1 + 1e-9)) and oracle.fp32_rounding_guard_ok(float(f))
    # unit RMS after normalisation (before narrowing the mean square is 1 up to eps)
    t = rng.standard_normal((3, 4096)).astype(np.float32) * 7
    out = _bf16_to_f32(oracle.rmsnorm_rows(t, None, 1e-5)).astype(np.float64)
    assert np.all(np.abs(np.sqrt((out ** 2).mean(axis=1)) - 1.0) < 2e-3)


def test_padded_pack_is_plain_pack_of_the_zero_padded_matrix():
    """The library's format for a ragged K or N: weight 0 (code 1) outside the matrix, rows of
    ceil(K/64)*64 weights, ceil(N/4)*4 rows.  Pinned by decoding the bytes by hand (layout 0: two
    bits per weight, lowest bits = lowest k) and by the round trip through unpack."""
    rng = np.random.default_rng(3)
    for N, K in [(1, 1), (3, 17), (5, 65), (8, 64), (6, 130)]:
        Wt = rng.integers(-1, 2, size=(N, K)).astype(np.int8)
        Np, Kp = -(-N // 4) * 4, oracle.padded_k(K)
        assert Kp % 64 == 0 and Kp >= K and Kp - K < 64
        for layout in (0, 1):
            p = oracle.pack_padded(Wt, layout)
            assert p.size == Np * Kp // 4
            back, bad = oracle.unpack(p, Np, Kp, layout)
            assert bad == 0
            assert np.array_equal(back[:N, :K], Wt)
            assert not back[N:].any() and not back[:, K:].any()
        p0 = oracle.pack_padded(Wt, 0).reshape(Np, Kp // 4)
        for n in range(Np):
            for k in range(Kp):
                code = (int(p0[n, k // 4]) >> (2 * (k % 4))) & 3
                assert code == (int(Wt[n, k]) + 1 if n < N and k < K else 1)
    Wt = rng.integers(-1, 2, size=(8, 128)).astype(np.int8)
    for layout in (0, 1):
        assert np.array_equal(oracle.pack_padded(Wt, layout), oracle.pack(Wt, layout))
    q = rng.integers(-127, 128, size=(3, 70)).astype(np.int8)
    pq = oracle.pad_q(q)
    assert pq.shape == (3, 128) and np.array_equal(pq[:, :70], q) and not pq[:, 70:].any()


def test_trit5_codes_exhaustive_and_hand_worked():
    """Five weights per byte.  Hand-worked bytes: all weights 0 -> codes 1,1,1,1,1 -> v = 81+27+9+3+1 = 121
    -> ceil(121*256/243) = ceil(127.47) = 128; all -1 -> v = 0 -> 0; all +1 -> v = 242 -> ceil(254.95) = 255;
    leading weight +1, rest -1 -> v = 2*81 = 162 -> ceil(170.67) = 171.  Then every one of the 243 digit
    strings, with the digits taken by plain integer division as the reference for the multiply-by-3 rule."""
    def one_byte(ws):      # ws: the five weights of byte 0 of word 0 = k 0, 4, 8, 12, 16
        Wt = np.zeros((1, 20), dtype=np.int8)
        Wt[0, 0:20:4] = ws
        return int(oracle.pack_trit5(Wt)[0])
    assert one_byte([0, 0, 0, 0, 0]) == 128
    assert one_byte([-1, -1, -1, -1, -1]) == 0
    assert one_byte([1, 1, 1, 1, 1]) == 255
    assert one_byte([1, -1, -1, -1, -1]) == 171
    seen = set()
    for v in range(243):
        digits = [(v // 3 ** (4 - i)) % 3 for i in range(5)]
        b = one_byte([d - 1 for d in digits])
        assert b == -(-v * 256 // 243) and 0 <= b <= 255
        seen.add(b)
        r, out = b, []
        for _ in range(5):
            t = r * 3
            out.append(t >> 8)
            r = t & 255
        assert out == digits
    assert len(seen) == 243                                   # distinct bytes: the code is invertible


def test_trit5_positions_padding_and_round_trip():
    """A single +1 at position k lands in word k // 20, byte (k % 20) % 4, digit (k % 20) // 4; padding
    decodes to weight 0; sizes are Np * ceil(K/80)*80 / 5; random matrices survive the round trip."""
    N, K = 3, 100
    Np, Kq = 4, 160
    zero_byte = 128
    for (n, k) in [(0, 0), (0, 1), (0, 4), (0, 19), (0, 20), (2, 99), (1, 57)]:
        Wt = np.zeros((N, K), dtype=np.int8)
        Wt[n, k] = 1
        p = oracle.pack_trit5(Wt).reshape(Np, Kq // 5)
        assert p.size == Np * Kq // 5
        g, j, i = k // 20, (k % 20) % 4, (k % 20) // 4
        want = np.full((Np, Kq // 5), zero_byte, dtype=np.uint8)
        want[n, 4 * g + j] = -(-(121 + 3 ** (4 - i)) * 256 // 243)
        assert np.array_equal(p, want)
    rng = np.random.default_rng(11)
    for N, K in [(1, 1), (4, 80), (5, 81), (7, 2560), (2, 6912)]:
        Wt = rng.integers(-1, 2, size=(N, K)).astype(np.int8)
        p = oracle.pack_trit5(Wt)
        assert p.size == (-(-N // 4) * 4) * oracle.padded_k5(K) // 5
        back, bad = oracle.unpack_trit5(p, N, K)
        assert bad == 0 and np.array_equal(back, Wt)
    assert oracle.padded_k5(2560) == 2560 and oracle.padded_k5(6912) == 6960
    p = oracle.pack_trit5(np.zeros((4, 80), dtype=np.int8)).copy()
    p[3] = 129                                                # 129 -> digits of v = 122 -> re-encodes to 129: valid
    p[5] = 1                                                  # 1 is not ceil(v*256/243) of any v (v=0 -> 0, v=1 -> 2)
    assert oracle.unpack_trit5(p, 4, 80)[1] == 1


def test_kmajor_form_is_the_packed_transpose():
    """Layout 3 by hand: weight (n, k) sits in byte k*(Nq/4) + n/4 at bits 2*(n%4); padding decodes to 0."""
    rng = np.random.default_rng(17)
    N, K = 70, 9
    Wt = rng.integers(-1, 2, size=(N, K)).astype(np.int8)
    p = oracle.pack_kmajor(Wt)
    Nq = 128
    assert p.size == K * Nq // 4
    for k in range(K):
        for n in range(Nq):
            code = (int(p[k * (Nq // 4) + n // 4]) >> (2 * (n % 4))) & 3
            assert code == (int(Wt[n, k]) + 1 if n < N else 1)
    back, bad = oracle.unpack_kmajor(p, N, K)
    assert bad == 0 and np.array_equal(back, Wt)
