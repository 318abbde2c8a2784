"""GPU parity of the fused producers and of the synthetic layer chain
(benchmark config 4) against the CPU oracle."""
import sys

import numpy as np
import pytest

import oracle
import synth
from helpers import assert_y_close, to_dev

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

SHAPES = synth.LAYER_SHAPES


@pytest.fixture(scope="module")
def bl():
    from paper_2504_12285_amd import binding
    binding.load()
    return binding


@pytest.fixture(scope="module")
def chain():
    from paper_2504_12285_amd import chain as c
    return c


def _layer_weights(seed, layer):
    """Oracle-side (Wt, beta) and latent W of the four matrices of one layer."""
    out = {}
    for name, (N, K) in SHAPES.items():
        W = synth.latent_weights(seed, N, K, layer=layer, matrix=name)
        beta, mean64 = oracle.absmean_beta(W, return_mean64=True)
        assert oracle.beta_guard_ok(mean64)
        out[name] = (oracle.ternarize(W, beta), beta, W)
    return out


def _to_gpu_weights(bl, ow, layout=1):
    gw = {}
    for name, (Wt, beta, W) in ow.items():
        packed, b = bl.bl_pack_ternary(to_dev(W), layout)
        gw[name] = (packed, b)
    return gw


# ------------------------------------------------------------------ producers
@pytest.mark.parametrize("M", [1, 5])
def test_producers_match_oracle_glue(bl, M):
    rng = np.random.default_rng(7)
    dev = "cuda:0"
    x = (rng.standard_normal((M, 2560)) * 3).astype(np.float32)
    o = rng.standard_normal((M, 2560)).astype(np.float32)
    qkv = rng.standard_normal((M, 3840)).astype(np.float32)
    gu = rng.standard_normal((M, 13824)).astype(np.float32)
    gu[:, 5] = 0.0
    # the descriptor holds raw pointers: keep the device tensors alive in `keep`
    keep = dict(x=to_dev(x), qkv=to_dev(qkv), gu=to_dev(gu), xb=to_dev(oracle.f32_to_bf16(x)))
    cases = [
        (bl.make_producer(bl.BL_PROD_F32, keep["x"]), 2560, oracle.f32_to_bf16(x)),
        (bl.make_producer(bl.BL_PROD_ATTN_V, keep["qkv"], n_q=20, n_kv=5, head_dim=128), 2560,
         oracle.chain_attn_stub(qkv)),
        (bl.make_producer(bl.BL_PROD_RELU2_GATE, keep["gu"]), 6912, oracle.chain_relu2_gate(gu)),
        (bl.make_producer(bl.BL_PROD_BF16, keep["xb"]), 2560, oracle.f32_to_bf16(x)),
    ]
    for prod, K, want_bits in cases:
        q_o, s_o, r_o = oracle.quant_act(want_bits)
        q, s, r = bl.bl_quant_act_ex(prod, M, K, dev)
        torch.cuda.synchronize()
        assert np.array_equal(q.cpu().numpy(), q_o)
        assert np.array_equal(s.cpu().numpy().view(np.uint32), s_o.view(np.uint32))
        assert np.array_equal(r.cpu().numpy(), r_o)
    # residual: also stores the fp32 sum
    xd, od = to_dev(x), to_dev(o)
    h1 = torch.empty((M, 2560), dtype=torch.float32, device=dev)
    q, s, r = bl.bl_quant_act_ex(bl.make_producer(bl.BL_PROD_RESIDUAL, xd, od, h1), M, 2560, dev)
    torch.cuda.synchronize()
    h1_o = oracle.chain_residual(x, o)
    assert np.array_equal(h1.cpu().numpy().view(np.uint32), h1_o.view(np.uint32))
    q_o, s_o, _ = oracle.quant_act(oracle.f32_to_bf16(h1_o))
    assert np.array_equal(q.cpu().numpy(), q_o) and np.array_equal(s.cpu().numpy(), s_o)


def _gain(seed, K):
    """Synthetic gains around 1 (no trained gains exist here)."""
    return (1.0 + 0.25 * np.random.default_rng(seed).standard_normal(K)).astype(np.float32)


@pytest.mark.parametrize("M", [1, 3, 6])
@pytest.mark.parametrize("with_gain", [False, True])
def test_normalising_producers_match_oracle(bl, M, with_gain):
    """RMS normalisation in front of the quantiser, every producer kind, through the
    prefill quantiser kernel and through the fused decode kernels (dot4 and matrix-core)."""
    rng = np.random.default_rng(11)
    dev = "cuda:0"
    x = (rng.standard_normal((M, 2560)) * 3).astype(np.float32)
    x[:, 7] *= 40.0
    o = rng.standard_normal((M, 2560)).astype(np.float32)
    qkv = rng.standard_normal((M, 3840)).astype(np.float32)
    gu = rng.standard_normal((M, 13824)).astype(np.float32)
    xb = oracle.f32_to_bf16(x)
    keep = dict(x=to_dev(x), o=to_dev(o), qkv=to_dev(qkv), gu=to_dev(gu), xb=to_dev(xb),
                h1=torch.empty((M, 2560), dtype=torch.float32, device=dev))
    gains = {K: (_gain(K, K) if with_gain else None) for K in (2560, 6912)}
    dgain = {K: (to_dev(g) if g is not None else None) for K, g in gains.items()}
    nk = lambda K: dict(norm=True, gain=dgain[K], eps=1e-5)
    cases = [
        ("f32", bl.make_producer(bl.BL_PROD_F32, keep["x"], **nk(2560)), 2560, x),
        ("attn", bl.make_producer(bl.BL_PROD_ATTN_V, keep["qkv"], n_q=20, n_kv=5, head_dim=128, **nk(2560)), 2560,
         oracle.chain_attn_f32(qkv)),
        ("relu2", bl.make_producer(bl.BL_PROD_RELU2_GATE, keep["gu"], **nk(6912)), 6912,
         oracle.chain_relu2_gate_f32(gu)),
        ("bf16", bl.make_producer(bl.BL_PROD_BF16, keep["xb"], **nk(2560)), 2560, synth.bf16_bits_to_f32(xb)),
        ("residual", bl.make_producer(bl.BL_PROD_RESIDUAL, keep["x"], keep["o"], keep["h1"], **nk(2560)), 2560,
         oracle.chain_residual(x, o)),
    ]
    N = 128
    for name, prod, K, t in cases:
        want_bits = oracle.rmsnorm_rows(t, gains[K], 1e-5)
        q_o, s_o, r_o = oracle.quant_act(want_bits)
        q, s, r = bl.bl_quant_act_ex(prod, M, K, dev)
        torch.cuda.synchronize()
        assert np.array_equal(q.cpu().numpy(), q_o), name
        assert np.array_equal(s.cpu().numpy().view(np.uint32), s_o.view(np.uint32)), name
        assert np.array_equal(r.cpu().numpy(), r_o), name
        if name == "residual":
            assert np.array_equal(keep["h1"].cpu().numpy().view(np.uint32), t.view(np.uint32))
        # the same producer inside the decode kernel
        Wt = synth.uniform_i8(60, (N, K), -1, 1)
        ref = oracle.bitlinear(want_bits, Wt, np.float32(0.75))
        it = dict(packed=to_dev(oracle.pack(Wt, 1)), beta=to_dev(np.array([0.75], dtype=np.float32)), N=N, K=K,
                  prod=prod, acc=torch.empty((M, N), dtype=torch.int32, device=dev),
                  y=torch.empty((M, N), dtype=torch.float32, device=dev),
                  q_out=torch.empty((M, K), dtype=torch.int8, device=dev),
                  scale_out=torch.empty(M, dtype=torch.float32, device=dev))
        bl.bl_bitlinear_decode_group(bl.make_decode_descs([it]), 1, M)
        torch.cuda.synchronize()
        assert np.array_equal(it["q_out"].cpu().numpy(), ref["q"]), name
        assert np.array_equal(it["scale_out"].cpu().numpy(), ref["scale"]), name
        assert np.array_equal(it["acc"].cpu().numpy(), ref["acc"]), name
        assert_y_close(it["y"].cpu().numpy(), ref["y"])


def test_bad_producer_is_rejected(bl):
    x = torch.zeros((1, 2560), device="cuda:0")
    with pytest.raises(bl.BitLinearError):
        bl.bl_quant_act_ex(bl.make_producer(9, x), 1, 2560, "cuda:0")
    with pytest.raises(bl.BitLinearError):   # head geometry does not give K
        bl.bl_quant_act_ex(bl.make_producer(bl.BL_PROD_ATTN_V, x, n_q=20, n_kv=5, head_dim=64), 1, 2560, "cuda:0")
    with pytest.raises(bl.BitLinearError):   # residual needs a second operand
        bl.bl_quant_act_ex(bl.make_producer(bl.BL_PROD_RESIDUAL, x), 1, 2560, "cuda:0")


# ---------------------------------------------------------------------- chain
def _oracle_chain(x0, layers, layer_gains=None):
    x = x0
    traces = []
    for li, ow in enumerate(layers):
        tr = []
        x = oracle.chain_layer(x, {k: (v[0], v[1]) for k, v in ow.items()}, trace=tr,
                               gains=None if layer_gains is None else layer_gains[li])
        traces.append(tr)
    return x, traces


def _compare_records(recs, traces, rows=None):
    for lrec, ltr in zip(recs, traces):
        for r, t in zip(lrec, ltr):
            assert r["name"] == t["name"]
            sel = slice(None) if rows is None else rows
            assert np.array_equal(r["q"].cpu().numpy()[sel], t["q"]), ("q", t["name"])
            assert np.array_equal(r["scale"].cpu().numpy()[sel], t["scale"]), ("scale", t["name"])
            assert np.array_equal(r["acc"].cpu().numpy()[sel], t["acc"]), ("acc", t["name"])


@pytest.mark.parametrize("mode,M", [("decode", 1), ("decode", 4), ("decode", 9), ("prefill", 4), ("prefill", 150)])
def test_chain_two_layers(bl, chain, mode, M):
    layers = [_layer_weights(3, l) for l in range(2)]
    gws = [_to_gpu_weights(bl, ow) for ow in layers]
    x0 = synth.bf16_bits_to_f32(synth.activations_bf16(3, M, 2560, layer=99))
    want, traces = _oracle_chain(x0, layers)
    recs = []
    got = chain.run_chain(gws, 1, to_dev(x0), mode=mode, records=recs)
    torch.cuda.synchronize()
    _compare_records(recs, traces)
    assert_y_close(got.cpu().numpy(), want)


@pytest.mark.parametrize("mode,M", [("decode", 1), ("decode", 9), ("prefill", 150)])
def test_chain_two_layers_with_normalisation(bl, chain, mode, M):
    """The chain with the RMS normalisation in front of every quantiser and the true
    absmax/127 rescale (no stand-in)."""
    layers = [_layer_weights(4, l) for l in range(2)]
    gws = [_to_gpu_weights(bl, ow) for ow in layers]
    ogains = [{name: _gain(100 * l + i, SHAPES[name][1]) for i, name in enumerate(SHAPES)} for l in range(2)]
    ogains[1]["o"] = None          # a site without gains
    dgains = [{k: (to_dev(v) if v is not None else None) for k, v in g.items()} for g in ogains]
    x0 = synth.bf16_bits_to_f32(synth.activations_bf16(4, M, 2560, layer=98))
    want, traces = _oracle_chain(x0, layers, ogains)
    recs = []
    got = chain.run_chain(gws, 1, to_dev(x0), mode=mode, records=recs, layer_gains=dgains)
    torch.cuda.synchronize()
    _compare_records(recs, traces)
    assert_y_close(got.cpu().numpy(), want)


@pytest.mark.timeout(900)
def test_config4_full_stack_decode_and_prefill(bl, chain):
    """30 layers of the 2B shapes.  Decode at M=1 is compared in full.  Prefill at M=4096 runs in
    full on the GPU and is compared here, through all 30 layers, on one row in every 32-row block
    (128 rows, at a different offset inside each block) plus the first two and the last row
    (tokens are independent in this chain, so the oracle runs just those rows); the comparison of
    every row of every layer is test_config4_prefill_every_row_every_layer below."""
    n_layers, Mp = synth.N_LAYERS, 4096
    blocks = np.arange(Mp // 32)
    sample = np.unique(np.concatenate([blocks * 32 + (blocks * 7 + 3) % 32, [0, 1, Mp - 1]]))
    x_dec = synth.bf16_bits_to_f32(synth.activations_bf16(0, 1, 2560, layer=100))
    x_pre = synth.bf16_bits_to_f32(synth.activations_bf16(0, Mp, 2560, layer=101))
    dev_dec, dev_pre = to_dev(x_dec), to_dev(x_pre)
    o_dec, o_pre = x_dec, x_pre[sample]
    Bd = chain.ChainBuffers(1, dev_dec.device)
    Bp = chain.ChainBuffers(Mp, dev_pre.device)
    for l in range(n_layers):
        ow = _layer_weights(0, l)
        gw = _to_gpu_weights(bl, ow)
        if l == 0:
            for name in SHAPES:
                assert np.array_equal(gw[name][0].cpu().numpy(), oracle.pack(ow[name][0], 1))
                assert gw[name][1].item() == float(ow[name][1])
        wts = {k: (v[0], v[1]) for k, v in ow.items()}
        tr_d, tr_p = [], []
        o_dec = oracle.chain_layer(o_dec, wts, trace=tr_d)
        o_pre = oracle.chain_layer(o_pre, wts, trace=tr_p)
        rec_d, rec_p = [], []
        out = chain.layer_decode(gw, 1, dev_dec, Bd, rec_d)
        Bd.x_next, dev_dec = dev_dec, out
        out = chain.layer_prefill(gw, 1, dev_pre, Bp, rec_p)
        Bp.x_next, dev_pre = dev_pre, out
        torch.cuda.synchronize()
        _compare_records([rec_d], [tr_d])
        _compare_records([rec_p], [tr_p], rows=sample)
        assert_y_close(dev_dec.cpu().numpy(), o_dec)
        assert_y_close(dev_pre.cpu().numpy()[sample], o_pre)
        print("layer %d ok (|x| max %.3g)" % (l, float(np.abs(o_dec).max())), file=sys.stderr, flush=True)
        del gw, ow, wts, rec_p, rec_d


# ------------------------------------------------- fused producer epilogues of the prefill product
@pytest.mark.parametrize("M,N,K", [(150, 384, 1280), (257, 2560, 2560), (64, 128, 128)])
def test_prefill_epilogue_residual(bl, M, N, K):
    """Product + residual + bf16 narrowing + row absmax in the GEMM epilogue, then the one-pass
    quantiser: every output bit for bit against the oracle's separate steps."""
    rng = np.random.default_rng(31)
    Wt = synth.uniform_i8(80, (N, K), -1, 1)
    beta = np.float32(0.0173)
    q = synth.uniform_i8(81, (M, K), -127, 127)
    scale = (rng.uniform(0.5, 2.0, size=M) / 127.0).astype(np.float32)
    rowsum = q.astype(np.int32).sum(axis=1).astype(np.int32)
    res = (rng.standard_normal((M, N)) * 5).astype(np.float32)
    acc_o = oracle.matmul_i32(q, Wt)
    t_o = oracle.chain_residual(res, oracle.rescale(acc_o, beta, scale))
    xb_o = oracle.f32_to_bf16(t_o)
    dev = "cuda:0"
    acc = torch.empty((M, N), dtype=torch.int32, device=dev)
    y = torch.empty((M, N), dtype=torch.float32, device=dev)
    xb = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    absmax = torch.zeros(M, dtype=torch.float32, device=dev)
    bl.bl_gemm_w158a8_fused(to_dev(oracle.pack(Wt, 1)), to_dev(np.array([beta], dtype=np.float32)), 1, to_dev(q),
                            to_dev(scale), to_dev(rowsum), N, bl.BL_EPI_RESIDUAL, xb, absmax, residual=to_dev(res),
                            y=y, acc=acc)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), acc_o)
    assert np.array_equal(y.cpu().numpy().view(np.uint32), t_o.view(np.uint32))
    assert np.array_equal(xb.view(torch.int16).cpu().numpy().view(np.uint16), xb_o)
    want_max = np.abs(synth.bf16_bits_to_f32(xb_o)).max(axis=1)
    assert np.array_equal(absmax.cpu().numpy(), want_max)
    q2, s2, r2 = bl.bl_quant_from_absmax(xb, absmax)
    torch.cuda.synchronize()
    q_o, s_o, r_o = oracle.quant_act(xb_o)
    assert np.array_equal(q2.cpu().numpy(), q_o)
    assert np.array_equal(s2.cpu().numpy().view(np.uint32), s_o.view(np.uint32))
    assert np.array_equal(r2.cpu().numpy(), r_o)
    assert not absmax.cpu().numpy().any()          # cleared for the next product


@pytest.mark.parametrize("M,F,K", [(130, 192, 1280), (300, 6912, 2560), (5, 64, 128)])
def test_prefill_epilogue_relu2_gate(bl, M, F, K):
    """[gate | up] product with the squared-ReLU gate, bf16 narrowing and row absmax in the epilogue."""
    rng = np.random.default_rng(32)
    N = 2 * F
    Wt = synth.uniform_i8(82, (N, K), -1, 1)
    beta = np.float32(0.0161)
    q = synth.uniform_i8(83, (M, K), -127, 127)
    scale = (rng.uniform(0.5, 2.0, size=M) / 127.0 / 40.0).astype(np.float32)
    rowsum = q.astype(np.int32).sum(axis=1).astype(np.int32)
    acc_o = oracle.matmul_i32(q, Wt)
    gu_o = oracle.rescale(acc_o, beta, scale)
    f_o = oracle.chain_relu2_gate(gu_o)
    dev = "cuda:0"
    acc = torch.empty((M, N), dtype=torch.int32, device=dev)
    xb = torch.empty((M, F), dtype=torch.bfloat16, device=dev)
    absmax = torch.zeros(M, dtype=torch.float32, device=dev)
    bl.bl_gemm_w158a8_fused(to_dev(oracle.pack(Wt, 1)), to_dev(np.array([beta], dtype=np.float32)), 1, to_dev(q),
                            to_dev(scale), to_dev(rowsum), N, bl.BL_EPI_RELU2_GATE, xb, absmax, acc=acc)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), acc_o)
    assert np.array_equal(xb.view(torch.int16).cpu().numpy().view(np.uint16), f_o)
    assert np.array_equal(absmax.cpu().numpy(), np.abs(synth.bf16_bits_to_f32(f_o)).max(axis=1))
    q2, s2, r2 = bl.bl_quant_from_absmax(xb, absmax)
    torch.cuda.synchronize()
    q_o, s_o, r_o = oracle.quant_act(f_o)
    assert np.array_equal(q2.cpu().numpy(), q_o) and np.array_equal(r2.cpu().numpy(), r_o)
    assert np.array_equal(s2.cpu().numpy().view(np.uint32), s_o.view(np.uint32))


@pytest.mark.timeout(3000)
@pytest.mark.skipif(__import__("os").environ.get("BL_SKIP_FULL_CONFIG4") == "1",
                    reason="8.5e12 oracle multiply-adds (80 s on the 16 host cores of a GPU box): skipped on request")
def test_config4_prefill_every_row_every_layer(bl, chain):
    """The complete comparison of the M=4096 prefill stack: every row, every BitLinear of all 30
    layers (quantised inputs, scales, int32 accumulators) and the residual stream after every
    layer.  Prints a line per layer so that a long run is seen to move (pytest -s)."""
    n_layers, Mp = synth.N_LAYERS, 4096
    x_pre = synth.bf16_bits_to_f32(synth.activations_bf16(0, Mp, 2560, layer=101))
    dev_pre, o_pre = to_dev(x_pre), x_pre
    Bp = chain.ChainBuffers(Mp, dev_pre.device)
    for l in range(n_layers):
        ow = _layer_weights(0, l)
        gw = _to_gpu_weights(bl, ow)
        wts = {k: (v[0], v[1]) for k, v in ow.items()}
        tr_p, rec_p = [], []
        o_pre = oracle.chain_layer(o_pre, wts, trace=tr_p)
        out = chain.layer_prefill(gw, 1, dev_pre, Bp, rec_p)
        Bp.x_next, dev_pre = dev_pre, out
        torch.cuda.synchronize()
        _compare_records([rec_p], [tr_p])
        assert_y_close(dev_pre.cpu().numpy(), o_pre)
        print("layer %d: all %d rows ok" % (l, Mp), flush=True)
        del gw, ow, wts, rec_p, tr_p
