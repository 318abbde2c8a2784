"""CPU oracle of the BitLinear W1.58A8 layer: TEST INFRASTRUCTURE ONLY.

A ctypes front to bitlinear_oracle.cpp (numpy arrays in, numpy arrays out).
Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this package; the GPU library never does, and nothing here imports the GPU
library.  Definitions and citations live in the C++ source.
"""
import ctypes
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "bitlinear_oracle.cpp")
_LIB = os.path.join(_DIR, "libbl_oracle.so")

CXXFLAGS = ["-O3", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
            "-Wall", "-Wextra"]


def build(force=False):
    """Compile the oracle with g++ into libbl_oracle.so next to its source."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["g++"] + CXXFLAGS + ["-o", tmp, _SRC])
    os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, vp, ci, f32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        lib.orc_absmean_beta.argtypes = [vp, i64, i64, vp]
        lib.orc_absmean_beta.restype = f32
        lib.orc_ternarize.argtypes = [vp, i64, i64, f32, vp]
        lib.orc_ternarize.restype = None
        lib.orc_pack.argtypes = [vp, i64, i64, ci, vp]
        lib.orc_pack.restype = ci
        lib.orc_unpack.argtypes = [vp, i64, i64, ci, vp]
        lib.orc_unpack.restype = i64
        lib.orc_quant_act.argtypes = [vp, i64, i64, vp, vp, vp]
        lib.orc_quant_act.restype = None
        lib.orc_matmul_i32.argtypes = [vp, vp, i64, i64, i64, vp]
        lib.orc_matmul_i32.restype = None
        lib.orc_matmul_i32_sampled.argtypes = [vp, vp, i64, i64, vp, vp, i64, vp]
        lib.orc_matmul_i32_sampled.restype = None
        lib.orc_rescale.argtypes = [vp, f32, vp, i64, i64, vp]
        lib.orc_rescale.restype = None
        lib.orc_f32_to_bf16.argtypes = [vp, i64, vp]
        lib.orc_f32_to_bf16.restype = None
        lib.orc_chain_attn_stub.argtypes = [vp, i64, ci, ci, ci, vp]
        lib.orc_chain_attn_stub.restype = None
        lib.orc_chain_residual.argtypes = [vp, vp, i64, vp]
        lib.orc_chain_residual.restype = None
        lib.orc_chain_relu2_gate.argtypes = [vp, i64, i64, vp]
        lib.orc_chain_relu2_gate.restype = None
        lib.orc_rmsnorm_rows.argtypes = [vp, i64, i64, vp, f32, vp, vp]
        lib.orc_rmsnorm_rows.restype = None
        lib.orc_chain_attn_f32.argtypes = [vp, i64, ci, ci, ci, vp]
        lib.orc_chain_attn_f32.restype = None
        lib.orc_chain_relu2_gate_f32.argtypes = [vp, i64, i64, vp]
        lib.orc_chain_relu2_gate_f32.restype = None
        lib.orc_omp_threads.argtypes = []
        lib.orc_omp_threads.restype = ci
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def omp_threads():
    return int(_load().orc_omp_threads())


def absmean_beta(W, return_mean64=False):
    """beta = fp32(mean |W|)  (Section 2, weight quantisation)."""
    W = _c(W, np.float32)
    N, K = W.shape
    m = ctypes.c_double(0.0)
    beta = _load().orc_absmean_beta(_p(W), N, K, ctypes.byref(m))
    beta = np.float32(beta)
    return (beta, m.value) if return_mean64 else beta


def beta_guard_ok(mean64, rel=1e-11):
    """True if the fp64 mean is not within `rel` (relative) of the midpoint of
    two adjacent fp32 values, i.e. any fp64 summation order rounds to the same
    fp32 beta."""
    f = np.float32(mean64)
    for nb in (np.nextafter(f, np.float32(np.inf)), np.nextafter(f, np.float32(-np.inf))):
        mid = (float(f) + float(nb)) / 2.0
        if abs(mean64 - mid) <= rel * abs(mean64):
            return False
    return True


def ternarize(W, beta):
    """Wt = clip(round(W/(beta+1e-5)), -1, 1) as int8 [N][K]."""
    W = _c(W, np.float32)
    N, K = W.shape
    Wt = np.empty((N, K), dtype=np.int8)
    _load().orc_ternarize(_p(W), N, K, float(np.float32(beta)), _p(Wt))
    return Wt


def pack(Wt, layout=0):
    """2-bit packing of a ternary int8 [N][K] matrix (Section 5.1)."""
    Wt = _c(Wt, np.int8)
    N, K = Wt.shape
    assert (N * K) % 4 == 0 and K % 4 == 0
    out = np.empty(N * K // 4, dtype=np.uint8)
    rc = _load().orc_pack(_p(Wt), N, K, int(layout), _p(out))
    if rc == 1:
        raise ValueError("weights outside {-1,0,1}")
    if rc == 2:
        raise ValueError("unknown layout %r" % (layout,))
    return out


def padded_k(K):
    """Row length of the packed form and of the quantised activations: K rounded up to a multiple of 64."""
    return -(-int(K) // 64) * 64


def pack_padded(Wt, layout=0):
    """Packed form of any N x K ternary matrix: the library's format (its own, like layout 1) pads every
    row with weight 0 to padded_k(K) weights and the row count with all-zero rows to a multiple of 4,
    then packs as above (Section 5.1).  Equal to pack() when nothing needs padding."""
    Wt = _c(Wt, np.int8)
    N, K = Wt.shape
    P = np.zeros((-(-N // 4) * 4, padded_k(K)), dtype=np.int8)
    P[:N, :K] = Wt
    return pack(P, layout)


def pad_q(q):
    """Quantised activations in the library's [M][padded_k(K)] form: zeros behind column K."""
    q = _c(q, np.int8)
    M, K = q.shape
    P = np.zeros((M, padded_k(K)), dtype=np.int8)
    P[:, :K] = q
    return P


def padded_k5(K):
    """Row length of the five-weights-per-byte form: K rounded up to a multiple of 80."""
    return -(-int(K) // 80) * 80


def pack_trit5(Wt):
    """Five weights per byte (1.6 bits per weight, the density behind the memory figure of Table 1;
    the library's layout 2, its own format).  Rows padded with weight 0 to padded_k5(K) weights and
    the row count to a multiple of 4.  The 4-byte word g of a row covers k = 20g .. 20g+19 and its
    byte j holds the offset codes c_i = Wt[k] + 1 of k = 20g + 4i + j, i = 0..4, as
    b = ceil(v * 256 / 243), v = sum_i c_i * 3^(4-i)."""
    Wt = _c(Wt, np.int8)
    if Wt.min(initial=0) < -1 or Wt.max(initial=0) > 1:
        raise ValueError("weights outside {-1,0,1}")
    N, K = Wt.shape
    Np, Kq = -(-N // 4) * 4, padded_k5(K)
    codes = np.ones((Np, Kq), dtype=np.int64)
    codes[:N, :K] = Wt.astype(np.int64) + 1
    c = codes.reshape(Np, Kq // 20, 5, 4)               # [row][word g][digit i][byte j]
    v = np.zeros((Np, Kq // 20, 4), dtype=np.int64)
    for i in range(5):
        v += c[:, :, i, :] * 3 ** (4 - i)
    b = (v * 256 + 242) // 243                          # ceil(v * 256 / 243)
    return b.astype(np.uint8).reshape(-1)


def unpack_trit5(packed, N, K):
    """Inverse of pack_trit5 by the decoding rule the format is built for: the leading digit of a byte
    is (3*b) >> 8, the low byte of 3*b carries the remaining digits.  Returns (Wt, number of bytes that
    are not the code of their own digits)."""
    Np, Kq = -(-N // 4) * 4, padded_k5(K)
    b = _c(packed, np.uint8).astype(np.int64).reshape(Np, Kq // 20, 4)
    r = b.copy()
    codes = np.empty((Np, Kq // 20, 5, 4), dtype=np.int64)
    v = np.zeros_like(b)
    for i in range(5):
        t = r * 3
        codes[:, :, i, :] = t >> 8
        r = t & 255
        v = v * 3 + codes[:, :, i, :]
    bad = int(np.count_nonzero((v * 256 + 242) // 243 != b))
    Wt = (codes.reshape(Np, Kq) - 1).astype(np.int8)
    return np.ascontiguousarray(Wt[:N, :K]), bad


def pack_kmajor(Wt):
    """k-major form (the library's layout 3, its own format): the transposed matrix, one row per input
    feature k, each row padded with weight 0 to a multiple of 64 output features and packed along n
    like layout 0 (Section 5.1: four 2-bit codes per byte).  Lets a decode kernel leave out the rows
    of zero activations (Section 2: squared ReLU is chosen for the sparsity it gives)."""
    Wt = _c(Wt, np.int8)
    N, K = Wt.shape
    Nq = -(-N // 64) * 64
    T = np.zeros((K, Nq), dtype=np.int8)
    T[:, :N] = Wt.T
    return pack(T, 0)


def unpack_kmajor(packed, N, K):
    Nq = -(-N // 64) * 64
    T, bad = unpack(packed, K, Nq, 0)
    return np.ascontiguousarray(T[:, :N].T), bad


def unpack(packed, N, K, layout=0):
    """Inverse of pack; returns (Wt int8 [N][K], number of invalid codes)."""
    packed = _c(packed, np.uint8)
    assert packed.size == N * K // 4
    Wt = np.empty((N, K), dtype=np.int8)
    bad = _load().orc_unpack(_p(packed), N, K, int(layout), _p(Wt))
    if bad < 0:
        raise ValueError("unknown layout %r" % (layout,))
    return Wt, int(bad)


def quant_act(X_bf16_bits):
    """Per-token absmax int8 quantiser on bf16 bit patterns uint16 [M][K].
    Returns (q int8 [M][K], scale fp32 [M], rowsum int32 [M])."""
    X = _c(X_bf16_bits, np.uint16)
    M, K = X.shape
    q = np.empty((M, K), dtype=np.int8)
    scale = np.empty(M, dtype=np.float32)
    rowsum = np.empty(M, dtype=np.int32)
    _load().orc_quant_act(_p(X), M, K, _p(q), _p(scale), _p(rowsum))
    return q, scale, rowsum


def matmul_i32(q, Wt):
    """acc[m][n] = sum_k q[m][k]*Wt[n][k], int32 [M][N]."""
    q = _c(q, np.int8)
    Wt = _c(Wt, np.int8)
    M, K = q.shape
    N, K2 = Wt.shape
    assert K == K2
    acc = np.empty((M, N), dtype=np.int32)
    _load().orc_matmul_i32(_p(q), _p(Wt), M, N, K, _p(acc))
    return acc


def matmul_i32_sampled(q, Wt, ms, ns):
    """acc[ms[i]][ns[i]] for the given index lists."""
    q = _c(q, np.int8)
    Wt = _c(Wt, np.int8)
    N, K = Wt.shape
    ms = _c(ms, np.int64)
    ns = _c(ns, np.int64)
    out = np.empty(ms.size, dtype=np.int32)
    _load().orc_matmul_i32_sampled(_p(q), _p(Wt), N, K, _p(ms), _p(ns), ms.size, _p(out))
    return out


def rescale(acc, beta, scale):
    """y = float(acc) * (beta * scale[m]), fp32 [M][N]."""
    acc = _c(acc, np.int32)
    scale = _c(scale, np.float32)
    M, N = acc.shape
    y = np.empty((M, N), dtype=np.float32)
    _load().orc_rescale(_p(acc), float(np.float32(beta)), _p(scale), M, N, _p(y))
    return y


def bitlinear(X_bf16_bits, Wt, beta, unit_scale=False):
    """Whole layer on prepared ternary weights: quantise, multiply, rescale.
    Returns dict(q, scale, rowsum, acc, y).  unit_scale: rescale with 1/127
    instead of absmax/127 (the chain's norm stand-in)."""
    q, scale, rowsum = quant_act(X_bf16_bits)
    acc = matmul_i32(q, Wt)
    s = np.full_like(scale, np.float32(1.0) / np.float32(127.0)) if unit_scale else scale
    y = rescale(acc, beta, s)
    return dict(q=q, scale=scale, rowsum=rowsum, acc=acc, y=y, used_scale=s)


def f32_to_bf16(x):
    x = _c(x, np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    _load().orc_f32_to_bf16(_p(x), x.size, _p(out))
    return out


def chain_attn_stub(qkv, n_q=20, n_kv=5, hd=128):
    qkv = _c(qkv, np.float32)
    M = qkv.shape[0]
    assert qkv.shape[1] == (n_q + 2 * n_kv) * hd
    a = np.empty((M, n_q * hd), dtype=np.uint16)
    _load().orc_chain_attn_stub(_p(qkv), M, n_q, n_kv, hd, _p(a))
    return a


def chain_residual(x, y):
    x = _c(x, np.float32)
    y = _c(y, np.float32)
    assert x.shape == y.shape
    h = np.empty_like(x)
    _load().orc_chain_residual(_p(x), _p(y), x.size, _p(h))
    return h


def chain_relu2_gate(gu):
    gu = _c(gu, np.float32)
    M, F2 = gu.shape
    f = np.empty((M, F2 // 2), dtype=np.uint16)
    _load().orc_chain_relu2_gate(_p(gu), M, F2 // 2, _p(f))
    return f


def fp32_rounding_guard_ok(v64, rel=1e-11):
    """True if the fp64 value is not within `rel` (relative) of the midpoint of two adjacent
    fp32 values: every fp64 evaluation that differs from it by less narrows to the same fp32."""
    f = np.float32(v64)
    for nb in (np.nextafter(f, np.float32(np.inf)), np.nextafter(f, np.float32(-np.inf))):
        mid = (float(f) + float(nb)) / 2.0
        if abs(v64 - mid) <= rel * abs(v64):
            return False
    return True


def rmsnorm_rows(t, gain=None, eps=1e-5, return_r64=False, check_guard=True):
    """bf16 bits of the RMS-normalised rows of t (fp32 [M][K]); the sum of squares is the
    exact real sum to fp64 accuracy (compensated), see orc_rmsnorm_rows.  check_guard: raise
    if a row's factor 1/sqrt(ss/K+eps) lies so close to an fp32 rounding boundary that another
    fp64 summation order could narrow differently (then the test input must change)."""
    t = _c(t, np.float32)
    M, K = t.shape
    assert K % 16 == 0
    g = None if gain is None else _c(gain, np.float32)
    assert g is None or g.shape == (K,)
    out = np.empty((M, K), dtype=np.uint16)
    r64 = np.empty(M, dtype=np.float64)
    _load().orc_rmsnorm_rows(_p(t), M, K, None if g is None else _p(g), float(np.float32(eps)), _p(out), _p(r64))
    if check_guard:
        bad = [m for m in range(M) if not fp32_rounding_guard_ok(float(r64[m]))]
        if bad:
            raise ValueError("rmsnorm factor of rows %s too close to an fp32 rounding midpoint: "
                             "change the input seed" % bad[:8])
    return (out, r64) if return_r64 else out


def chain_attn_f32(qkv, n_q=20, n_kv=5, hd=128):
    qkv = _c(qkv, np.float32)
    M = qkv.shape[0]
    a = np.empty((M, n_q * hd), dtype=np.float32)
    _load().orc_chain_attn_f32(_p(qkv), M, n_q, n_kv, hd, _p(a))
    return a


def chain_relu2_gate_f32(gu):
    gu = _c(gu, np.float32)
    M, F2 = gu.shape
    f = np.empty((M, F2 // 2), dtype=np.float32)
    _load().orc_chain_relu2_gate_f32(_p(gu), M, F2 // 2, _p(f))
    return f


def chain_layer(x, weights, trace=None, gains=None, eps=1e-5):
    """One synthetic layer of the chain on fp32 residual x [M][H].
    weights: dict name -> (Wt int8 [N][K], beta) for qkv, o, gate_up, down.
    If trace is a list, the inputs/outputs of every BitLinear are appended.
    gains: None = the norm stand-in (every BitLinear rescales with 1/127); a dict
    name -> fp32 [K] (or None) = RMS normalisation in front of every quantiser and the
    true absmax/127 rescale."""
    if gains is not None:
        def bln(name, t):
            Wt, beta = weights[name]
            xb = rmsnorm_rows(t, gains.get(name), eps)
            r = bitlinear(xb, Wt, beta)
            if trace is not None:
                trace.append(dict(name=name, x_bf16=xb, **r))
            return r["y"]

        qkv = bln("qkv", x)
        o = bln("o", chain_attn_f32(qkv))
        h1 = chain_residual(x, o)
        gu = bln("gate_up", h1)
        dn = bln("down", chain_relu2_gate_f32(gu))
        return chain_residual(h1, dn)

    def bl(name, xb):
        Wt, beta = weights[name]
        r = bitlinear(xb, Wt, beta, unit_scale=True)
        if trace is not None:
            trace.append(dict(name=name, x_bf16=xb, **r))
        return r["y"]

    qkv = bl("qkv", f32_to_bf16(x))
    o = bl("o", chain_attn_stub(qkv))
    h1 = chain_residual(x, o)
    gu = bl("gate_up", f32_to_bf16(h1))
    dn = bl("down", chain_relu2_gate(gu))
    return chain_residual(h1, dn)
