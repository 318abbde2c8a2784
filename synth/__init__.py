"""Seeded synthetic inputs (latent weights, bf16 activations) shared by the
oracle's tests and the GPU path's tests.  Holds none of the method's
arithmetic: it only draws numbers (see gen.c for the generator).

Recipe (the benchmark configurations of this repository):
  * latent weights  fp32  N(0, 0.02^2), one stream per (layer, matrix id);
  * activations     bf16  N(0,1) with round(0.01*K) fixed outlier channels
    multiplied by 20; the down-projection input is relu(.)^2 of that.
"""
import ctypes
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "gen.c")
_LIB = os.path.join(_DIR, "libbl_synth.so")

MATRIX_IDS = {"qkv": 0, "o": 1, "gate_up": 2, "down": 3}
# (N, K) of the four BitLinear matrices of one 2B-style layer.
LAYER_SHAPES = {"qkv": (3840, 2560), "o": (2560, 2560), "gate_up": (13824, 2560), "down": (2560, 6912)}
N_LAYERS = 30


def build(force=False):
    """Compile gen.c with gcc (OpenMP) into libbl_synth.so next to it."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u64, i64, vp = ctypes.c_uint64, ctypes.c_int64, ctypes.c_void_p
        lib.synth_normal_f32.argtypes = [u64, u64, i64, i64, ctypes.c_double, vp]
        lib.synth_outlier_channels.argtypes = [u64, u64, i64, i64, vp]
        lib.synth_activations_bf16.argtypes = [u64, u64, i64, i64, i64, vp, i64, ctypes.c_float, ctypes.c_int, vp]
        lib.synth_uniform_i8.argtypes = [u64, u64, i64, ctypes.c_int, ctypes.c_int, vp]
        for f in (lib.synth_normal_f32, lib.synth_outlier_channels, lib.synth_activations_bf16, lib.synth_uniform_i8):
            f.restype = None
        _lib = lib
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def weight_stream_id(layer, matrix):
    mid = MATRIX_IDS[matrix] if isinstance(matrix, str) else int(matrix)
    return (1 << 40) | (int(layer) << 8) | mid


def act_stream_id(layer, matrix):
    mid = MATRIX_IDS[matrix] if isinstance(matrix, str) else int(matrix)
    return (2 << 40) | (int(layer) << 8) | mid


def latent_weights(seed, N, K, layer=0, matrix=0, sigma=0.02):
    """fp32 [N][K] ~ N(0, sigma^2)."""
    out = np.empty((N, K), dtype=np.float32)
    _load().synth_normal_f32(seed, weight_stream_id(layer, matrix), 0, N * K, float(sigma), _ptr(out))
    return out


def outlier_channels(seed, K, frac=0.01, layer=0, matrix=0):
    n_out = int(round(frac * K))
    out = np.empty(max(n_out, 1), dtype=np.int32)
    _load().synth_outlier_channels(seed, act_stream_id(layer, matrix), K, n_out, _ptr(out))
    return out[:n_out].copy()


def activations_bf16(seed, M, K, layer=0, matrix=0, relu2=False, outlier_frac=0.01, outlier_mul=20.0, row0=0):
    """bf16 bit patterns, uint16 [M][K]."""
    ch = outlier_channels(seed, K, outlier_frac, layer, matrix)
    out = np.empty((M, K), dtype=np.uint16)
    chp = np.ascontiguousarray(ch) if ch.size else np.zeros(1, dtype=np.int32)
    _load().synth_activations_bf16(seed, act_stream_id(layer, matrix), row0, M, K, _ptr(chp), ch.size,
                                   float(outlier_mul), int(bool(relu2)), _ptr(out))
    return out


def uniform_i8(seed, shape, lo=-127, hi=127, stream=0):
    out = np.empty(shape, dtype=np.int8)
    _load().synth_uniform_i8(seed, (3 << 40) | int(stream), out.size, int(lo), int(hi), _ptr(out))
    return out


def bf16_bits_to_f32(u16):
    """Exact widening of bf16 bit patterns to fp32 (a format conversion)."""
    return (np.asarray(u16, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
