"""ctypes loader for the PEQA CPU oracle -- TEST INFRASTRUCTURE ONLY.

The oracle (peqa_oracle.c) is the plain fp64 statement of the PEQA quantized
linear layer (arXiv 2305.14152, Eq. 1 and Eq. 2) that the GPU library is
checked against.  Only tests, the smoke check and the benchmark's cpu_baseline
leg may import this module; the product package never does.

This file only marshals numpy arrays into the C functions; it holds no
arithmetic of the method.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "peqa_oracle.c")
_LIB = os.path.join(_HERE, "libpeqa_oracle.so")

_lib = None


def build(force=True):
    """Compile the oracle with gcc.  fp contraction is off and there is no
    fast-math, because the quantizer's fp32 arithmetic is part of its definition."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
    subprocess.check_call(cmd)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        L = ctypes.CDLL(_LIB)
        L.oracle_packed_words.restype = ctypes.c_size_t
        L.oracle_packed_words.argtypes = [ctypes.c_int] * 3
        L.oracle_max_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(rc, what):
    if rc != 0:
        raise ValueError("oracle %s failed with code %d" % (what, rc))


def max_threads():
    return int(lib().oracle_max_threads())


def num_groups(K, group):
    return K // group if group else 1


def quantize(W0, bits, group=0):
    """Eq. 1 min-max RTN in fp32.  Returns (codes u8 [N,K], s0 f32 [N,G], z0 u8 [N,G])."""
    W0 = np.ascontiguousarray(W0, dtype=np.float32)
    N, K = W0.shape
    G = num_groups(K, group)
    codes = np.empty((N, K), np.uint8)
    s0 = np.empty((N, G), np.float32)
    z0 = np.empty((N, G), np.uint8)
    _chk(lib().oracle_quantize(_p(W0), N, K, bits, group, _p(codes), _p(s0), _p(z0)), "quantize")
    return codes, s0, z0


def quantize_search(W0, bits, group=0, n_ratios=20, min_ratio=0.5):
    """Error-minimising initialisation over a grid of clipped ranges.  Returns (codes, s0, z0, choice)."""
    W0 = np.ascontiguousarray(W0, dtype=np.float32)
    N, K = W0.shape
    G = num_groups(K, group)
    codes = np.empty((N, K), np.uint8)
    s0 = np.empty((N, G), np.float32)
    z0 = np.empty((N, G), np.uint8)
    choice = np.empty((N, G), np.int32)
    f = lib().oracle_quantize_search
    f.argtypes = [ctypes.c_void_p] + [ctypes.c_int] * 5 + [ctypes.c_float] + [ctypes.c_void_p] * 4
    _chk(f(_p(W0), N, K, bits, group, int(n_ratios), float(min_ratio), _p(codes), _p(s0), _p(z0), _p(choice)),
         "quantize_search")
    return codes, s0, z0, choice


def quantize_f64(W0, bits, group=0):
    """fp64 shadow of the quantizer.  Returns (codes, s0 f64, z0, dist-to-tie f64)."""
    W0 = np.ascontiguousarray(W0, dtype=np.float32)
    N, K = W0.shape
    G = num_groups(K, group)
    codes = np.empty((N, K), np.uint8)
    s0 = np.empty((N, G), np.float64)
    z0 = np.empty((N, G), np.uint8)
    frac = np.empty((N, K), np.float64)
    _chk(lib().oracle_quantize_f64(_p(W0), N, K, bits, group, _p(codes), _p(s0), _p(z0), _p(frac)),
         "quantize_f64")
    return codes, s0, z0, frac


def packed_words(N, K, bits):
    return int(lib().oracle_packed_words(N, K, bits))


def bit_location(K, bits, i, k, t):
    w = ctypes.c_size_t()
    b = ctypes.c_int()
    _chk(lib().oracle_bit_location(K, bits, i, k, t, ctypes.byref(w), ctypes.byref(b)), "bit_location")
    return int(w.value), int(b.value)


def pack(codes, bits):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    words = np.empty(packed_words(N, K, bits), np.uint32)
    _chk(lib().oracle_pack(_p(codes), N, K, bits, _p(words)), "pack")
    return words


def unpack(words, N, K, bits):
    words = np.ascontiguousarray(words, dtype=np.uint32)
    assert words.size == packed_words(N, K, bits)
    codes = np.empty((N, K), np.uint8)
    _chk(lib().oracle_unpack(_p(words), N, K, bits, _p(codes)), "unpack")
    return codes


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def dequant(codes, s0, ds, z0, group=0):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    s0, ds = _f32(s0), _f32(ds)
    z0 = np.ascontiguousarray(z0, dtype=np.uint8)
    What = np.empty((N, K), np.float64)
    _chk(lib().oracle_dequant(_p(codes), _p(s0), _p(ds), _p(z0), N, K, group, _p(What)), "dequant")
    return What


def fwd(codes, s0, ds, z0, X_bf16, group=0):
    """Y = X What^T in fp64.  X_bf16: uint16 bit patterns [T,K]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    X = np.ascontiguousarray(X_bf16, dtype=np.uint16)
    T = X.shape[0]
    assert X.shape == (T, K)
    s0, ds = _f32(s0), _f32(ds)
    z0 = np.ascontiguousarray(z0, dtype=np.uint8)
    Y = np.empty((T, N), np.float64)
    _chk(lib().oracle_fwd(_p(codes), _p(s0), _p(ds), _p(z0), _p(X), T, N, K, group, _p(Y)), "fwd")
    return Y


def bwd(codes, s0, ds, z0, X_bf16, dY_bf16, group=0, want_dX=True, want_P=True, want_W=False):
    """Returns (dX f64 [T,K] | None, dds via P route | None, dds via dWhat route | None)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    X = np.ascontiguousarray(X_bf16, dtype=np.uint16)
    dY = np.ascontiguousarray(dY_bf16, dtype=np.uint16)
    T = X.shape[0]
    assert X.shape == (T, K) and dY.shape == (T, N)
    G = num_groups(K, group)
    s0, ds = _f32(s0), _f32(ds)
    z0 = np.ascontiguousarray(z0, dtype=np.uint8)
    dX = np.empty((T, K), np.float64) if want_dX else None
    gP = np.empty((N, G), np.float64) if want_P else None
    gW = np.empty((N, G), np.float64) if want_W else None
    _chk(lib().oracle_bwd(_p(codes), _p(s0), _p(ds), _p(z0), _p(X), _p(dY), T, N, K, group,
                          _p(dX), _p(gP), _p(gW)), "bwd")
    return dX, gP, gW


def fwd_z(codes, s0, ds, z0, dz, X_bf16, group=0):
    """Forward with trainable zero-points z = z0 + dz (Appendix K), fp64."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    X = np.ascontiguousarray(X_bf16, dtype=np.uint16)
    T = X.shape[0]
    assert X.shape == (T, K)
    s0, ds, dz = _f32(s0), _f32(ds), _f32(dz)
    z0 = np.ascontiguousarray(z0, dtype=np.uint8)
    Y = np.empty((T, N), np.float64)
    _chk(lib().oracle_fwd_z(_p(codes), _p(s0), _p(ds), _p(z0), _p(dz), _p(X), T, N, K, group, _p(Y)), "fwd_z")
    return Y


def bwd_z(codes, s0, ds, z0, dz, X_bf16, dY_bf16, group=0, want_dX=True):
    """Returns (dX | None, dds, ddz) for zero-points z = z0 + dz (Appendix K), fp64."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    X = np.ascontiguousarray(X_bf16, dtype=np.uint16)
    dY = np.ascontiguousarray(dY_bf16, dtype=np.uint16)
    T = X.shape[0]
    assert X.shape == (T, K) and dY.shape == (T, N)
    G = num_groups(K, group)
    s0, ds, dz = _f32(s0), _f32(ds), _f32(dz)
    z0 = np.ascontiguousarray(z0, dtype=np.uint8)
    dX = np.empty((T, K), np.float64) if want_dX else None
    gs = np.empty((N, G), np.float64)
    gz = np.empty((N, G), np.float64)
    _chk(lib().oracle_bwd_z(_p(codes), _p(s0), _p(ds), _p(z0), _p(dz), _p(X), _p(dY), T, N, K, group,
                            _p(dX), _p(gs), _p(gz)), "bwd_z")
    return dX, gs, gz


def adamw(ds, g, m, v, s0, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, step=1):
    """One AdamW step in fp64; returns new (ds, m, v) without touching the inputs."""
    ds = np.array(ds, dtype=np.float64).ravel().copy()
    m = np.array(m, dtype=np.float64).ravel().copy()
    v = np.array(v, dtype=np.float64).ravel().copy()
    g = np.ascontiguousarray(np.asarray(g, dtype=np.float64).ravel())
    s0 = np.ascontiguousarray(np.asarray(s0, dtype=np.float64).ravel())
    f = lib().oracle_adamw
    f.argtypes = [ctypes.c_size_t] + [ctypes.c_void_p] * 5 + [ctypes.c_double] * 5 + [ctypes.c_int]
    _chk(f(ds.size, _p(ds), _p(g), _p(m), _p(v), _p(s0), lr, beta1, beta2, eps, weight_decay, step),
         "adamw")
    return ds, m, v
