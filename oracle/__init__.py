"""CPU oracle for the W4A8 / W4A16 quantized linear layer.

TEST INFRASTRUCTURE: only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package.  It shares no code
with the HIP library (``paper_2506_10443_amd``) and never imports it.

The arithmetic lives in ``mnnq_oracle.c`` (plain scalar C); this file only
compiles it with gcc and marshals numpy arrays through ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

GROUP = 64
_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mnnq_oracle.c")
# MNNQ_ORACLE_SANITIZE=1 (tests only): a second build with AddressSanitizer and UndefinedBehaviorSanitizer;
# the process must then have been started with libasan preloaded.
_SANITIZE = os.environ.get("MNNQ_ORACLE_SANITIZE") == "1"
_LIB = os.path.join(_HERE, "libmnnq_oracle_san.so" if _SANITIZE else "libmnnq_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math, no FMA contraction; OpenMP
    only spreads output rows over the host cores."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"]
        if _SANITIZE:
            cmd[1:2] = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                        "-fno-sanitize-recover=all"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            _lib = ctypes.CDLL(build())
            for name in ("orc_quant_weights", "orc_dequant", "orc_quant_act", "orc_linear_w4a8",
                         "orc_linear_w4a16", "orc_linear_w4a8_sampled", "orc_linear_w4a16_sampled",
                         "orc_quant_weights_minf", "orc_dequant_minf", "orc_linear_w4a8_minf",
                         "orc_linear_w4a8_minf_sampled", "orc_quant_weights8", "orc_linear_w8a8",
                         "orc_linear_w8a8_sampled", "orc_linear_a16_minf", "orc_linear_a16_minf_sampled"):
                getattr(_lib, name).restype = None
            _lib.orc_omp_enabled.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _i64(v):
    return ctypes.c_int64(int(v))


def set_threads(n: int) -> None:
    """Number of OpenMP threads the next calls use (timing only)."""
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(int(n))


def quant_weights(W):
    """O1.  W fp32 [N,K] -> (q u8 [N,K], s f32 [N,G], z u8 [N,G])."""
    W = _c(W, np.float32)
    N, K = W.shape
    assert K % GROUP == 0
    G = K // GROUP
    q = np.empty((N, K), np.uint8)
    s = np.empty((N, G), np.float32)
    z = np.empty((N, G), np.uint8)
    _load().orc_quant_weights(_p(W), _i64(N), _i64(K), _p(q), _p(s), _p(z))
    return q, s, z


def dequant(q, s, z):
    """O2.  fp32 [N,K] of (q - z) * s."""
    q = _c(q, np.uint8); s = _c(s, np.float32); z = _c(z, np.uint8)
    N, K = q.shape
    out = np.empty((N, K), np.float32)
    _load().orc_dequant(_p(q), _p(s), _p(z), _i64(N), _i64(K), _p(out))
    return out


def quant_act(x):
    """O3.  x fp32 [M,K] -> (xq i8 [M,K], sx f32 [M], xsum i32 [M,G])."""
    x = _c(x, np.float32)
    M, K = x.shape
    assert K % GROUP == 0
    xq = np.empty((M, K), np.int8)
    sx = np.empty((M,), np.float32)
    xsum = np.empty((M, K // GROUP), np.int32)
    _load().orc_quant_act(_p(x), _i64(M), _i64(K), _p(xq), _p(sx), _p(xsum))
    return xq, sx, xsum


def linear_w4a8(xq, sx, q, s, z, bias=None, want_acc=True):
    """O4.  Returns (I int32 [M,N,G] or None, y fp32 [M,N])."""
    xq = _c(xq, np.int8); sx = _c(sx, np.float32)
    q = _c(q, np.uint8); s = _c(s, np.float32); z = _c(z, np.uint8)
    if bias is not None:
        bias = _c(bias, np.float32)
    M, K = xq.shape
    N = q.shape[0]
    assert q.shape[1] == K and K % GROUP == 0
    G = K // GROUP
    acc = np.empty((M, N, G), np.int32) if want_acc else None
    y = np.empty((M, N), np.float32)
    _load().orc_linear_w4a8(_p(xq), _p(sx), _p(q), _p(s), _p(z), _p(bias),
                            _i64(M), _i64(N), _i64(K), _p(acc), _p(y))
    return acc, y


def linear_w4a16(x16, q, s, z, bias=None):
    """O5.  x16 is fp16 [M,K]; returns y fp32 [M,N]."""
    x16 = _c(x16, np.float16)
    q = _c(q, np.uint8); s = _c(s, np.float32); z = _c(z, np.uint8)
    if bias is not None:
        bias = _c(bias, np.float32)
    M, K = x16.shape
    N = q.shape[0]
    y = np.empty((M, N), np.float32)
    _load().orc_linear_w4a16(_p(x16.view(np.uint16)), _p(q), _p(s), _p(z), _p(bias),
                             _i64(M), _i64(N), _i64(K), _p(y))
    return y


def linear_w4a8_sampled(xq, sx, q, s, z, ms, ns, bias=None, want_acc=True):
    """O4 on the listed (m, n) pairs only: (I [count,G] or None, y [count])."""
    xq = _c(xq, np.int8); sx = _c(sx, np.float32)
    q = _c(q, np.uint8); s = _c(s, np.float32); z = _c(z, np.uint8)
    ms = _c(ms, np.int64); ns = _c(ns, np.int64)
    if bias is not None:
        bias = _c(bias, np.float32)
    M, K = xq.shape
    N = q.shape[0]
    G = K // GROUP
    cnt = ms.shape[0]
    acc = np.empty((cnt, G), np.int32) if want_acc else None
    y = np.empty((cnt,), np.float32)
    _load().orc_linear_w4a8_sampled(_p(xq), _p(sx), _p(q), _p(s), _p(z), _p(bias),
                                    _i64(M), _i64(N), _i64(K), _p(ms), _p(ns), _i64(cnt),
                                    _p(acc), _p(y))
    return acc, y


def linear_w4a16_sampled(x16, q, s, z, ms, ns, bias=None):
    """O5 on the listed (m, n) pairs only: y [count]."""
    x16 = _c(x16, np.float16)
    q = _c(q, np.uint8); s = _c(s, np.float32); z = _c(z, np.uint8)
    ms = _c(ms, np.int64); ns = _c(ns, np.int64)
    if bias is not None:
        bias = _c(bias, np.float32)
    M, K = x16.shape
    N = q.shape[0]
    cnt = ms.shape[0]
    y = np.empty((cnt,), np.float32)
    _load().orc_linear_w4a16_sampled(_p(x16.view(np.uint16)), _p(q), _p(s), _p(z), _p(bias),
                                     _i64(M), _i64(N), _i64(K), _p(ms), _p(ns), _i64(cnt), _p(y))
    return y


def omp_enabled() -> bool:
    return bool(_load().orc_omp_enabled())


# ---- Eq. 1 taken literally: the group minimum stays a float offset (O6..O8)

def quant_weights_minf(W):
    """O6.  W fp32 [N,K] -> (q u8 [N,K], step f32 [N,G], wmin f32 [N,G])."""
    W = _c(W, np.float32)
    N, K = W.shape
    assert K % GROUP == 0
    G = K // GROUP
    q = np.empty((N, K), np.uint8)
    s = np.empty((N, G), np.float32)
    mn = np.empty((N, G), np.float32)
    _load().orc_quant_weights_minf(_p(W), _i64(N), _i64(K), _p(q), _p(s), _p(mn))
    return q, s, mn


def dequant_minf(q, s, wmin):
    """O7.  fp32 [N,K] of q * step + wmin (binary64, rounded once)."""
    q = _c(q, np.uint8); s = _c(s, np.float32); wmin = _c(wmin, np.float32)
    N, K = q.shape
    out = np.empty((N, K), np.float32)
    _load().orc_dequant_minf(_p(q), _p(s), _p(wmin), _i64(N), _i64(K), _p(out))
    return out


def linear_w4a8_minf(xq, sx, q, s, wmin, bias=None, want_acc=True):
    """O8.  Returns (A int32 [M,N,G] or None, y fp32 [M,N])."""
    xq = _c(xq, np.int8); sx = _c(sx, np.float32)
    q = _c(q, np.uint8); s = _c(s, np.float32); wmin = _c(wmin, np.float32)
    if bias is not None:
        bias = _c(bias, np.float32)
    M, K = xq.shape
    N = q.shape[0]
    assert q.shape[1] == K and K % GROUP == 0
    G = K // GROUP
    acc = np.empty((M, N, G), np.int32) if want_acc else None
    y = np.empty((M, N), np.float32)
    _load().orc_linear_w4a8_minf(_p(xq), _p(sx), _p(q), _p(s), _p(wmin), _p(bias),
                                 _i64(M), _i64(N), _i64(K), _p(acc), _p(y))
    return acc, y


def linear_w4a8_minf_sampled(xq, sx, q, s, wmin, ms, ns, bias=None, want_acc=True):
    """O8 on the listed (m, n) pairs only: (A [count,G] or None, y [count])."""
    xq = _c(xq, np.int8); sx = _c(sx, np.float32)
    q = _c(q, np.uint8); s = _c(s, np.float32); wmin = _c(wmin, np.float32)
    ms = _c(ms, np.int64); ns = _c(ns, np.int64)
    if bias is not None:
        bias = _c(bias, np.float32)
    M, K = xq.shape
    N = q.shape[0]
    G = K // GROUP
    cnt = ms.shape[0]
    acc = np.empty((cnt, G), np.int32) if want_acc else None
    y = np.empty((cnt,), np.float32)
    _load().orc_linear_w4a8_minf_sampled(_p(xq), _p(sx), _p(q), _p(s), _p(wmin), _p(bias),
                                         _i64(M), _i64(N), _i64(K), _p(ms), _p(ns), _i64(cnt), _p(acc), _p(y))
    return acc, y


# ---- int8 weights, Eq. 1 with clip range 0..255 and a float group minimum (O9, O10)

def quant_weights8(W):
    """O9.  W fp32 [N,K] -> (q u8 [N,K] 0..255, step f32 [N,G], wmin f32 [N,G])."""
    W = _c(W, np.float32)
    N, K = W.shape
    assert K % GROUP == 0
    G = K // GROUP
    q = np.empty((N, K), np.uint8)
    s = np.empty((N, G), np.float32)
    mn = np.empty((N, G), np.float32)
    _load().orc_quant_weights8(_p(W), _i64(N), _i64(K), _p(q), _p(s), _p(mn))
    return q, s, mn


def linear_w8a8(xq, sx, q, s, wmin, bias=None, want_acc=True):
    """O10.  Returns (A int32 [M,N,G] or None, y fp32 [M,N]); q holds 8-bit codes."""
    xq = _c(xq, np.int8); sx = _c(sx, np.float32)
    q = _c(q, np.uint8); s = _c(s, np.float32); wmin = _c(wmin, np.float32)
    if bias is not None:
        bias = _c(bias, np.float32)
    M, K = xq.shape
    N = q.shape[0]
    assert q.shape[1] == K and K % GROUP == 0
    G = K // GROUP
    acc = np.empty((M, N, G), np.int32) if want_acc else None
    y = np.empty((M, N), np.float32)
    _load().orc_linear_w8a8(_p(xq), _p(sx), _p(q), _p(s), _p(wmin), _p(bias),
                            _i64(M), _i64(N), _i64(K), _p(acc), _p(y))
    return acc, y


def linear_w8a8_sampled(xq, sx, q, s, wmin, ms, ns, bias=None, want_acc=True):
    """O10 on the listed (m, n) pairs only."""
    xq = _c(xq, np.int8); sx = _c(sx, np.float32)
    q = _c(q, np.uint8); s = _c(s, np.float32); wmin = _c(wmin, np.float32)
    ms = _c(ms, np.int64); ns = _c(ns, np.int64)
    if bias is not None:
        bias = _c(bias, np.float32)
    M, K = xq.shape
    N = q.shape[0]
    G = K // GROUP
    cnt = ms.shape[0]
    acc = np.empty((cnt, G), np.int32) if want_acc else None
    y = np.empty((cnt,), np.float32)
    _load().orc_linear_w8a8_sampled(_p(xq), _p(sx), _p(q), _p(s), _p(wmin), _p(bias),
                                    _i64(M), _i64(N), _i64(K), _p(ms), _p(ns), _i64(cnt), _p(acc), _p(y))
    return acc, y


# ---- fp16 activations on float-minimum weights, 4- or 8-bit codes (O11)

def linear_a16_minf(x16, q, s, wmin, bias=None):
    """O11.  x16 fp16 [M,K]; q codes (0..15 or 0..255); returns y fp32 [M,N]."""
    x16 = _c(x16, np.float16)
    q = _c(q, np.uint8); s = _c(s, np.float32); wmin = _c(wmin, np.float32)
    if bias is not None:
        bias = _c(bias, np.float32)
    M, K = x16.shape
    N = q.shape[0]
    assert q.shape[1] == K and K % GROUP == 0
    y = np.empty((M, N), np.float32)
    _load().orc_linear_a16_minf(_p(x16.view(np.uint16)), _p(q), _p(s), _p(wmin), _p(bias),
                                _i64(M), _i64(N), _i64(K), _p(y))
    return y


def linear_a16_minf_sampled(x16, q, s, wmin, ms, ns, bias=None):
    """O11 on the listed (m, n) pairs only: y [count]."""
    x16 = _c(x16, np.float16)
    q = _c(q, np.uint8); s = _c(s, np.float32); wmin = _c(wmin, np.float32)
    ms = _c(ms, np.int64); ns = _c(ns, np.int64)
    if bias is not None:
        bias = _c(bias, np.float32)
    M, K = x16.shape
    N = q.shape[0]
    cnt = ms.shape[0]
    y = np.empty((cnt,), np.float32)
    _load().orc_linear_a16_minf_sampled(_p(x16.view(np.uint16)), _p(q), _p(s), _p(wmin), _p(bias),
                                        _i64(M), _i64(N), _i64(K), _p(ms), _p(ns), _i64(cnt), _p(y))
    return y
