"""Thin Python binding of libmnnq.so: argument marshalling only.

Every function has the name of the C-ABI entry point it calls (include/mnnq.h)
and takes torch tensors that already live on the GPU; torch supplies device
memory and the current stream, nothing else.  No step of the path runs in
Python or on the CPU: if the library is missing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import torch  # noqa: F401  (must be imported first: the library binds to the HIP runtime torch loaded)

GROUP = 64
MODE_W4_ZP_INT = 0      # integer zero point per (row, group)
MODE_W4_MIN_FLOAT = 1   # Eq. 1 as printed: fp32 group minimum per (row, group)
MODE_W8_MIN_FLOAT = 2   # int8 weights (codes 0..255), fp32 group minimum; K must be a multiple of 128
WITH_MATRIX_PLANE = 16  # flag for MODE_W4_ZP_INT: the packed buffer also holds the fp6 matrix-core plane
NATIVE_8BIT = 32        # flag for MODE_W8_MIN_FLOAT: the codes as bytes q8 - 128 instead of two 4-bit planes

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libmnnq.so")

EXPORTS = (
    "mnnq_status_string", "mnnq_last_hip_error", "mnnq_version", "mnnq_packed_size", "mnnq_workspace_size",
    "mnnq_pack_weights", "mnnq_unpack_weights", "mnnq_quant_act", "mnnq_linear_decode",
    "mnnq_linear_decode_fused",
    "mnnq_linear_prefill", "mnnq_linear_decode_f16", "mnnq_linear_prefill_f16", "mnnq_linear_acc_debug",
    "mnnq_pack_from_quantized",
    "mnnq_linear_decode_o16", "mnnq_linear_prefill_o16", "mnnq_linear_decode_f16_o16", "mnnq_linear_prefill_f16_o16",
    "mnnq_plan_debug", "mnnq_linear_prefill_fused", "mnnq_linear_decode_fused_o16", "mnnq_linear_prefill_fused_o16",
    "mnnq_linear_prefill_fused_static", "mnnq_static_scratch_bytes",
    "mnnq_linear_acc_debug_planes", "mnnq_debug_set",
    "mnnq_act_planes", "mnnq_linear_prefill_planes", "mnnq_act_planes_size",
)


class MnnqError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s failed: %s (status %d, hip error %d)" % (
            what, lib().mnnq_status_string(status).decode(), status, lib().mnnq_last_hip_error()))


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libmnnq.so is not built (%s); run `python -c 'import __graft_entry__ as g; g.build()'`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
        L.mnnq_status_string.restype = ctypes.c_char_p
        L.mnnq_status_string.argtypes = [i32]
        L.mnnq_last_hip_error.restype = i32
        L.mnnq_version.restype = i32
        L.mnnq_packed_size.restype = sz
        L.mnnq_packed_size.argtypes = [i64, i64, i32, i32]
        L.mnnq_workspace_size.restype = sz
        L.mnnq_workspace_size.argtypes = [i64, i64, i64, i32, i32]
        L.mnnq_pack_weights.argtypes = [vp, i64, i64, i32, i32, vp, sz, vp]
        L.mnnq_unpack_weights.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp]
        L.mnnq_quant_act.argtypes = [vp, i64, i64, i32, vp, vp, vp, vp]
        L.mnnq_linear_decode.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.mnnq_linear_decode_fused.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp, sz, vp]
        L.mnnq_linear_prefill.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.mnnq_linear_decode_f16.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp, sz, vp]
        L.mnnq_linear_prefill_f16.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.mnnq_linear_acc_debug.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, i32, vp]
        L.mnnq_pack_from_quantized.argtypes = [vp, vp, vp, i64, i64, i32, i32, vp, sz, vp]
        L.mnnq_linear_prefill_fused.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, sz, vp]
        L.mnnq_linear_decode_fused_o16.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp, sz, vp]
        L.mnnq_linear_prefill_fused_o16.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, sz, vp]
        L.mnnq_plan_debug.argtypes = [i32, i64, i64, i64, i32, i32, vp]
        L.mnnq_linear_decode_o16.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp, vp]
        L.mnnq_linear_prefill_o16.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp]
        L.mnnq_linear_decode_f16_o16.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp]
        L.mnnq_linear_prefill_f16_o16.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp]
        L.mnnq_linear_acc_debug_planes.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp, sz, vp]
        L.mnnq_debug_set.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
        L.mnnq_linear_prefill_fused_static.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp, vp]
        for name in EXPORTS[5:]:
            getattr(L, name).restype = i32
        L.mnnq_act_planes.argtypes = [vp, i64, i64, i32, vp, sz, vp]
        L.mnnq_linear_prefill_planes.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp]
        L.mnnq_act_planes_size.restype = sz
        L.mnnq_act_planes_size.argtypes = [i64, i64, i32]
        L.mnnq_static_scratch_bytes.restype = sz
        L.mnnq_static_scratch_bytes.argtypes = []
        _lib = L
    return _lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, what: str) -> None:
    if status != 0:
        raise MnnqError(status, what)


def _dev(t, dtype, what):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous %s tensor on the GPU" % (what, dtype))
    return t


def _need(t, n: int, what: str):
    """The C-ABI takes plain pointers and trusts the sizes it is told: a buffer smaller than the shape
    implies is an out-of-bounds access on the GPU.  Refuse it here, on the host."""
    if t is not None and t.numel() < n:
        raise ValueError("%s holds %d elements, the shape needs %d" % (what, t.numel(), n))
    return t


def _need_packed(packed, N: int, K: int, mode: int):
    size = mnnq_packed_size(N, K, GROUP, mode)
    if size == 0:
        raise ValueError("unsupported shape N=%d K=%d mode=%d" % (N, K, mode))
    return _need(packed, size, "packed")


def mnnq_packed_size(N: int, K: int, group: int = GROUP, mode: int = MODE_W4_ZP_INT) -> int:
    return int(lib().mnnq_packed_size(N, K, group, mode))


def mnnq_workspace_size(M: int, N: int, K: int, group: int = GROUP, mode: int = MODE_W4_ZP_INT) -> int:
    return int(lib().mnnq_workspace_size(M, N, K, group, mode))


def mnnq_pack_weights(W: torch.Tensor, out: torch.Tensor | None = None, mode: int = MODE_W4_ZP_INT) -> torch.Tensor:
    """W fp32 [N, K] on the GPU -> packed uint8 buffer."""
    _dev(W, torch.float32, "W")
    N, K = W.shape
    size = mnnq_packed_size(N, K, GROUP, mode)
    if size == 0:
        _check(lib().mnnq_pack_weights(_ptr(W), N, K, GROUP, mode, _ptr(W), 0, _stream()),
               "mnnq_pack_weights")
    if out is None:
        out = torch.empty(size, dtype=torch.uint8, device=W.device)
    _check(lib().mnnq_pack_weights(_ptr(W), N, K, GROUP, mode, _ptr(out), out.numel(), _stream()),
           "mnnq_pack_weights")
    return out


def mnnq_unpack_weights(packed: torch.Tensor, N: int, K: int, mode: int = MODE_W4_ZP_INT):
    """Canonical view: (q u8 [N,K], scale f32 [N,G], zero u8 [N,G]); in mode MODE_W4_MIN_FLOAT the
    third array holds the fp32 group minima."""
    _dev(packed, torch.uint8, "packed")
    _need_packed(packed, N, K, mode)
    G = K // GROUP
    q = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    s = torch.empty((N, G), dtype=torch.float32, device=packed.device)
    z = torch.empty((N, G), dtype=torch.uint8 if (mode & 15) == MODE_W4_ZP_INT else torch.float32,
                    device=packed.device)
    _check(lib().mnnq_unpack_weights(_ptr(packed), N, K, GROUP, mode, _ptr(q), _ptr(s), _ptr(z),
                                     _stream()), "mnnq_unpack_weights")
    return q, s, z


def mnnq_quant_act(x: torch.Tensor, want_xsum: bool = True, out=None):
    """x fp32 [M, K] -> (xq i8 [M,K], sx f32 [M], xsum i32 [M,G] or None)."""
    _dev(x, torch.float32, "x")
    M, K = x.shape
    if out is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
        sx = torch.empty((M,), dtype=torch.float32, device=x.device)
        xsum = torch.empty((M, max(K // GROUP, 1)), dtype=torch.int32, device=x.device) if want_xsum else None
    else:
        xq, sx, xsum = out
    _check(lib().mnnq_quant_act(_ptr(x), M, K, GROUP, _ptr(xq), _ptr(sx), _ptr(xsum), _stream()),
           "mnnq_quant_act")
    return xq, sx, xsum


def mnnq_linear_decode(packed, N: int, K: int, xq, sx, bias=None, out=None, mode: int = MODE_W4_ZP_INT):
    """One token: xq i8 [K] (or [1,K]), sx f32 [1] -> y f32 [N]."""
    _dev(packed, torch.uint8, "packed"); _dev(xq, torch.int8, "xq"); _dev(sx, torch.float32, "sx")
    _need_packed(packed, N, K, mode)
    if xq.numel() != K:
        raise ValueError("xq must hold K values")
    y = torch.empty((N,), dtype=torch.float32, device=packed.device) if out is None else out
    _need(y, N, "out"); _need(bias, N, "bias")
    _check(lib().mnnq_linear_decode(_ptr(packed), N, K, GROUP, mode, _ptr(xq), _ptr(sx), _ptr(bias),
                                    _ptr(y), None, 0, _stream()), "mnnq_linear_decode")
    return y


def mnnq_linear_decode_fused(packed, N: int, K: int, x, bias=None, out=None, workspace=None,
                             mode: int = MODE_W4_ZP_INT):
    """One token, activation quantizer fused in: x f32 [K] (or [1,K]) -> y f32 [N].
    workspace: optional uint8 tensor of mnnq_workspace_size(1, N, K) bytes."""
    _dev(packed, torch.uint8, "packed"); _dev(x, torch.float32, "x")
    _need_packed(packed, N, K, mode)
    if x.numel() != K:
        raise ValueError("x must hold K values")
    y = torch.empty((N,), dtype=torch.float32, device=packed.device) if out is None else out
    _need(y, N, "out"); _need(bias, N, "bias")
    if workspace is not None:
        _dev(workspace, torch.uint8, "workspace")
    _check(lib().mnnq_linear_decode_fused(_ptr(packed), N, K, GROUP, mode, _ptr(x), _ptr(bias),
                                          _ptr(y), _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                          _stream()), "mnnq_linear_decode_fused")
    return y


def mnnq_linear_prefill(packed, N: int, K: int, xq, sx, bias=None, out=None, mode: int = MODE_W4_ZP_INT,
                        workspace=None):
    """M tokens: xq i8 [M,K], sx f32 [M] -> y f32 [M,N].  workspace: optional uint8 tensor
    (mnnq_workspace_size bytes); with the matrix-core plane in `packed` it selects the fp6 GEMM."""
    _dev(packed, torch.uint8, "packed"); _dev(xq, torch.int8, "xq"); _dev(sx, torch.float32, "sx")
    _need_packed(packed, N, K, mode)
    M = xq.shape[0]
    if xq.shape[1] != K or sx.numel() != M:
        raise ValueError("xq must be [M,K] and sx [M]")
    if workspace is not None:
        _dev(workspace, torch.uint8, "workspace")
    y = torch.empty((M, N), dtype=torch.float32, device=packed.device) if out is None else out
    _need(y, M * N, "out"); _need(bias, N, "bias")
    _check(lib().mnnq_linear_prefill(_ptr(packed), M, N, K, GROUP, mode, _ptr(xq), _ptr(sx),
                                     _ptr(bias), _ptr(y), _ptr(workspace),
                                     0 if workspace is None else workspace.numel(), _stream()), "mnnq_linear_prefill")
    return y


def mnnq_linear_acc_debug_planes(packed, N: int, K: int, xq, mode: int, workspace=None):
    """int32 group accumulators [M,N,G] from the fp6 GEMM (mode must carry WITH_MATRIX_PLANE)."""
    _dev(packed, torch.uint8, "packed"); _dev(xq, torch.int8, "xq")
    _need_packed(packed, N, K, mode)
    M = xq.shape[0]
    if workspace is None:
        workspace = torch.empty(max(16, mnnq_workspace_size(M, N, K, GROUP, mode)), dtype=torch.uint8,
                                device=packed.device)
    acc = torch.empty((M, N, K // GROUP), dtype=torch.int32, device=packed.device)
    _check(lib().mnnq_linear_acc_debug_planes(_ptr(packed), M, N, K, GROUP, mode, _ptr(xq), _ptr(acc),
                                              _ptr(workspace), workspace.numel(), _stream()),
           "mnnq_linear_acc_debug_planes")
    return acc


def mnnq_act_planes(xq, out=None):
    """int8 codes [M,K] -> the activation operand of the fp6 GEMM (uint8 tensor)."""
    _dev(xq, torch.int8, "xq")
    M, K = xq.shape
    size = int(lib().mnnq_act_planes_size(M, K, GROUP))
    planes = torch.empty(size, dtype=torch.uint8, device=xq.device) if out is None else out
    _check(lib().mnnq_act_planes(_ptr(xq), M, K, GROUP, _ptr(planes), planes.numel(), _stream()), "mnnq_act_planes")
    return planes


def mnnq_linear_prefill_planes(packed, M: int, N: int, K: int, planes, sx, bias=None, out=None,
                               mode: int = MODE_W4_ZP_INT | WITH_MATRIX_PLANE):
    """y f32 [M,N] from activation planes (mnnq_act_planes), scales sx [M] and packed weights with the plane."""
    _dev(packed, torch.uint8, "packed"); _dev(planes, torch.uint8, "planes"); _dev(sx, torch.float32, "sx")
    _need_packed(packed, N, K, mode)
    _need(planes, int(lib().mnnq_act_planes_size(M, K, GROUP)), "planes"); _need(sx, M, "sx")
    y = torch.empty((M, N), dtype=torch.float32, device=packed.device) if out is None else out
    _need(y, M * N, "out"); _need(bias, N, "bias")
    _check(lib().mnnq_linear_prefill_planes(_ptr(packed), M, N, K, GROUP, mode, _ptr(planes), _ptr(sx), _ptr(bias),
                                            _ptr(y), _stream()), "mnnq_linear_prefill_planes")
    return y


def mnnq_debug_set(key: str, value) -> None:
    """Test / tuning override of a launch plan (see mnnq.h); value None clears it."""
    _check(lib().mnnq_debug_set(key.encode(), None if value is None else str(value).encode()), "mnnq_debug_set")


def mnnq_linear_decode_f16(packed, N: int, K: int, x16, bias=None, out=None, mode: int = MODE_W4_ZP_INT):
    """One token, fp16 activations (W4A16; W8A16 with MODE_W8_MIN_FLOAT): x16 fp16 [K] -> y f32 [N]."""
    _dev(packed, torch.uint8, "packed"); _dev(x16, torch.float16, "x16")
    _need_packed(packed, N, K, mode)
    if x16.numel() != K:
        raise ValueError("x16 must hold K values")
    y = torch.empty((N,), dtype=torch.float32, device=packed.device) if out is None else out
    _need(y, N, "out"); _need(bias, N, "bias")
    _check(lib().mnnq_linear_decode_f16(_ptr(packed), N, K, GROUP, mode, _ptr(x16), _ptr(bias),
                                        _ptr(y), None, 0, _stream()), "mnnq_linear_decode_f16")
    return y


def mnnq_linear_prefill_f16(packed, N: int, K: int, x16, bias=None, out=None, row_scale=None,
                            mode: int = MODE_W4_ZP_INT):
    """M tokens, fp16 activations (W4A16; W8A16 with MODE_W8_MIN_FLOAT): x16 fp16 [M,K] -> y f32 [M,N];
    row_scale f32 [M] optional."""
    _dev(packed, torch.uint8, "packed"); _dev(x16, torch.float16, "x16")
    _need_packed(packed, N, K, mode)
    M = x16.shape[0]
    if x16.shape[1] != K:
        raise ValueError("x16 must be [M,K]")
    y = torch.empty((M, N), dtype=torch.float32, device=packed.device) if out is None else out
    _need(y, M * N, "out"); _need(bias, N, "bias")
    _check(lib().mnnq_linear_prefill_f16(_ptr(packed), M, N, K, GROUP, mode, _ptr(x16), _ptr(row_scale),
                                         _ptr(bias), _ptr(y), None, 0, _stream()), "mnnq_linear_prefill_f16")
    return y


def mnnq_pack_from_quantized(q, scale, zero, out=None, mode: int = MODE_W4_ZP_INT):
    """q u8 [N,K], scale f32 [N,G], zero u8 [N,G] (fp32 group minima in mode MODE_W4_MIN_FLOAT) on the
    GPU -> packed uint8 buffer."""
    _dev(q, torch.uint8, "q"); _dev(scale, torch.float32, "scale")
    _dev(zero, torch.uint8 if (mode & 15) == MODE_W4_ZP_INT else torch.float32, "zero")
    N, K = q.shape
    if tuple(scale.shape) != (N, K // GROUP) or tuple(zero.shape) != (N, K // GROUP):
        raise ValueError("scale and zero must be [N, K/%d]" % GROUP)
    nbytes = mnnq_packed_size(N, K, GROUP, mode)
    if nbytes == 0:
        raise ValueError("unsupported shape N=%d K=%d" % (N, K))
    packed = torch.empty(nbytes, dtype=torch.uint8, device=q.device) if out is None else out
    _check(lib().mnnq_pack_from_quantized(_ptr(q), _ptr(scale), _ptr(zero), N, K, GROUP, mode,
                                          _ptr(packed), packed.numel(), _stream()), "mnnq_pack_from_quantized")
    return packed


def mnnq_linear_acc_debug(packed, N: int, K: int, xq, use_prefill_kernel: bool, mode: int = MODE_W4_ZP_INT):
    """Integer group accumulators I[m,n,g] (int32 [M,N,G]) from the decode or the prefill kernel."""
    _dev(packed, torch.uint8, "packed"); _dev(xq, torch.int8, "xq")
    _need_packed(packed, N, K, mode)
    xq2 = xq.reshape(-1, K)
    M = xq2.shape[0]
    # int8 weights are two 4-bit planes: 2 K / 64 sums per (m, n), high-nibble planes first
    Gp = (2 if mode == MODE_W8_MIN_FLOAT else 1) * (K // GROUP)
    acc = torch.empty((M, N, Gp), dtype=torch.int32, device=packed.device)
    _check(lib().mnnq_linear_acc_debug(_ptr(packed), M, N, K, GROUP, mode, _ptr(xq2), _ptr(acc),
                                       1 if use_prefill_kernel else 0, _stream()), "mnnq_linear_acc_debug")
    return acc


# ---- the same linear calls with IEEE binary16 output

def mnnq_linear_decode_o16(packed, N: int, K: int, xq, sx, bias=None, out=None, mode: int = MODE_W4_ZP_INT):
    """One token: xq i8 [K], sx f32 [1] -> y fp16 [N]."""
    _dev(packed, torch.uint8, "packed"); _dev(xq, torch.int8, "xq"); _dev(sx, torch.float32, "sx")
    _need_packed(packed, N, K, mode)
    if xq.numel() != K:
        raise ValueError("xq must hold K values")
    y = torch.empty((N,), dtype=torch.float16, device=packed.device) if out is None else out
    _need(y, N, "out"); _need(bias, N, "bias")
    _dev(y, torch.float16, "out")
    _check(lib().mnnq_linear_decode_o16(_ptr(packed), N, K, GROUP, mode, _ptr(xq), _ptr(sx), _ptr(bias),
                                        _ptr(y), _stream()), "mnnq_linear_decode_o16")
    return y


def mnnq_linear_prefill_o16(packed, N: int, K: int, xq, sx, bias=None, out=None, mode: int = MODE_W4_ZP_INT):
    """M tokens: xq i8 [M,K], sx f32 [M] -> y fp16 [M,N]."""
    _dev(packed, torch.uint8, "packed"); _dev(xq, torch.int8, "xq"); _dev(sx, torch.float32, "sx")
    _need_packed(packed, N, K, mode)
    M = xq.shape[0]
    if xq.shape[1] != K or sx.numel() != M:
        raise ValueError("xq must be [M,K] and sx [M]")
    y = torch.empty((M, N), dtype=torch.float16, device=packed.device) if out is None else out
    _need(y, M * N, "out"); _need(bias, N, "bias")
    _dev(y, torch.float16, "out")
    _check(lib().mnnq_linear_prefill_o16(_ptr(packed), M, N, K, GROUP, mode, _ptr(xq), _ptr(sx),
                                         _ptr(bias), _ptr(y), _stream()), "mnnq_linear_prefill_o16")
    return y


def mnnq_linear_decode_f16_o16(packed, N: int, K: int, x16, bias=None, out=None, mode: int = MODE_W4_ZP_INT):
    """One token, fp16 activations: x16 fp16 [K] -> y fp16 [N]."""
    _dev(packed, torch.uint8, "packed"); _dev(x16, torch.float16, "x16")
    _need_packed(packed, N, K, mode)
    if x16.numel() != K:
        raise ValueError("x16 must hold K values")
    y = torch.empty((N,), dtype=torch.float16, device=packed.device) if out is None else out
    _need(y, N, "out"); _need(bias, N, "bias")
    _dev(y, torch.float16, "out")
    _check(lib().mnnq_linear_decode_f16_o16(_ptr(packed), N, K, GROUP, mode, _ptr(x16), _ptr(bias),
                                            _ptr(y), _stream()), "mnnq_linear_decode_f16_o16")
    return y


def mnnq_linear_prefill_f16_o16(packed, N: int, K: int, x16, bias=None, out=None, row_scale=None,
                                mode: int = MODE_W4_ZP_INT):
    """M tokens, fp16 activations: x16 fp16 [M,K] -> y fp16 [M,N]; row_scale f32 [M] optional."""
    _dev(packed, torch.uint8, "packed"); _dev(x16, torch.float16, "x16")
    _need_packed(packed, N, K, mode)
    M = x16.shape[0]
    if x16.shape[1] != K:
        raise ValueError("x16 must be [M,K]")
    y = torch.empty((M, N), dtype=torch.float16, device=packed.device) if out is None else out
    _need(y, M * N, "out"); _need(bias, N, "bias")
    _dev(y, torch.float16, "out")
    _check(lib().mnnq_linear_prefill_f16_o16(_ptr(packed), M, N, K, GROUP, mode, _ptr(x16), _ptr(row_scale),
                                             _ptr(bias), _ptr(y), _stream()), "mnnq_linear_prefill_f16_o16")
    return y


def mnnq_linear_prefill_fused(packed, N: int, K: int, x, bias=None, out=None, workspace=None,
                              mode: int = MODE_W4_ZP_INT):
    """M tokens, activation quantizer inside the call: x f32 [M,K] -> y f32 [M,N].
    workspace: uint8 tensor of at least mnnq_workspace_size(M, N, K) bytes (required by the library;
    this wrapper brings one along when none is given)."""
    _dev(packed, torch.uint8, "packed"); _dev(x, torch.float32, "x")
    _need_packed(packed, N, K, mode)
    M = x.shape[0]
    if x.shape[1] != K:
        raise ValueError("x must be [M,K]")
    if workspace is None:
        workspace = torch.empty(max(16, mnnq_workspace_size(M, N, K, GROUP, mode)), dtype=torch.uint8,
                                device=packed.device)
    _dev(workspace, torch.uint8, "workspace")
    y = torch.empty((M, N), dtype=torch.float32, device=packed.device) if out is None else out
    _need(y, M * N, "out"); _need(bias, N, "bias")
    _check(lib().mnnq_linear_prefill_fused(_ptr(packed), M, N, K, GROUP, mode, _ptr(x), _ptr(bias), _ptr(y),
                                           _ptr(workspace), workspace.numel(), _stream()),
           "mnnq_linear_prefill_fused")
    return y


def mnnq_linear_prefill_fused_static(packed, N: int, K: int, x, bias=None, out=None, mode: int = MODE_W4_ZP_INT):
    """mnnq_linear_prefill_fused through the library's own scratch array: x f32 [M,K] -> y f32 [M,N];
    `out` must be given by callers that may not allocate (this wrapper allocates it otherwise)."""
    _dev(packed, torch.uint8, "packed"); _dev(x, torch.float32, "x")
    _need_packed(packed, N, K, mode)
    M = x.shape[0]
    if x.shape[1] != K:
        raise ValueError("x must be [M,K]")
    y = torch.empty((M, N), dtype=torch.float32, device=packed.device) if out is None else out
    _need(y, M * N, "out"); _need(bias, N, "bias")
    _check(lib().mnnq_linear_prefill_fused_static(_ptr(packed), M, N, K, GROUP, mode, _ptr(x), _ptr(bias), _ptr(y),
                                                  _stream()), "mnnq_linear_prefill_fused_static")
    return y


def mnnq_static_scratch_bytes() -> int:
    return int(lib().mnnq_static_scratch_bytes())


def mnnq_linear_decode_fused_o16(packed, N: int, K: int, x, bias=None, out=None, workspace=None,
                                 mode: int = MODE_W4_ZP_INT):
    """One token, activation quantizer fused in: x f32 [K] -> y fp16 [N]."""
    _dev(packed, torch.uint8, "packed"); _dev(x, torch.float32, "x")
    _need_packed(packed, N, K, mode)
    if x.numel() != K:
        raise ValueError("x must hold K values")
    y = torch.empty((N,), dtype=torch.float16, device=packed.device) if out is None else out
    _need(y, N, "out"); _need(bias, N, "bias")
    _dev(y, torch.float16, "out")
    if workspace is not None:
        _dev(workspace, torch.uint8, "workspace")
    _check(lib().mnnq_linear_decode_fused_o16(_ptr(packed), N, K, GROUP, mode, _ptr(x), _ptr(bias), _ptr(y),
                                              _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                              _stream()), "mnnq_linear_decode_fused_o16")
    return y


def mnnq_linear_prefill_fused_o16(packed, N: int, K: int, x, bias=None, out=None, workspace=None,
                                  mode: int = MODE_W4_ZP_INT):
    """M tokens, activation quantizer inside the call: x f32 [M,K] -> y fp16 [M,N]."""
    _dev(packed, torch.uint8, "packed"); _dev(x, torch.float32, "x")
    _need_packed(packed, N, K, mode)
    M = x.shape[0]
    if x.shape[1] != K:
        raise ValueError("x must be [M,K]")
    if workspace is None:
        workspace = torch.empty(max(16, mnnq_workspace_size(M, N, K, GROUP, mode)), dtype=torch.uint8,
                                device=packed.device)
    _dev(workspace, torch.uint8, "workspace")
    y = torch.empty((M, N), dtype=torch.float16, device=packed.device) if out is None else out
    _need(y, M * N, "out"); _need(bias, N, "bias")
    _dev(y, torch.float16, "out")
    _check(lib().mnnq_linear_prefill_fused_o16(_ptr(packed), M, N, K, GROUP, mode, _ptr(x), _ptr(bias), _ptr(y),
                                               _ptr(workspace), workspace.numel(), _stream()),
           "mnnq_linear_prefill_fused_o16")
    return y


def mnnq_plan_debug(what: int, M: int, N: int, K: int, mode: int = MODE_W4_ZP_INT):
    """Launch configuration a call would choose (host logic, no GPU needed): a list of 8 ints, see mnnq.h."""
    out = (ctypes.c_int32 * 8)()
    _check(lib().mnnq_plan_debug(what, M, N, K, GROUP, mode, ctypes.cast(out, ctypes.c_void_p)), "mnnq_plan_debug")
    return list(out)
