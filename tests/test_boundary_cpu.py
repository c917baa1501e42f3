"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol include/mnnq.h declares, and rejects bad arguments before touching
HIP.  No compute call is made here."""
import ctypes
import os
import re

import pytest

from paper_2506_10443_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # non-NULL, 16-byte aligned; never dereferenced because validation fails first
ODD = 0x10004   # 4-byte aligned only


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.lib()


def _declared():
    text = open(os.path.join(ROOT, "include", "mnnq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mnnq_[a-z0-9_]+)\s*\(", text)))


def test_exports_match_header(L):
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_packed_size(L):
    # K multiple of 128: exactly codes + fp32 scale + one-byte zero
    for N, K in [(8960, 1536), (3584, 18944), (152064, 3584), (16, 128)]:
        assert binding.mnnq_packed_size(N, K) == N * K // 2 + 5 * N * (K // 64)
    # odd number of groups: one padding group per row
    assert binding.mnnq_packed_size(32, 192) == 32 * 256 // 2 + 5 * 32 * 4
    assert binding.mnnq_packed_size(32, 64) == 32 * 128 // 2 + 5 * 32 * 2
    # unsupported arguments
    assert binding.mnnq_packed_size(8, 128) == 0       # N not a multiple of 16
    assert binding.mnnq_packed_size(16, 100) == 0      # K not a multiple of 64
    assert binding.mnnq_packed_size(16, 128, 32) == 0  # group
    assert binding.mnnq_packed_size(16, 128, 64, 3) == 0  # mode
    # int8 weights: two nibble planes, each with fp32 step and minimum; K must be a multiple of 128
    assert binding.mnnq_packed_size(16, 128, 64, 2) == 16 * 128 + 16 * 16 * 2
    assert binding.mnnq_packed_size(16, 192, 64, 2) == 0
    # float-minimum form: fp32 minimum instead of a one-byte zero point per group
    assert binding.mnnq_packed_size(3584, 18944, 64, 1) == 3584 * 18944 // 2 + 8 * 3584 * (18944 // 64)
    assert binding.mnnq_packed_size(0, 128) == 0 and binding.mnnq_packed_size(16, -64) == 0
    assert binding.mnnq_workspace_size(1, 16, 128) == 128 + 16     # optional scratch of the fused decode call
    assert binding.mnnq_workspace_size(1, 16, 192) == 256 + 16
    assert binding.mnnq_workspace_size(4, 16, 128) == 4 * 128 + 16   # fused prefill call: codes [M,K] + scales [M]
    assert binding.mnnq_workspace_size(3, 16, 192) == 576 + 16
    assert binding.mnnq_workspace_size(1, 8, 128) == 0 and binding.mnnq_workspace_size(0, 16, 128) == 0


def test_status_strings(L):
    seen = set()
    for s in range(0, -7, -1):
        txt = L.mnnq_status_string(s).decode()
        assert txt and txt != "unknown status"
        seen.add(txt)
    assert len(seen) == 7
    assert L.mnnq_status_string(-99).decode() == "unknown status"
    assert L.mnnq_version() >= 100


def test_argument_validation_precedes_hip(L):
    i64 = ctypes.c_int64
    OK, NULL, SHAPE, UNSUP, SIZE, ALIGN = 0, -1, -2, -3, -4, -5
    pw = L.mnnq_pack_weights
    assert pw(None, 16, 128, 64, 0, FAKE, 10**9, None) == NULL
    assert pw(FAKE, 16, 128, 64, 0, None, 10**9, None) == NULL
    assert pw(FAKE, 0, 128, 64, 0, FAKE, 10**9, None) == SHAPE
    assert pw(FAKE, 16, 100, 64, 0, FAKE, 10**9, None) == SHAPE
    assert pw(FAKE, 16, 128, 32, 0, FAKE, 10**9, None) == UNSUP
    assert pw(FAKE, 16, 128, 64, 7, FAKE, 10**9, None) == UNSUP
    assert pw(FAKE, 16, 128, 64, 1, FAKE, binding.mnnq_packed_size(16, 128, 64, 1) - 1, None) == SIZE
    assert pw(FAKE, 24, 128, 64, 0, FAKE, 10**9, None) == UNSUP
    assert pw(ODD, 16, 128, 64, 0, FAKE, 10**9, None) == ALIGN
    assert pw(FAKE, 16, 128, 64, 0, FAKE, binding.mnnq_packed_size(16, 128) - 1, None) == SIZE

    qa = L.mnnq_quant_act
    assert qa(None, 1, 128, 64, FAKE, FAKE, None, None) == NULL
    assert qa(FAKE, 1, 128, 64, None, FAKE, None, None) == NULL
    assert qa(FAKE, 0, 128, 64, FAKE, FAKE, None, None) == SHAPE
    assert qa(FAKE, 1, 96, 64, FAKE, FAKE, None, None) == SHAPE
    assert qa(FAKE, 1, 128, 16, FAKE, FAKE, None, None) == UNSUP
    assert qa(ODD, 1, 128, 64, FAKE, FAKE, None, None) == ALIGN

    ld = L.mnnq_linear_decode
    assert ld(None, 16, 128, 64, 0, FAKE, FAKE, None, FAKE, None, 0, None) == NULL
    assert ld(FAKE, 16, 128, 64, 0, FAKE, None, None, FAKE, None, 0, None) == NULL
    assert ld(FAKE, 16, 128, 64, 0, FAKE, FAKE, None, None, None, 0, None) == NULL
    assert ld(FAKE, 16, 192 + 32, 64, 0, FAKE, FAKE, None, FAKE, None, 0, None) == SHAPE
    assert ld(FAKE, 20, 128, 64, 0, FAKE, FAKE, None, FAKE, None, 0, None) == UNSUP
    assert ld(FAKE, 16, 126976 + 64, 64, 0, FAKE, FAKE, None, FAKE, None, 0, None) == UNSUP  # row too long for LDS
    assert ld(FAKE, 16, 128, 64, 0, ODD, FAKE, None, FAKE, None, 0, None) == ALIGN
    assert ld(FAKE, 16, 128, 64, 0, FAKE, FAKE, ODD, FAKE, None, 0, None) == ALIGN

    lf = L.mnnq_linear_decode_fused
    assert lf(FAKE, 16, 128, 64, 0, None, None, FAKE, None, 0, None) == NULL
    assert lf(FAKE, 16, 128, 64, 0, ODD, None, FAKE, None, 0, None) == ALIGN
    assert lf(FAKE, 16, 100, 64, 0, FAKE, None, FAKE, None, 0, None) == SHAPE
    assert lf(FAKE, 16, 128, 64, 0, FAKE, None, FAKE, ODD, 1024, None) == ALIGN

    lp = L.mnnq_linear_prefill
    assert lp(FAKE, 0, 16, 128, 64, 0, FAKE, FAKE, None, FAKE, None, 0, None) == SHAPE
    assert lp(FAKE, 4, 16, 128, 64, 0, None, FAKE, None, FAKE, None, 0, None) == NULL
    assert lp(FAKE, 4, 16, 128, 64, 3, FAKE, FAKE, None, FAKE, None, 0, None) == UNSUP
    assert lp(FAKE, 4, 16, 192, 64, 2, FAKE, FAKE, None, FAKE, None, 0, None) == UNSUP   # int8 weights: K % 128
    assert lp(FAKE, 4, 16, 128, 64, 0, FAKE, FAKE, None, ODD, None, 0, None) == ALIGN

    assert L.mnnq_linear_decode_f16(FAKE, 16, 128, 64, 0, None, None, FAKE, None, 0, None) == NULL
    assert L.mnnq_linear_decode_f16(FAKE, 16, 100, 64, 0, FAKE, None, FAKE, None, 0, None) == SHAPE
    assert L.mnnq_linear_decode_f16(FAKE, 16, 128, 64, 3, FAKE, None, FAKE, None, 0, None) == UNSUP   # no such mode
    assert L.mnnq_linear_decode_f16(FAKE, 16, 192, 64, 2, FAKE, None, FAKE, None, 0, None) == UNSUP   # int8 weights: K % 128
    assert L.mnnq_linear_decode_f16(FAKE, 16, 79872 + 64, 64, 0, FAKE, None, FAKE, None, 0, None) == UNSUP  # row too long for LDS
    assert L.mnnq_linear_decode_f16(FAKE, 16, 71680 + 64, 64, 1, FAKE, None, FAKE, None, 0, None) == UNSUP  # same, float minimum
    assert L.mnnq_linear_decode_f16(FAKE, 16, 35840 + 128, 64, 2, FAKE, None, FAKE, None, 0, None) == UNSUP  # same, two planes
    assert L.mnnq_linear_prefill_f16(FAKE, 4, 16, 128, 64, 3, FAKE, None, None, FAKE, None, 0, None) == UNSUP
    assert L.mnnq_linear_prefill_f16(FAKE, 4, 16, 192, 64, 2, FAKE, None, None, FAKE, None, 0, None) == UNSUP
    assert L.mnnq_linear_prefill_f16(FAKE, 4, 16, 128, 64, 0, FAKE, None, None, None, None, 0, None) == NULL
    assert L.mnnq_linear_prefill_f16(FAKE, -1, 16, 128, 64, 0, FAKE, None, None, FAKE, None, 0, None) == SHAPE
    # the matrix-core plane: a flag of the integer zero point mode only
    PL = 16
    # chunk layout rounded up to 256 bytes, then 2 groups x 8 column tiles (padded) x (1536 B of codes + 32 scales)
    assert binding.mnnq_packed_size(64, 128, 64, 0) == 4736
    assert binding.mnnq_packed_size(64, 128, 64, PL) == 4864 + 2 * 8 * (1536 + 128)
    assert binding.mnnq_packed_size(64, 128, 64, PL | 1) == 0 and binding.mnnq_packed_size(64, 128, 64, 32) == 0
    assert L.mnnq_pack_weights(FAKE, 64, 128, 64, PL, FAKE, binding.mnnq_packed_size(64, 128, 64, 0), None) == SIZE
    assert L.mnnq_pack_weights(FAKE, 64, 128, 64, PL | 2, FAKE, 10**9, None) == UNSUP
    assert binding.mnnq_workspace_size(64, 64, 128, 64, PL) == 2 * 8 * 2 * 1536 + 64 * 128 + 256
    assert binding.mnnq_workspace_size(64, 64, 128, 64, 0) == 64 * 128 + 256
    assert binding.mnnq_workspace_size(32, 64, 128, 64, PL) == 32 * 128 + 128      # 32 tokens or fewer: the int8 kernels
    ap_, lp = L.mnnq_act_planes, L.mnnq_linear_prefill_planes
    assert L.mnnq_act_planes_size(64, 128, 64) == 2 * 8 * 2 * 1536 and L.mnnq_act_planes_size(64, 100, 64) == 0
    assert ap_(None, 64, 128, 64, FAKE, 10**9, None) == NULL and ap_(FAKE, 64, 100, 64, FAKE, 10**9, None) == SHAPE
    assert ap_(FAKE, 64, 128, 64, FAKE, 100, None) == SIZE and ap_(FAKE, 64, 128, 64, ODD, 10**9, None) == ALIGN
    assert lp(FAKE, 64, 64, 128, 64, PL, None, FAKE, None, FAKE, None) == NULL
    assert lp(FAKE, 64, 64, 128, 64, 0, FAKE, FAKE, None, FAKE, None) == UNSUP      # no plane in the buffer
    assert lp(FAKE, 16, 64, 128, 64, PL, FAKE, FAKE, None, FAKE, None) == UNSUP     # too few tokens for this kernel
    assert lp(FAKE, 64, 64, 128, 64, PL, FAKE, FAKE, None, ODD, None) == ALIGN
    ad = L.mnnq_linear_acc_debug_planes
    assert ad(FAKE, 64, 64, 128, 64, PL, FAKE, FAKE, None, 0, None) == NULL
    assert ad(FAKE, 64, 64, 128, 64, PL, FAKE, FAKE, FAKE, 100, None) == SIZE
    assert ad(FAKE, 64, 64, 128, 64, 0, FAKE, FAKE, FAKE, 10**9, None) == UNSUP
    assert L.mnnq_debug_set(b"MNNQ_PREFILL6_PLAN", b"2") == OK and L.mnnq_debug_set(b"MNNQ_PREFILL6_PLAN", None) == OK
    st = L.mnnq_linear_prefill_fused_static
    assert st(None, 4, 16, 128, 64, 0, FAKE, None, FAKE, None) == NULL
    assert st(FAKE, 4096, 16, 8192, 64, 0, FAKE, None, FAKE, None) == SIZE          # codes and scales beyond the array
    assert st(FAKE, 4, 16, 128, 64, 0, ODD, None, FAKE, None) == ALIGN
    assert L.mnnq_static_scratch_bytes() == 32 << 20
    pf = L.mnnq_linear_prefill_fused
    assert pf(FAKE, 4, 16, 128, 64, 0, FAKE, None, FAKE, None, 0, None) == NULL        # the workspace is required
    assert pf(FAKE, 4, 16, 128, 64, 0, FAKE, None, FAKE, FAKE, 100, None) == SIZE
    assert pf(FAKE, 4, 16, 128, 64, 0, FAKE, None, FAKE, ODD, 4096, None) == ALIGN
    assert pf(FAKE, 0, 16, 128, 64, 0, FAKE, None, FAKE, FAKE, 4096, None) == SHAPE
    assert pf(FAKE, 4, 16, 128, 64, 3, FAKE, None, FAKE, FAKE, 4096, None) == UNSUP
    # binary16 output: the same checks as the calls they mirror
    assert L.mnnq_linear_decode_o16(FAKE, 16, 128, 64, 0, FAKE, FAKE, None, None, None) == NULL
    assert L.mnnq_linear_decode_o16(FAKE, 16, 100, 64, 0, FAKE, FAKE, None, FAKE, None) == SHAPE
    assert L.mnnq_linear_prefill_o16(FAKE, 0, 16, 128, 64, 0, FAKE, FAKE, None, FAKE, None) == SHAPE
    assert L.mnnq_linear_prefill_o16(FAKE, 4, 16, 128, 64, 0, FAKE, FAKE, None, ODD, None) == ALIGN
    assert L.mnnq_linear_decode_f16_o16(FAKE, 16, 128, 64, 3, FAKE, None, FAKE, None) == UNSUP
    assert L.mnnq_linear_prefill_f16_o16(FAKE, 4, 16, 128, 64, 0, None, None, None, FAKE, None) == NULL
    assert L.mnnq_linear_decode_fused_o16(FAKE, 16, 128, 64, 0, FAKE, None, None, None, 0, None) == NULL
    assert L.mnnq_linear_decode_fused_o16(FAKE, 16, 128, 64, 0, FAKE, None, ODD, None, 0, None) == ALIGN
    assert L.mnnq_linear_prefill_fused_o16(FAKE, 4, 16, 128, 64, 0, FAKE, None, FAKE, None, 0, None) == NULL
    assert L.mnnq_linear_prefill_fused_o16(FAKE, 4, 16, 128, 64, 0, FAKE, None, FAKE, FAKE, 16, None) == SIZE
    assert L.mnnq_linear_acc_debug(FAKE, 1, 16, 128, 64, 0, FAKE, None, 0, None) == NULL
    assert L.mnnq_linear_acc_debug(FAKE, 70000, 16, 128, 64, 0, FAKE, FAKE, 0, None) == UNSUP
    pq = L.mnnq_pack_from_quantized
    assert pq(None, FAKE, FAKE, 16, 128, 64, 0, FAKE, 10**9, None) == NULL
    assert pq(FAKE, FAKE, None, 16, 128, 64, 0, FAKE, 10**9, None) == NULL
    assert pq(FAKE, FAKE, FAKE, 16, 96, 64, 0, FAKE, 10**9, None) == SHAPE
    assert pq(FAKE, FAKE, FAKE, 16, 128, 64, 3, FAKE, 10**9, None) == UNSUP
    assert pq(FAKE, FAKE, ODD + 2, 16, 128, 64, 1, FAKE, 10**9, None) == ALIGN   # fp32 minima
    assert pq(ODD, FAKE, FAKE, 16, 128, 64, 0, FAKE, 10**9, None) == ALIGN
    assert pq(FAKE, FAKE, FAKE, 16, 128, 64, 0, FAKE, binding.mnnq_packed_size(16, 128) - 1, None) == SIZE
    assert L.mnnq_unpack_weights(None, 16, 128, 64, 0, FAKE, FAKE, FAKE, None) == NULL
    assert L.mnnq_unpack_weights(FAKE, 16, 128, 64, 0, None, None, None, None) == OK  # nothing asked for
    # byte form of int8 weights: a flag of mode 2 only; the calls that read the plane form refuse it
    NB = 2 | 32
    assert binding.mnnq_packed_size(16, 128, 64, NB) == 16 * 128 + 8 * 16 * 2
    assert binding.mnnq_packed_size(152064, 3584, 64, NB) == 152064 * 3584 + 8 * 152064 * 56
    assert binding.mnnq_packed_size(16, 192, 64, NB) == 0                      # K a multiple of 128
    assert binding.mnnq_packed_size(16, 128, 64, 0 | 32) == 0 and binding.mnnq_packed_size(16, 128, 64, 1 | 32) == 0
    assert binding.mnnq_packed_size(16, 128, 64, NB | 16) == 0                 # the fp6 plane belongs to mode 0
    assert binding.mnnq_workspace_size(4, 16, 128, 64, NB) == 4 * 128 + 16
    assert L.mnnq_linear_decode(FAKE, 16, 128, 64, NB, FAKE, FAKE, None, None, None, 0, None) == NULL
    assert L.mnnq_linear_decode(FAKE, 16, 128, 64, NB, FAKE, FAKE, None, ODD, None, 0, None) == ALIGN
    assert L.mnnq_linear_decode_f16(FAKE, 16, 128, 64, NB, FAKE, None, FAKE, None, 0, None) == UNSUP
    assert L.mnnq_linear_prefill_f16(FAKE, 4, 16, 128, 64, NB, FAKE, None, None, FAKE, None, 0, None) == UNSUP
    assert L.mnnq_linear_decode_f16_o16(FAKE, 16, 128, 64, NB, FAKE, None, FAKE, None) == UNSUP
    assert L.mnnq_linear_acc_debug(FAKE, 1, 16, 128, 64, NB, FAKE, FAKE, 0, None) == UNSUP
    assert L.mnnq_linear_acc_debug(FAKE, 40, 16, 128, 64, NB, FAKE, FAKE, 1, None) == UNSUP
    assert L.mnnq_linear_prefill(FAKE, 4, 16, 128, 64, NB, FAKE, FAKE, None, ODD, None, 0, None) == ALIGN
    assert L.mnnq_last_hip_error() == 0
    del i64


def test_binding_refuses_cpu_tensors(L):
    import torch
    with pytest.raises(TypeError):
        binding.mnnq_pack_weights(torch.zeros(16, 128))
    with pytest.raises(TypeError):
        binding.mnnq_quant_act(torch.zeros(1, 128))
