"""Host logic of the launchers, checked without a GPU through mnnq_plan_debug: for every layer shape of
the benchmark models the chosen kernel configuration fits the hardware limits the kernels assume
(1024 threads, 160 KiB of LDS per workgroup), covers the whole
problem, and is the one the design documents for the Qwen2-7B shapes.  Nothing is launched."""
import os

import pytest

from paper_2506_10443_amd import binding as B, synth

LDS_GEMM, LDS_GEMV = 160 * 1024, 160 * 1024


@pytest.fixture(scope="module", autouse=True)
def built():
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    for v in ("MNNQ_PREFILL_TILE", "MNNQ_DECODE_KSPLIT", "MNNQ_DECODE_WAVES", "MNNQ_DECODE_EARLY", "MNNQ_W8_PLANES"):
        B.mnnq_debug_set(v, None)


def shapes():
    out = []
    for model, spec in synth.MODELS.items():
        for fused in (True, False):
            for name, N, K in synth.block_layers(model, fused=fused):
                out.append((model, name, spec["prefill_m"], N, K))
        if spec["lm_head"]:
            out.append((model, "lm_head", spec["prefill_m"], *spec["lm_head"]))
    return out


@pytest.mark.parametrize("mode", [B.MODE_W4_ZP_INT, B.MODE_W4_MIN_FLOAT, B.MODE_W8_MIN_FLOAT])
@pytest.mark.parametrize("model,name,M,N,K", shapes())
def test_prefill_plan_fits_and_covers(model, name, M, N, K, mode):
    for m in sorted({M, 17, 100, 129, 300}):
        bm, bn, ks, s, waves, lds, wgs, merged = B.mnnq_plan_debug(0, m, N, K, mode)
        assert (bm, bn) in ((64, 64), (64, 128), (128, 128), (256, 128)) and ks in (1, 2, 4) and s in (1, 2)
        assert (bm == 64) == (m <= 128 and not merged and not (m > 64 and -(-N // 128) >= 1024))
        assert ks < 4 or bm == 64
        assert waves in (4, 8, 16) and waves * 64 <= 1024 and waves % ks == 0
        assert lds <= LDS_GEMM
        if waves // ks == 4:
            assert 2 * lds <= LDS_GEMM or ks >= 2      # the four-wave forms count on two workgroups per CU
        assert wgs >= -(-m // bm) * s * -(-N // bn)     # every output tile (and K part) has a workgroup
        assert merged == (1 if mode == B.MODE_W8_MIN_FLOAT else 0)
        if merged:
            assert bm == 128


@pytest.mark.parametrize("mode", [B.MODE_W4_ZP_INT, B.MODE_W4_MIN_FLOAT, B.MODE_W8_MIN_FLOAT])
@pytest.mark.parametrize("model,name,M,N,K", shapes())
def test_decode_plan_fits_and_covers(model, name, M, N, K, mode):
    chunks = -(-(K * (2 if mode == B.MODE_W8_MIN_FLOAT else 1)) // 128)
    tiles = N // 16
    for what in (1, 2):
        if chunks * 128 > 126976:
            with pytest.raises(B.MnnqError):
                B.mnnq_plan_debug(what, 1, N, K, mode)
            continue
        waves, ks, unroll, prefetch, lds, wgs, tiles_per_wg, _ = B.mnnq_plan_debug(what, 1, N, K, mode)
        assert waves in (4, 8, 16) and ks in (1, 2, 4, 8, 16) and waves % ks == 0 and tiles_per_wg == waves // ks
        assert lds <= LDS_GEMV
        assert wgs * tiles_per_wg >= tiles
        per_wave = -(-chunks // ks)
        assert prefetch == (1 if per_wave > unroll else 0)      # else the whole range sits in registers


def test_documented_plans_of_the_qwen2_7b_block():
    plan = lambda n, k: B.mnnq_plan_debug(0, 1024, n, k)[:5]
    assert plan(37888, 3584) == [256, 128, 1, 1, 8]      # gate|up: two workgroups of eight waves per CU
    assert plan(4608, 3584) == [256, 128, 2, 1, 16]      # q|k|v: two K parts of eight waves
    assert plan(3584, 3584) == [128, 128, 2, 1, 16]      # o
    assert plan(3584, 18944) == [128, 128, 2, 1, 16]     # down
    assert B.mnnq_plan_debug(1, 1, 37888, 3584)[:4] == [4, 4, 7, 0]      # GEMV: four waves per row tile, 7 chunks each
    assert B.mnnq_plan_debug(1, 1, 3584, 18944)[:4] == [16, 16, 12, 0]   # 148 chunks over sixteen waves
    assert B.mnnq_plan_debug(1, 1, 4096, 14336)[:4] == [16, 16, 7, 0]    # (Llama-3-8B down) 112 chunks: seven each
    assert B.mnnq_plan_debug(2, 1, 4608, 3584)[0] == 8                    # fused quantizer: larger workgroups
    # the activation row is handled under the weight stream where (nearly) every wave's registers are filled:
    # small layers with at most two chunks fewer per wave than registers for them, and exactly fitting ones
    early = lambda what, n, k: B.mnnq_plan_debug(what, 1, n, k)[7]
    shapes = ((4608, 3584), (3584, 3584), (3584, 18944), (37888, 3584))
    assert [early(1, n, k) for n, k in shapes] == [1, 1, 0, 1]
    assert [early(2, n, k) for n, k in shapes] == [1, 1, 0, 1]
    assert B.mnnq_plan_debug(2, 1, 3584, 3584)[:3] == [8, 8, 4]    # fused o: eight waves per row tile, 3 - 4 chunks each
    assert early(1, 1536, 8960) == 0 and early(1, 2048, 1536) == 1  # Qwen2-1.5B down (4 - 5 of 8 chunks) and q|k|v


def test_plans_of_the_byte_form_of_int8_weights():
    """mode MNNQ_W8_MIN_FLOAT | MNNQ_NATIVE_8BIT: the GEMV keeps seven chunks of two kilobytes per wave in
    registers (a rolling window beyond sixteen waves per row tile), the GEMM runs 128 x 128 tiles."""
    NB = B.MODE_W8_MIN_FLOAT | B.NATIVE_8BIT
    for model, name, M, N, K in shapes():
        if K % 128:
            continue
        chunks = K // 128
        for what in (1, 2):
            waves, ks, unroll, prefetch, lds, wgs, tiles_per_wg, early = B.mnnq_plan_debug(what, 1, N, K, NB)
            assert unroll == 7 and early == 0 and waves % ks == 0 and tiles_per_wg == waves // ks
            assert ks == 16 or -(-chunks // ks) <= 7
            assert prefetch == (1 if -(-chunks // ks) > 7 else 0)
            assert (waves, ks) in (((4, 1), (4, 2), (4, 4), (8, 8), (16, 16)) if what == 1 else
                                   ((8, 1), (8, 2), (8, 4), (8, 8), (16, 16)))
            assert lds <= LDS_GEMV and wgs * tiles_per_wg >= N // 16
        bm, bn, kparts, s, w, lds, wgs, form = B.mnnq_plan_debug(0, M, N, K, NB)
        assert (bm, bn, form) == (128, 128, 2) and kparts in (1, 2) and lds <= LDS_GEMM
        assert wgs >= -(-M // 128) * s * -(-N // 128)
    assert B.mnnq_plan_debug(1, 1, 152064, 3584, NB)[:4] == [4, 4, 7, 0]     # LM head: 28 chunks on four waves
    assert B.mnnq_plan_debug(1, 1, 3584, 18944, NB)[:4] == [16, 16, 7, 1]    # down: 148 chunks, a window of seven


def test_documented_plans_for_few_tokens():
    """Batched decoding (17 .. 128 tokens): 64-row tiles, 64 columns wide unless there are very many,
    the K range in more parts the fewer workgroups there are; very many tiles beyond 64 tokens take
    128-row tiles."""
    plan = lambda m, n, k: B.mnnq_plan_debug(0, m, n, k)[:5]
    assert plan(64, 4608, 3584) == [64, 64, 4, 1, 16]        # q|k|v: 72 workgroups
    assert plan(64, 3584, 18944) == [64, 64, 4, 2, 16]       # down: long rows cut in two as well
    assert plan(64, 37888, 3584) == [64, 64, 2, 1, 8]        # gate|up: 592 workgroups, two to three per CU
    assert plan(128, 37888, 3584) == [64, 64, 1, 1, 4]       # 1184 workgroups of four waves
    assert plan(64, 152064, 3584) == [64, 128, 1, 1, 4]      # lm_head: 1188 tiles of 64 x 128
    assert plan(128, 152064, 3584) == [128, 128, 1, 1, 4]    # ... and 128-row tiles beyond 64 tokens


def test_switches_and_errors():
    B.mnnq_debug_set("MNNQ_PREFILL_TILE", "s1")
    try:
        assert B.mnnq_plan_debug(0, 1024, 37888, 3584)[:5] == [128, 128, 1, 1, 4]
    finally:
        B.mnnq_debug_set("MNNQ_PREFILL_TILE", None)
    B.mnnq_debug_set("MNNQ_W8_PLANES", "1")
    try:
        assert B.mnnq_plan_debug(0, 1024, 37888, 3584, B.MODE_W8_MIN_FLOAT)[7] == 0
    finally:
        B.mnnq_debug_set("MNNQ_W8_PLANES", None)
    # the library does not read the environment: a stray variable changes nothing
    os.environ["MNNQ_PREFILL_TILE"] = "s1"
    try:
        assert B.mnnq_plan_debug(0, 1024, 37888, 3584)[:5] != [128, 128, 1, 1, 4]
    finally:
        os.environ.pop("MNNQ_PREFILL_TILE")
    L = B.lib()
    assert L.mnnq_debug_set(b"MNNQ_NO_SUCH_SWITCH", b"1") == -3 and L.mnnq_debug_set(None, b"1") == -1
    assert L.mnnq_debug_set(b"MNNQ_PREFILL_TILE", b"0123456789abcdef") == -4
    assert L.mnnq_plan_debug(0, 4, 16, 128, 64, 0, None) == -1
    import ctypes
    out = (ctypes.c_int32 * 8)()
    p = ctypes.cast(out, ctypes.c_void_p)
    assert L.mnnq_plan_debug(3, 4, 16, 128, 64, 0, p) == -3
    assert L.mnnq_plan_debug(0, 0, 16, 128, 64, 0, p) == -2
    assert L.mnnq_plan_debug(1, 1, 16, 100, 64, 0, p) == -2
    assert L.mnnq_plan_debug(1, 1, 16, 131072, 64, 0, p) == -3    # longer than the GEMV stages in LDS
    assert L.mnnq_plan_debug(1, 1, 16, 53248, 64, 0, p) == 0 and out[4] > 64 * 1024 and out[4] <= 160 * 1024
