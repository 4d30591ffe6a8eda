"""Host-side checks of the C-ABI library: it loads, exports every symbol the header
declares, sizes blobs as the paper's memory formula says, and rejects bad arguments before
touching the GPU.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "qg.h")


@pytest.fixture(scope="module")
def qg():
    from paper_2307_03738_amd import binding
    binding.lib()
    return binding


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qg_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(qg):
    names = _declared_symbols()
    assert {"qg_quantize", "qg_pack", "qg_unpack", "qg_gemv", "qg_gemv_grouped", "qg_gemm_small",
            "qg_packed_bytes", "qg_workspace_bytes", "qg_workspace_init", "qg_status_string",
            "qg_cell", "qg_set_gemv_tuning", "qg_set_gemm_tuning", "qg_gemv_autotune", "qg_gemv_swiglu",
            "qg_gemv_noalloc", "qg_last_gemv_kernel", "qg_gemv_record_tuning", "qg_clear_tuning",
            "qg_gemm_autotune", "qg_gemm_autotune_report", "qg_gemv_autotune_report", "qg_build_id",
            "qg_to_narrow", "qg_from_narrow", "qg_gemv_narrow", "qg_gemv_grouped_narrow",
            "qg_last_narrow_kernel"} <= set(names)
    L = qg.lib()
    for n in names:
        assert hasattr(L, n), n


def test_cells(qg):
    # Section 3: 8 codes per word at 4 bits, 16 at 2 bits, 32 codes per three words at 3 bits
    assert [qg.qg_cell(b) for b in (4, 2, 3)] == [8, 16, 32]
    assert qg.qg_cell(5) == 0


@pytest.mark.parametrize("N,K,bits,group", [(512, 512, 4, 64), (4096, 11008, 4, 128),
                                            (5120, 13824, 3, 64), (8192, 22016, 2, 32), (64, 128, 4, 128)])
def test_canonical_bytes_follow_the_memory_formula(qg, oracle, N, K, bits, group):
    # b*N*K + (32 + b)*N*K/G bits, with the zero-point stream padded to whole words per output
    got = qg.qg_packed_bytes(N, K, bits, group, qg.QG_LAYOUT_CANONICAL)
    zero_words = (K // group * bits + 31) // 32
    assert got == N * K * bits // 8 + N * (K // group) * 4 + N * zero_words * 4
    if (K // group * bits) % 32 == 0:
        assert got * 8 == oracle.storage_bits(N, K, bits, group)
    # the device layout holds the same information plus padding only
    dev = qg.qg_packed_bytes(N, K, bits, group, qg.QG_LAYOUT_DEVICE)
    assert dev >= N * K * bits // 8 + N * (K // group) * 4
    assert dev <= got * 1.02 + 3 * 256 + 64 * 3 * 1024


def test_bad_shapes_are_rejected_without_a_gpu(qg):
    assert qg.qg_packed_bytes(64, 100, 4, 32) == 0          # K % G != 0
    assert qg.qg_packed_bytes(64, 96, 4, 12) == 0           # G not a multiple of the 4-bit cell
    assert qg.qg_packed_bytes(64, 96, 3, 48) == 0           # G not a multiple of the 3-bit cell
    assert qg.qg_packed_bytes(64, 96, 5, 32) == 0           # bits
    assert qg.qg_packed_bytes(0, 96, 4, 32) == 0
    assert qg.qg_workspace_bytes(64, 96, 4, 32, 0) == 0
    L = qg.lib()
    # null pointers and misaligned pointers: an error code, nothing enqueued
    assert L.qg_gemv(None, 64, 128, 4, 32, None, None, None, 0, None) == 1
    assert L.qg_quantize(None, 64, 128, 4, 32, None, None, None, None) == 1
    assert L.qg_quantize(16, 64, 128, 7, 32, 16, 16, 16, None) == 3
    assert L.qg_quantize(16, 64, 100, 4, 32, 16, 16, 16, None) == 2
    assert L.qg_quantize(20, 64, 128, 4, 32, 16, 16, 16, None) == 4
    assert L.qg_pack(16, 16, 16, 64, 128, 4, 32, 9, 16, None) == 3
    assert L.qg_gemv(16, 64, 128, 4, 32, 64, 16, 16, 0, None) == 5      # workspace too small
    assert L.qg_gemv(16, 64, 128, 4, 32, 16, 16, 16, 0, None) == 4      # x not 64-byte aligned
    assert L.qg_gemv_grouped(None, 1, None, 0, None) == 1
    assert L.qg_gemv_swiglu(16, 100, 128, 4, 32, 64, 16, 16, 0, None) == 2     # I not a multiple of 64
    assert L.qg_gemv_swiglu(16, 128, 128, 4, 32, 64, None, 16, 1 << 20, None) == 1
    assert L.qg_gemv_swiglu(16, 128, 128, 4, 32, 64, 16, 16, 0, None) == 5      # workspace too small
    assert L.qg_gemv_autotune(None, 1, 1, None, 0, None, 5, None, None, None, None) == 1
    assert L.qg_gemv_autotune(None, 1, 1, None, 0, None, 0, None, None, None, None) == 2   # repeats <= 0
    assert L.qg_gemm_small(16, 64, 128, 4, 32, 64, 0, 16, 16, 1 << 20, None) == 2          # M <= 0
    assert L.qg_gemm_small(16, 64, 128, 4, 32, 64, 129, 16, 16, 1 << 20, None) == 2        # M > 128
    assert L.qg_set_gemm_tuning(9, 0) == 2 and L.qg_set_gemm_tuning(0, 14) == 2 and L.qg_set_gemm_tuning(0, 0) == 0
    assert L.qg_set_gemv_tuning(99, 0, 0) == 2 and L.qg_set_gemv_tuning(0, 0, 5) == 2
    assert L.qg_set_gemv_tuning(0, 0, 0) == 0
    assert b"aligned" in L.qg_status_string(4)


@pytest.mark.parametrize("N,K,bits,group", [(4096, 4096, 4, 128), (4096, 11008, 4, 128), (100, 1024, 4, 16),
                                            (5120, 13824, 3, 64), (8192, 22016, 2, 32), (70, 512, 2, 16), (1, 256, 3, 256)])
def test_narrow_bytes_follow_the_record_formula(qg, N, K, bits, group):
    # one record per 16 outputs and 4 steps of K: the steps' codes, a scale per group and lane of
    # 64, the zero-points of the 64 lanes packed and padded to 16 bytes; the blob to 256 bytes
    step = 128 if bits == 4 else 256
    groups = step // group
    zero_bits = 2 if bits == 2 else 4
    record = 4 * 16 * step * bits // 8 + groups * 64 * 4 + -(-(64 * groups * zero_bits // 8) // 16) * 16
    records = -(-N // 16) * -(-(K // step) // 4)
    assert qg.qg_packed_bytes(N, K, bits, group, qg.QG_LAYOUT_DEVICE_NARROW) == -(-records * record // 256) * 256
    # algorithmic bytes plus padding only
    assert records * record >= N * K * bits // 8 + N * (K // group) * 4


def test_narrow_calls_reject_bad_arguments_without_a_gpu(qg):
    L = qg.lib()
    for (N, K, bits, group) in [(64, 192, 4, 64), (64, 1024, 4, 256), (64, 1024, 4, 8), (16, 65536, 4, 128),
                                (64, 1024, 3, 1024), (64, 1024, 3, 16)]:
        assert qg.qg_packed_bytes(N, K, bits, group, qg.QG_LAYOUT_DEVICE_NARROW) == 0
        assert L.qg_to_narrow(16, N, K, bits, group, 16, None) in (2, 3)
    assert L.qg_to_narrow(None, 64, 1024, 4, 128, 16, None) == 1
    assert L.qg_to_narrow(16, 64, 1024, 4, 128, 24, None) == 4              # narrow not 16-byte aligned
    assert L.qg_from_narrow(16, 64, 1024, 4, 128, None, None) == 1
    assert L.qg_gemv_narrow(None, 64, 1024, 4, 128, 64, 64, None) == 1
    assert L.qg_gemv_narrow(16, 64, 1024, 4, 128, 16, 64, None) == 4        # x not 64-byte aligned
    assert L.qg_gemv_narrow(16, 64, 1000, 4, 128, 64, 64, None) == 2        # K % G != 0
    assert L.qg_gemv_grouped_narrow(None, 1, None) == 1
    assert L.qg_set_narrow_tuning(3) == 2 and L.qg_set_narrow_tuning(0) == 0
