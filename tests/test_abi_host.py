"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/qspec.h declares, and rejects bad arguments before it
touches the device."""
import os
import re

import pytest

from paper_2410_11305_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "qspec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qspec_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    L = B.lib()
    names = _declared_symbols()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_size_queries():
    assert B.version() >= 1000
    assert B.packed_weight_bytes(1024, 1024) == 1024 * 1024 // 2 + 1024 * 8 * 2
    assert B.packed_weight_bytes(4096, 11008) == 4096 * 11008 // 2 + 4096 * 86 * 2
    assert B.packed_weight_bytes(1024, 1000) == 0          # K not a multiple of 128
    assert B.packed_weight_bytes(1000, 1024) == 0          # N not a multiple of 16
    assert B.packed_weight_bytes(1024, 1024, 64) == 0      # group size is fixed
    assert B.workspace_bytes(0, 1024, 1024) == 0
    for code in range(8):
        assert B.status_string(code)


@pytest.mark.parametrize("fn", ["qspec_gemm_w4a16", "qspec_gemm_w4a4"])
def test_gemm_argument_validation_without_device(fn):
    L = B.lib()
    a = 4096          # any 16-byte aligned non-null address: rejected before use
    if fn == "qspec_gemm_w4a16":
        call = lambda packed, act, M, N, K, g, y: L.qspec_gemm_w4a16(packed, act, M, N, K, g, y, None, 0, None)
    else:
        call = lambda packed, act, M, N, K, g, y: L.qspec_gemm_w4a4(packed, act, a, M, N, K, g, y, None, 0, None)
    assert call(None, a, 1, 16, 128, 128, a) == B.ERR_NULL
    assert call(a, a, 1, 16, 128, 128, None) == B.ERR_NULL
    assert call(a, a, 0, 16, 128, 128, a) == B.ERR_SHAPE
    assert call(a, a, 1, 24, 128, 128, a) == B.ERR_SHAPE
    assert call(a, a, 1, 16, 192, 128, a) == B.ERR_SHAPE
    assert call(a, a, 1, 16, 128, 64, a) == B.ERR_SHAPE
    assert call(a, a + 2, 1, 16, 128, 128, a) == B.ERR_ALIGN
    assert call(a + 8, a, 1, 16, 128, 128, a) == B.ERR_ALIGN


def test_other_entries_validate_without_device():
    L = B.lib()
    a = 4096
    assert L.qspec_pack_weights(None, a, 16, 128, 128, a, None) == B.ERR_NULL
    assert L.qspec_pack_weights(a, a, 8, 128, 128, a, None) == B.ERR_SHAPE
    assert L.qspec_pack_weights(a, a + 4, 16, 128, 128, a, None) == B.ERR_ALIGN
    assert L.qspec_unpack_weights(a, 16, 100, 128, a, a, None) == B.ERR_SHAPE
    assert L.qspec_quant_act(a, 0, 128, 128, a, a, None) == B.ERR_SHAPE
    assert L.qspec_quant_act(a, 1, 128, 128, None, a, None) == B.ERR_NULL
    assert L.qspec_quant_act(a + 1, 1, 128, 128, a, a, None) == B.ERR_ALIGN
    assert L.qspec_gemm_w4a4_partials(a, a, 1, 32, 128, 128, 8, 16, a, None) == B.ERR_SHAPE
    assert L.qspec_gemm_w4a4_partials(a, a, 1, 32, 128, 128, 16, 32, a, None) == B.ERR_SHAPE
    assert L.qspec_gemm_w4a4_partials(a, a, 1, 32, 128, 128, 0, 0, a, None) == B.ERR_SHAPE
    assert L.qspec_gemm_w4a4_partials(a, a, 1, 32, 128, 128, 0, 32, None, None) == B.ERR_NULL


def test_accept_entries_validate_without_device():
    L = B.lib()
    a = 4096
    assert B.accept_workspace_bytes(8, 3, 32000) == 8 * 4 * 8 * 8          # 8 chunks of 4000 logits per row
    assert B.accept_workspace_bytes(1, 1, 17) == 2 * 8
    assert B.accept_workspace_bytes(0, 3, 32000) == 0
    assert B.accept_workspace_bytes(20000, 3, 32000) == 0                  # more than 65535 logits rows
    assert L.qspec_greedy_accept(None, a, 1, 1, 16, a, a, a, 64, None) == B.ERR_NULL
    assert L.qspec_greedy_accept(a, a, 1, 1, 16, a, a, None, 0, None) == B.ERR_NULL
    assert L.qspec_greedy_accept(a, a, 1, 0, 16, a, a, a, 64, None) == B.ERR_SHAPE
    assert L.qspec_greedy_accept(a, a, 1, 1, 0, a, a, a, 64, None) == B.ERR_SHAPE
    assert L.qspec_greedy_accept(a + 2, a, 1, 1, 16, a, a, a, 64, None) == B.ERR_ALIGN
    assert L.qspec_greedy_accept(a, a + 2, 1, 1, 16, a, a, a, 64, None) == B.ERR_ALIGN
    assert L.qspec_greedy_accept(a, a, 1, 1, 16, a, a, a, 8, None) == B.ERR_WORKSPACE
    assert L.qspec_kv_overwrite(a, a, a, 1, 1, 12, 4, a, None) == B.ERR_SHAPE    # D not a multiple of 8
    assert L.qspec_kv_overwrite(a, a, a, 1, 1, 16, 0, a, None) == B.ERR_SHAPE
    assert L.qspec_kv_overwrite(a, None, a, 1, 1, 16, 4, a, None) == B.ERR_NULL
    assert L.qspec_kv_overwrite(a, a, a, 1, 1, 16, 4, a + 4, None) == B.ERR_ALIGN


def test_producer_and_outlier_entries_validate_without_device():
    L = B.lib()
    a = 4096
    eps = 1e-5
    assert L.qspec_rmsnorm_quant(None, a, eps, 1, 128, 128, 0, a, a, None, None) == B.ERR_NULL
    assert L.qspec_rmsnorm_quant(a, None, eps, 1, 128, 128, 0, a, a, None, None) == B.ERR_NULL
    assert L.qspec_rmsnorm_quant(a, a, eps, 0, 128, 128, 0, a, a, None, None) == B.ERR_SHAPE
    assert L.qspec_rmsnorm_quant(a, a, eps, 1, 192, 128, 0, a, a, None, None) == B.ERR_SHAPE
    assert L.qspec_rmsnorm_quant(a, a, -1.0, 1, 128, 128, 0, a, a, None, None) == B.ERR_SHAPE
    assert L.qspec_rmsnorm_quant(a, a, float("inf"), 1, 128, 128, 0, a, a, None, None) == B.ERR_SHAPE
    assert L.qspec_rmsnorm_quant(a, a, eps, 1, 128, 128, 4, a, a, None, None) == B.ERR_SHAPE        # flag bits 0 and 1 only
    assert L.qspec_rmsnorm_quant(a, a + 8, eps, 1, 128, 128, 0, a, a, None, None) == B.ERR_ALIGN
    assert L.qspec_rmsnorm_quant(a, a, eps, 1, 128, 128, 0, a, a, a + 2, None) == B.ERR_ALIGN
    assert L.qspec_silu_mul_quant(None, 1, 128, 128, 0, a, a, None, None) == B.ERR_NULL
    assert L.qspec_silu_mul_quant(a, 1, 100, 128, 0, a, a, None, None) == B.ERR_SHAPE
    assert L.qspec_silu_mul_quant(a, 1, 128, 128, -1, a, a, None, None) == B.ERR_SHAPE
    assert L.qspec_silu_mul_quant(a, 1, 128, 128, 0, a + 4, a, None, None) == B.ERR_ALIGN
    assert L.qspec_hadamard_quant(a, 1, 128, 128, None, a, None, None) == B.ERR_NULL
    assert L.qspec_hadamard_quant(a, 1, 128, 64, a, a, None, None) == B.ERR_SHAPE
    assert L.qspec_hadamard_quant(a + 2, 1, 128, 128, a, a, None, None) == B.ERR_ALIGN
    assert L.qspec_reorder_quant(a, None, 1, 128, 128, 1, a, a, None, None) == B.ERR_NULL
    assert L.qspec_reorder_quant(a, a, 1, 128, 128, 2, a, a, None, None) == B.ERR_SHAPE             # more outlier groups than groups
    assert L.qspec_reorder_quant(a, a, 1, 128, 128, -1, a, a, None, None) == B.ERR_SHAPE
    assert L.qspec_reorder_quant(a, a + 4, 1, 128, 128, 1, a, a, None, None) == B.ERR_ALIGN
