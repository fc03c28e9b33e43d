"""CPU-side checks of the C ABI: the shared library loads, exports every function the
header declares, and its host-only logic (names, sizes, argument checks that come before
any device work) behaves as the header says.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "quota.h")
LIB = os.path.join(ROOT, "paper_2604_17320_amd", "libquota.so")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)          # comments out
    src = re.sub(r"typedef\s+struct\s+\w*\s*\{.*?\}\s*\w+\s*;", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(quota_[a-z0-9_]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail("libquota.so is not built: run __graft_entry__.build() first")
    return C.CDLL(LIB)


def test_header_declares_the_boundary_calls():
    names = declared_functions()
    for must in ("quota_quantize_act", "quota_w4a4_gemm", "quota_score_tokens", "quota_topk_prune",
                 "quota_kv_quant_append", "quota_prefill_layer"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    missing = [n for n in declared_functions() if not hasattr(lib, n)]
    assert not missing, f"declared in quota.h but not exported: {missing}"


def test_binding_mirrors_the_header():
    from paper_2604_17320_amd import binding
    missing = [n for n in declared_functions() if not hasattr(binding, n)]
    assert not missing, f"declared in quota.h but absent from the Python binding: {missing}"


def test_kernel_names_and_strerror(lib):
    lib.quota_kernel_name.restype = C.c_char_p
    lib.quota_strerror.restype = C.c_char_p
    from paper_2604_17320_amd import binding
    names = [lib.quota_kernel_name(i).decode() for i in range(binding.KERNEL_COUNT)]
    assert len(set(names)) == binding.KERNEL_COUNT and "?" not in names
    assert lib.quota_kernel_name(binding.KERNEL_COUNT).decode() == "?"
    assert lib.quota_kernel_name(-1).decode() == "?"
    msgs = [lib.quota_strerror(c).decode() for c in range(0, -6, -1)]
    assert len(set(msgs)) == 6                                 # distinct text per error code
    assert lib.quota_strerror(-99).decode() not in msgs


def test_null_and_shape_checks_come_before_device_work(lib):
    # every call below must be rejected on the host: there is no GPU in this process
    ERR_NULL = -1
    assert lib.quota_quantize_act(None, 4, 128, 128, None, None, None, None, None) == ERR_NULL
    assert lib.quota_w4a4_gemm(None, None, 4, None, None, 0, None, 0, None, None) == ERR_NULL
    assert lib.quota_topk_prune(None, 1, 8, 4, None, None) == ERR_NULL
    assert lib.quota_prefill_layer(None, None, 0, None, None, None, None, None) == ERR_NULL
    lib.quota_prefill_workspace_bytes.restype = C.c_size_t
    assert lib.quota_prefill_workspace_bytes(None, 1, 16) == 0
    lib.quota_attention_workspace_bytes.restype = C.c_size_t
    assert lib.quota_attention_workspace_bytes(1, 640, 32, 128) > 0
