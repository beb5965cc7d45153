"""The C-ABI library builds, loads, exports every symbol include/gptaq.h declares, and
rejects bad arguments on the host before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "gptaq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gptaq_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    from paper_2504_02692_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2504_02692_amd import build
        build.build(verbose=False)
    return binding.load()


def test_header_symbols_are_exported(lib):
    from paper_2504_02692_amd import binding
    names = declared_symbols()
    assert len(names) >= 9
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == names


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2504_02692_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libgptaq.so")
    with pytest.raises(binding.GptaqError):
        binding.load()


def test_workspace_queries(lib):
    assert lib.gptaq_accumulate_workspace_bytes(4096, 512) == 3 * 512 * 4096 * 2
    assert lib.gptaq_accumulate_workspace_bytes(262144, 4096) == 3 * 4096 * 32768 * 2
    assert lib.gptaq_accumulate_workspace_bytes(0, 512) == 0
    assert lib.gptaq_prepare_workspace_bytes(512) > 512 * 512 * 8
    # two sets of (-E / V of a super-block of 1024 columns, left operands of the updates inside it), the right operands
    # of one super-block for the block-by-block path, and the far right operands of every super-block that has columns
    # after it: 3072 + 2048 + 1024 rows and a 256-row tile of padding each at n = 4096, none at n = 512
    sets = lambda m: 2 * (4 * m * 1024 + 4 * (1024 // 16) * 1024 * 16) * 2
    assert lib.gptaq_quantize_workspace_bytes(512, 512) == sets(512) + 4 * (512 + 256) * 1024 * 2
    assert lib.gptaq_quantize_workspace_bytes(512, 4096) == sets(512) + 4 * (4096 + 256) * 1024 * 2 + 4 * (6144 + 3 * 256) * 1024 * 2
    assert lib.gptaq_status_string(0) == b"ok"


def test_argument_errors_are_reported_before_any_launch(lib):
    one = ctypes.c_void_p(256)      # a non-null, aligned, never dereferenced address
    null = ctypes.c_void_p(0)
    for f in (lib.gptaq_accumulate, lib.gptaq_accumulate_upper):
        assert f(null, one, 64, 64, 64, one, one, 64, one, 1 << 20, null) == -1
        assert f(one, one, 64, 60, 64, one, one, 64, one, 1 << 20, null) == -2          # n % 8
        assert f(one, one, 64, 64, 32, one, one, 64, one, 1 << 20, null) == -2          # ldx < n
        assert f(one, one, 64, 64, 64, one, one, 64, one, 16, null) == -4               # workspace
        assert f(one, one, 64, 64, 64, one, one, 64, ctypes.c_void_p(264), 1 << 20, null) == -4
        assert f(one, one, 0, 64, 64, one, one, 64, one, 1 << 20, null) == 0            # empty chunk: no-op
    assert lib.gptaq_accumulate_upper_permuted(one, one, 64, 64, 64, null, one, one, 64, one, 1 << 20, null) == -1   # inv_perm
    assert lib.gptaq_accumulate_upper_permuted(one, one, 64, 60, 64, one, one, one, 64, one, 1 << 20, null) == -2
    assert lib.gptaq_accumulate_diag(null, 64, 64, 64, one, null) == -1
    assert lib.gptaq_accumulate_diag(one, 64, 64, 32, one, null) == -2                  # ldx < n
    assert lib.gptaq_accumulate_diag(one, 0, 64, 64, one, null) == 0
    assert lib.gptaq_invert_permutation(one, 0, one, null) == -2
    assert lib.gptaq_act_order(one, 64, 32, one, null) == -2                            # 0 < ldh < n
    big = 6 * 256 * 32768
    for g in (lib.gptaq_accumulate_staged, lib.gptaq_accumulate_staged_upper):
        pend = ctypes.c_int64(0)
        assert g(one, one, 64, 64, 64, one, one, 64, one, big, None, 0, null) == -1     # pending required
        assert g(one, one, 100, 64, 64, one, one, 64, one, big, ctypes.byref(pend), 0, null) == -2   # ragged, no flush
        assert g(one, one, 64, 64, 64, one, one, 64, one, 1 << 20, ctypes.byref(pend), 0, null) == -4
        pend.value = 32
        assert g(one, one, 64, 64, 64, one, one, 64, one, big, ctypes.byref(pend), 0, null) == -2    # pending % 64
        pend.value = 0
        assert g(null, null, 0, 64, 64, one, one, 64, one, big, ctypes.byref(pend), 1, null) == 0    # empty flush: no-op
        assert pend.value == 0
    p = lib.gptaq_prepare
    assert p(one, one, 64, 64, 0.01, null, null, one, 1 << 30, null) == -1          # info required
    assert p(one, one, 64, 32, 0.01, null, one, one, 1 << 30, null) == -2
    assert p(one, one, 64, 64, 0.01, null, one, one, 1024, null) == -4
    q = lib.gptaq_quantize_layer
    ok = (one, 64, 64, 64, one, one, 64, null)
    assert q(*ok, 1, 0, 0, 128, one, one, one, one, 1 << 30, null) == -3            # bits
    assert q(*ok, 4, 48, 0, 128, one, one, one, one, 1 << 30, null) == -3           # n % group
    assert q(*ok, 4, 32, 0, 48, one, one, one, one, 1 << 30, null) == -3            # blocksize % group
    assert q(*ok, 4, 0, 0, 256, one, one, one, one, 1 << 30, null) == -3            # blocksize > 128
    assert q(*ok, 4, 0, 0, 128, one, one, one, one, 16, null) == -4
    assert b"workspace" in lib.gptaq_status_string(-4)
