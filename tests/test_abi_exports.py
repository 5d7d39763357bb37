"""The built C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import os
import re

from paper_2511_04805_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "puzzle_moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(pzl_[a-z_0-9]+)\s*\(", text))
    assert declared == set(binding.EXPORTS), declared ^ set(binding.EXPORTS)
    lib = binding.load()
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.pzl_abi_version() == 6
    assert lib.pzl_moe_ffn_static_max_bytes() == 32 << 20
    assert lib.pzl_packed_bytes(14336, 4096) == 14336 * 4096 * 2
    assert lib.pzl_strerror(0) == b"ok" and b"workspace" in lib.pzl_strerror(binding.PZL_ENOSPC)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """There is no CPU fallback: without the built library the binding raises, it never computes."""
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libpuzzle_moe.so"))
    import pytest
    with pytest.raises(RuntimeError, match="not built"):
        binding.load()
    with pytest.raises(RuntimeError, match="not built"):
        binding.pzl_moe_ffn_plan(8, 128, 256, 4, 2)
