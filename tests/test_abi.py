"""The C-ABI library loads without a GPU and exports every function that
include/ha_rag.h declares; the Python binding names the same set."""
import ctypes
import os
import re

from paper_2510_20878_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ha_rag.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ha_rag_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert len(names) >= 20
    dll = ctypes.CDLL(B.lib_path())
    for n in names:
        assert hasattr(dll, n), n
    assert sorted(B.SYMBOLS) == names


def test_strerror_and_version():
    assert B.version().startswith("ha_rag")
    assert B.strerror(B.OK) == "ok"
    for code in (B.EINVAL, B.ENOENT, B.ENOSPC, B.EFORMAT, B.EHIP, B.EIO):
        assert B.strerror(code) and B.strerror(code) != "unknown error code"


def test_struct_sizes_match_the_header_layout():
    assert ctypes.sizeof(B.Config) == 52
    assert ctypes.sizeof(B.PackedChunk) == 24
    assert ctypes.sizeof(B.ChunkTrace) == 24
    assert ctypes.sizeof(B.LoadStats) == 12 * 4 + 7 * 8
    assert ctypes.sizeof(B.ChunkInfo) == 8 * 4 + 2 * 8 + 2 * 8
