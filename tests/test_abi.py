"""The C-ABI library loads and exports every function include/spec_verify.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "spec_verify.h")
LIB = os.path.join(ROOT, "paper_2605_08151_amd", "libspecverify.so")


def _declared():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(spec_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_calls():
    names = _declared()
    for need in ("spec_verify_attn", "spec_lm_head", "spec_accept", "spec_kv_commit"):
        assert need in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    lib = ctypes.CDLL(LIB)
    for name in _declared():
        assert hasattr(lib, name), name
    assert lib.spec_version() >= 1000


def test_host_side_argument_checks_need_no_gpu():
    lib = ctypes.CDLL(LIB)
    lib.spec_last_error_string.restype = ctypes.c_char_p
    lib.spec_lm_head.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int] * 3 + [ctypes.c_void_p]
    assert lib.spec_lm_head(None, None, None, 1, 64, 1, None) == -1
    assert lib.spec_lm_head(None, None, None, 0, 64, 1, None) == 0
    assert b"NULL" in lib.spec_last_error_string()
    lib.spec_verify_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.spec_verify_attn_workspace_bytes.argtypes = [ctypes.c_int] * 7
    assert lib.spec_verify_attn_workspace_bytes(32, 160, 32, 8, 128, 2053, 5) > 0
    lib.spec_accept_workspace_bytes.restype = ctypes.c_size_t
    lib.spec_accept_workspace_bytes.argtypes = [ctypes.c_int] * 4
    assert lib.spec_accept_workspace_bytes(32, 160, 151936, 4) > 0
    # the packed LM head: size arithmetic, and shapes and pointers rejected before anything is launched
    lib.spec_lm_head_packed_bytes.restype = ctypes.c_size_t
    lib.spec_lm_head_packed_bytes.argtypes = [ctypes.c_int] * 2
    assert lib.spec_lm_head_packed_bytes(151936, 4096) == 151936 * 4096 * 2
    assert lib.spec_lm_head_packed_bytes(1013, 256) == 1024 * 256 * 2          # entries padded to whole panels of 16
    assert lib.spec_lm_head_packed_bytes(0, 256) == 0
    lib.spec_lm_head_packed.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int] * 3 + [ctypes.c_void_p]
    assert lib.spec_lm_head_packed(None, None, None, 4, 256, 40, None) == -1    # NULL operands
    assert lib.spec_lm_head_packed(None, None, None, 0, 256, 40, None) == 0     # no rows: nothing to do
    assert lib.spec_lm_head_packed(None, None, None, -1, 256, 40, None) == -1
    one = ctypes.c_void_p(256)                                                  # aligned, never dereferenced on the host
    assert lib.spec_lm_head_packed(one, one, one, 4, 192, 40, None) == -2       # H must be a multiple of 256
    assert b"256" in lib.spec_last_error_string()
    assert lib.spec_lm_head_packed(one, one, one, 4, 256, 7_000_000, None) == -2    # row offsets would leave 32 bits
    lib.spec_lm_head_pack.argtypes = [ctypes.c_void_p] * 2 + [ctypes.c_int] * 2 + [ctypes.c_void_p]
    assert lib.spec_lm_head_pack(one, one, 40, 48, None) == -2                  # H must be a multiple of 32
    assert lib.spec_lm_head_pack(None, None, 0, 64, None) == 0
    lib.spec_lm_head_packed_stats_blocks.argtypes = [ctypes.c_int] * 3
    assert lib.spec_lm_head_packed_stats_blocks(160, 192, 4000) == 0


def test_binding_names_match_the_header():
    import paper_2605_08151_amd.binding as b
    for name in _declared():
        assert name in b.EXPORTS and hasattr(b, name) or name == "spec_last_error_string", name
