"""Thin Python binding of libspecverify.so: argument marshalling only.

Every function has the name and the argument order of the C entry point in include/spec_verify.h and
hands it device pointers of torch tensors plus torch's current HIP stream.  Nothing is computed here;
if the library is missing the import fails (there is no fallback path).
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecverify.so")

EXPORTS = (
    "spec_last_error_string", "spec_version", "spec_set_tuning",
    "spec_verify_attn_workspace_bytes", "spec_verify_attn", "spec_lm_head",
    "spec_accept_workspace_bytes", "spec_accept", "spec_kv_commit", "spec_next_mode",
    "spec_lm_head_stats_blocks", "spec_lm_head_stats", "spec_accept_stats", "spec_assemble_next",
    "spec_divergence", "spec_kv_truncate", "spec_compress_prompts",
    "spec_verify_attn_tree", "spec_accept_tree", "spec_kv_commit_tree",
    "spec_lm_head_packed_bytes", "spec_lm_head_pack", "spec_lm_head_packed",
    "spec_lm_head_packed_stats_blocks", "spec_lm_head_packed_stats",
    "spec_probe_read", "spec_probe_read_pages", "spec_probe_mfma", "spec_accept_static",
    "spec_lm_head_packed_summary_blocks", "spec_lm_head_packed_summary", "spec_accept_summary",
)

FLAG_BAD_PAGE, FLAG_BAD_LENGTH, FLAG_BAD_LOGITS, FLAG_BAD_TOKEN, FLAG_FREE_OVERFLOW, FLAG_NO_SEED = 1, 2, 4, 8, 16, 32
FLAG_BAD_TREE = 64


class SpecError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"libspecverify status {code}: {text}")
        self.code = code


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, f32, u32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_uint32, ctypes.c_size_t
    lib.spec_last_error_string.restype = ctypes.c_char_p
    lib.spec_last_error_string.argtypes = []
    lib.spec_version.restype = i32
    lib.spec_set_tuning.restype = i32
    lib.spec_set_tuning.argtypes = [ctypes.c_char_p, i32]
    lib.spec_verify_attn_workspace_bytes.restype = sz
    lib.spec_verify_attn_workspace_bytes.argtypes = [i32] * 7
    lib.spec_verify_attn.restype = i32
    lib.spec_verify_attn.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp, vp,
                                     i32, i32, i32, i32, i32, i32, i32, i32, f32, vp, vp, sz, vp]
    lib.spec_lm_head.restype = i32
    lib.spec_lm_head.argtypes = [vp, vp, vp, i32, i32, i32, vp]
    lib.spec_accept_workspace_bytes.restype = sz
    lib.spec_accept_workspace_bytes.argtypes = [i32] * 4
    lib.spec_accept.restype = i32
    lib.spec_accept.argtypes = [vp, vp, vp, vp, vp, u32, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.spec_accept_static.restype = i32
    lib.spec_accept_static.argtypes = [vp, vp, vp, vp, vp, u32, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp]
    lib.spec_kv_commit.restype = i32
    lib.spec_kv_commit.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp, i32, i32, vp, vp]
    lib.spec_lm_head_stats_blocks.restype = i32
    lib.spec_lm_head_stats_blocks.argtypes = [i32] * 3
    lib.spec_lm_head_stats.restype = i32
    lib.spec_lm_head_stats.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp]
    lib.spec_lm_head_packed_bytes.restype = sz
    lib.spec_lm_head_packed_bytes.argtypes = [i32, i32]
    lib.spec_lm_head_pack.restype = i32
    lib.spec_lm_head_pack.argtypes = [vp, vp, i32, i32, vp]
    lib.spec_lm_head_packed.restype = i32
    lib.spec_lm_head_packed.argtypes = [vp, vp, vp, i32, i32, i32, vp]
    lib.spec_lm_head_packed_stats_blocks.restype = i32
    lib.spec_lm_head_packed_stats_blocks.argtypes = [i32] * 3
    lib.spec_lm_head_packed_stats.restype = i32
    lib.spec_lm_head_packed_stats.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp]
    lib.spec_lm_head_packed_summary_blocks.restype = i32
    lib.spec_lm_head_packed_summary_blocks.argtypes = [i32] * 3
    lib.spec_lm_head_packed_summary.restype = i32
    lib.spec_lm_head_packed_summary.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, i32, vp, vp, vp, vp]
    lib.spec_accept_summary.restype = i32
    lib.spec_accept_summary.argtypes = [vp, vp, vp, vp, vp, u32, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, i32, vp, vp, sz, vp]
    lib.spec_accept_stats.restype = i32
    lib.spec_accept_stats.argtypes = [vp, vp, vp, vp, vp, u32, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, i32, vp, vp, sz, vp]
    lib.spec_verify_attn_tree.restype = i32
    lib.spec_verify_attn_tree.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp,
                                          i32, i32, i32, i32, i32, i32, i32, i32, f32, vp, vp, sz, vp]
    lib.spec_accept_tree.restype = i32
    lib.spec_accept_tree.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.spec_kv_commit_tree.restype = i32
    lib.spec_kv_commit_tree.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp, i32, vp, i32, vp, i32, i32, i32, i32, vp, vp]
    lib.spec_divergence.restype = i32
    lib.spec_divergence.argtypes = [vp, vp, vp, vp, vp, i32, vp]
    lib.spec_kv_truncate.restype = i32
    lib.spec_kv_truncate.argtypes = [vp, i32, vp, vp, vp, i32, vp, i32, i32, vp, vp]
    lib.spec_compress_prompts.restype = i32
    lib.spec_compress_prompts.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp]
    lib.spec_assemble_next.restype = i32
    lib.spec_assemble_next.argtypes = [vp, vp, i32, vp, i32, vp, i32, vp, vp, i32, vp, i32, i32, vp, vp, vp, vp, vp]
    lib.spec_probe_read.restype = i32
    lib.spec_probe_read.argtypes = [vp, sz, vp, vp]
    lib.spec_probe_read_pages.restype = i32
    lib.spec_probe_read_pages.argtypes = [vp, vp, i32, vp, vp]
    lib.spec_probe_mfma.restype = ctypes.c_double
    lib.spec_probe_mfma.argtypes = [i32, i32, vp, vp]
    lib.spec_next_mode.restype = i32
    lib.spec_next_mode.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                   ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    return lib


_lib = _load()


def _ptr(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc):
    if rc != 0:
        raise SpecError(rc, _lib.spec_last_error_string().decode())


def spec_version():
    return _lib.spec_version()


MODE_ORDINARY, MODE_PARALLEL = 0, 1


def spec_assemble_next(accept_len, out_tokens, qo_indptr, cont, cont_len, repair, repair_len, mode, gamma_next,
                       next_tokens, next_qo_indptr, rollback, stats):
    B = accept_len.shape[0]
    gamma_max = out_tokens.shape[1] - 1
    assert next_tokens.numel() >= B * (gamma_next + 1) and next_qo_indptr.numel() == B + 1
    _check(_lib.spec_assemble_next(
        _ptr(accept_len, torch.int32), _ptr(out_tokens, torch.int32), gamma_max, _ptr(qo_indptr, torch.int32), B,
        _ptr(cont, torch.int32), cont.shape[1] if cont is not None else 0, _ptr(cont_len, torch.int32),
        _ptr(repair, torch.int32), repair.shape[1] if repair is not None else 0, _ptr(repair_len, torch.int32),
        int(mode), int(gamma_next), _ptr(next_tokens, torch.int32), _ptr(next_qo_indptr, torch.int32),
        _ptr(rollback, torch.uint8), _ptr(stats, torch.int32), _stream()))


def spec_next_mode(stats_host, gamma, t_draft, t_target):
    """(mode, r_hat, r_star) from a host copy of spec_accept's stats[4]."""
    arr = (ctypes.c_int32 * 4)(*[int(x) for x in stats_host])
    rh, rs = ctypes.c_double(), ctypes.c_double()
    mode = _lib.spec_next_mode(arr, float(gamma), float(t_draft), float(t_target), ctypes.byref(rh), ctypes.byref(rs))
    _check(mode if mode < 0 else 0)
    return int(mode), rh.value, rs.value


def spec_set_tuning(key: str, value: int):
    _check(_lib.spec_set_tuning(key.encode(), int(value)))


def spec_verify_attn_workspace_bytes(B, M, Hq, Hkv, D, max_kv_len, max_q_len):
    return int(_lib.spec_verify_attn_workspace_bytes(B, M, Hq, Hkv, D, max_kv_len, max_q_len))


def spec_verify_attn(q, k_cache, v_cache, page_table, seq_lens, qo_indptr, out, lse, max_kv_len, max_q_len, scale,
                     status_flags, workspace):
    M, Hq, D = q.shape
    num_pages, Hkv, P, _ = k_cache.shape
    B = seq_lens.shape[0]
    _check(_lib.spec_verify_attn(
        _ptr(q, torch.bfloat16), _ptr(k_cache, torch.bfloat16), _ptr(v_cache, torch.bfloat16),
        _ptr(page_table, torch.int32), page_table.shape[1], num_pages, _ptr(seq_lens, torch.int32),
        _ptr(qo_indptr, torch.int32), _ptr(out, torch.bfloat16), _ptr(lse, torch.float32),
        B, M, Hq, Hkv, D, P, int(max_kv_len), int(max_q_len), float(scale), _ptr(status_flags, torch.int32),
        _ptr(workspace), workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream()))


def spec_lm_head(hidden, W, logits):
    M, H = hidden.shape
    V = W.shape[0]
    assert W.shape[1] == H and tuple(logits.shape) == (M, V)
    _check(_lib.spec_lm_head(_ptr(hidden, torch.bfloat16), _ptr(W, torch.bfloat16), _ptr(logits, torch.float32),
                             M, H, V, _stream()))


def spec_lm_head_stats_blocks(M, H, V):
    return int(_lib.spec_lm_head_stats_blocks(int(M), int(H), int(V)))


def spec_lm_head_stats(hidden, W, logits, blk_max, blk_arg):
    M, H = hidden.shape
    V = W.shape[0]
    assert W.shape[1] == H and tuple(logits.shape) == (M, V)
    _check(_lib.spec_lm_head_stats(_ptr(hidden, torch.bfloat16), _ptr(W, torch.bfloat16), _ptr(logits, torch.float32),
                                   M, H, V, _ptr(blk_max, torch.float32), _ptr(blk_arg, torch.int32), _stream()))


def spec_lm_head_packed_bytes(V, H):
    return int(_lib.spec_lm_head_packed_bytes(int(V), int(H)))


def spec_lm_head_pack(W, Wp):
    """W [V, H] bf16 -> Wp, a flat bf16 tensor of spec_lm_head_packed_bytes(V, H) / 2 elements."""
    V, H = W.shape
    assert Wp.numel() * Wp.element_size() == spec_lm_head_packed_bytes(V, H)
    _check(_lib.spec_lm_head_pack(_ptr(W, torch.bfloat16), _ptr(Wp, torch.bfloat16), V, H, _stream()))


def spec_lm_head_packed(hidden, Wp, logits):
    M, H = hidden.shape
    V = logits.shape[1]
    assert logits.shape[0] == M and Wp.numel() * Wp.element_size() == spec_lm_head_packed_bytes(V, H)
    _check(_lib.spec_lm_head_packed(_ptr(hidden, torch.bfloat16), _ptr(Wp, torch.bfloat16), _ptr(logits, torch.float32),
                                    M, H, V, _stream()))


def spec_lm_head_packed_stats_blocks(M, H, V):
    return int(_lib.spec_lm_head_packed_stats_blocks(int(M), int(H), int(V)))


def spec_lm_head_packed_stats(hidden, Wp, logits, blk_max, blk_arg):
    M, H = hidden.shape
    V = logits.shape[1]
    assert logits.shape[0] == M and Wp.numel() * Wp.element_size() == spec_lm_head_packed_bytes(V, H)
    blocks = spec_lm_head_packed_stats_blocks(M, H, V)
    assert tuple(blk_max.shape) == (M, blocks) and tuple(blk_arg.shape) == (M, blocks)
    _check(_lib.spec_lm_head_packed_stats(_ptr(hidden, torch.bfloat16), _ptr(Wp, torch.bfloat16), _ptr(logits, torch.float32),
                                          M, H, V, _ptr(blk_max, torch.float32), _ptr(blk_arg, torch.int32), _stream()))


def spec_lm_head_packed_summary_blocks(M, H, V):
    return int(_lib.spec_lm_head_packed_summary_blocks(int(M), int(H), int(V)))


def spec_lm_head_packed_summary(hidden, Wp, logits, temperature, qo_indptr, blk_max, blk_sum, blk_span):
    M, H = hidden.shape
    V = logits.shape[1]
    B = qo_indptr.shape[0] - 1
    assert logits.shape[0] == M and Wp.numel() * Wp.element_size() == spec_lm_head_packed_bytes(V, H)
    blocks = spec_lm_head_packed_summary_blocks(M, H, V)
    assert blocks > 0, "spec_lm_head_packed_summary does not take this shape"
    assert temperature.numel() == B and tuple(blk_max.shape) == (M, blocks) and tuple(blk_sum.shape) == (M, blocks)
    assert tuple(blk_span.shape) == (blocks, 2)
    _check(_lib.spec_lm_head_packed_summary(_ptr(hidden, torch.bfloat16), _ptr(Wp, torch.bfloat16), _ptr(logits, torch.float32),
                                            M, H, V, _ptr(temperature, torch.float32), _ptr(qo_indptr, torch.int32), B,
                                            _ptr(blk_max, torch.float32), _ptr(blk_sum, torch.float32),
                                            _ptr(blk_span, torch.int32), _stream()))


def spec_accept_workspace_bytes(B, M, V, gamma_max):
    return int(_lib.spec_accept_workspace_bytes(B, M, V, gamma_max))


def spec_accept(logits, tokens, draft_probs, temperature, seeds, round_, qo_indptr, accept_len, out_tokens, rollback,
                stats, gamma_max, status_flags, workspace):
    M, V = logits.shape
    B = qo_indptr.shape[0] - 1
    assert tuple(out_tokens.shape) == (B, gamma_max + 1)
    _check(_lib.spec_accept(
        _ptr(logits, torch.float32), _ptr(tokens, torch.int32), _ptr(draft_probs, torch.float32),
        _ptr(temperature, torch.float32), _ptr(seeds, torch.int64), int(round_), _ptr(qo_indptr, torch.int32),
        _ptr(accept_len, torch.int32), _ptr(out_tokens, torch.int32), _ptr(rollback, torch.uint8),
        _ptr(stats, torch.int32), B, M, V, int(gamma_max), _ptr(status_flags, torch.int32),
        _ptr(workspace), workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream()))


def spec_accept_static(logits, tokens, draft_probs, temperature, seeds, round_, qo_indptr, accept_len, out_tokens, rollback,
                       stats, gamma_max, status_flags):
    M, V = logits.shape
    B = qo_indptr.shape[0] - 1
    assert tuple(out_tokens.shape) == (B, gamma_max + 1)
    _check(_lib.spec_accept_static(
        _ptr(logits, torch.float32), _ptr(tokens, torch.int32), _ptr(draft_probs, torch.float32),
        _ptr(temperature, torch.float32), _ptr(seeds, torch.int64), int(round_), _ptr(qo_indptr, torch.int32),
        _ptr(accept_len, torch.int32), _ptr(out_tokens, torch.int32), _ptr(rollback, torch.uint8),
        _ptr(stats, torch.int32), B, M, V, int(gamma_max), _ptr(status_flags, torch.int32), _stream()))


def spec_accept_stats(logits, tokens, draft_probs, temperature, seeds, round_, qo_indptr, accept_len, out_tokens, rollback,
                      stats, gamma_max, blk_max, blk_arg, blocks, status_flags, workspace):
    M, V = logits.shape
    B = qo_indptr.shape[0] - 1
    assert tuple(out_tokens.shape) == (B, gamma_max + 1)
    assert blocks == 0 or (tuple(blk_max.shape) == (M, blocks) and tuple(blk_arg.shape) == (M, blocks))
    _check(_lib.spec_accept_stats(
        _ptr(logits, torch.float32), _ptr(tokens, torch.int32), _ptr(draft_probs, torch.float32),
        _ptr(temperature, torch.float32), _ptr(seeds, torch.int64), int(round_), _ptr(qo_indptr, torch.int32),
        _ptr(accept_len, torch.int32), _ptr(out_tokens, torch.int32), _ptr(rollback, torch.uint8),
        _ptr(stats, torch.int32), B, M, V, int(gamma_max),
        _ptr(blk_max, torch.float32) if blocks else None, _ptr(blk_arg, torch.int32) if blocks else None, int(blocks),
        _ptr(status_flags, torch.int32),
        _ptr(workspace), workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream()))


def spec_accept_summary(logits, tokens, draft_probs, temperature, seeds, round_, qo_indptr, accept_len, out_tokens, rollback,
                        stats, gamma_max, blk_max, blk_sum, blk_span, blocks, status_flags, workspace):
    M, V = logits.shape
    B = qo_indptr.shape[0] - 1
    assert tuple(out_tokens.shape) == (B, gamma_max + 1)
    assert blocks == 0 or (tuple(blk_max.shape) == (M, blocks) and tuple(blk_sum.shape) == (M, blocks)
                           and tuple(blk_span.shape) == (blocks, 2))
    _check(_lib.spec_accept_summary(
        _ptr(logits, torch.float32), _ptr(tokens, torch.int32), _ptr(draft_probs, torch.float32),
        _ptr(temperature, torch.float32), _ptr(seeds, torch.int64), int(round_), _ptr(qo_indptr, torch.int32),
        _ptr(accept_len, torch.int32), _ptr(out_tokens, torch.int32), _ptr(rollback, torch.uint8),
        _ptr(stats, torch.int32), B, M, V, int(gamma_max),
        _ptr(blk_max, torch.float32) if blocks else None, _ptr(blk_sum, torch.float32) if blocks else None,
        _ptr(blk_span, torch.int32) if blocks else None, int(blocks),
        _ptr(status_flags, torch.int32),
        _ptr(workspace), workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream()))


def spec_kv_commit(page_table, seq_lens, qo_indptr, accept_len, free_list, free_count, page_size, status_flags):
    B = seq_lens.shape[0]
    _check(_lib.spec_kv_commit(
        _ptr(page_table, torch.int32), page_table.shape[1], _ptr(seq_lens, torch.int32), _ptr(qo_indptr, torch.int32),
        _ptr(accept_len, torch.int32), _ptr(free_list, torch.int32), free_list.shape[0], _ptr(free_count, torch.int32),
        B, int(page_size), _ptr(status_flags, torch.int32), _stream()))


def spec_divergence(p_tokens, p_indptr, h_tokens, h_indptr, delta):
    B = p_indptr.shape[0] - 1
    _check(_lib.spec_divergence(_ptr(p_tokens, torch.int32), _ptr(p_indptr, torch.int32), _ptr(h_tokens, torch.int32),
                                _ptr(h_indptr, torch.int32), _ptr(delta, torch.int32), B, _stream()))


def spec_kv_truncate(page_table, seq_lens, keep_len, free_list, free_count, page_size, status_flags):
    B = seq_lens.shape[0]
    _check(_lib.spec_kv_truncate(
        _ptr(page_table, torch.int32), page_table.shape[1], _ptr(seq_lens, torch.int32), _ptr(keep_len, torch.int32),
        _ptr(free_list, torch.int32), free_list.shape[0], _ptr(free_count, torch.int32), B, int(page_size),
        _ptr(status_flags, torch.int32), _stream()))


def spec_compress_prompts(tokens, indptr, p_num, p_den, out_tokens, out_indptr, kept_index):
    B = indptr.shape[0] - 1
    assert out_tokens.numel() >= tokens.numel() and out_indptr.numel() == B + 1
    _check(_lib.spec_compress_prompts(_ptr(tokens, torch.int32), _ptr(indptr, torch.int32), B, int(p_num), int(p_den),
                                      _ptr(out_tokens, torch.int32), _ptr(out_indptr, torch.int32),
                                      _ptr(kept_index, torch.int32), _stream()))


def spec_verify_attn_tree(q, k_cache, v_cache, page_table, seq_lens, qo_indptr, parent, out, lse, max_kv_len, max_q_len, scale,
                          status_flags, workspace):
    M, Hq, D = q.shape
    num_pages, Hkv, P, _ = k_cache.shape
    B = seq_lens.shape[0]
    _check(_lib.spec_verify_attn_tree(
        _ptr(q, torch.bfloat16), _ptr(k_cache, torch.bfloat16), _ptr(v_cache, torch.bfloat16),
        _ptr(page_table, torch.int32), page_table.shape[1], num_pages, _ptr(seq_lens, torch.int32),
        _ptr(qo_indptr, torch.int32), _ptr(parent, torch.int32), _ptr(out, torch.bfloat16), _ptr(lse, torch.float32),
        B, M, Hq, Hkv, D, P, int(max_kv_len), int(max_q_len), float(scale), _ptr(status_flags, torch.int32),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def spec_accept_tree(logits, tokens, parent, qo_indptr, accept_len, out_tokens, path, rollback, stats, gamma_max,
                     status_flags, workspace):
    M, V = logits.shape
    B = qo_indptr.shape[0] - 1
    assert tuple(out_tokens.shape) == (B, gamma_max + 1) and tuple(path.shape) == (B, gamma_max + 1)
    _check(_lib.spec_accept_tree(
        _ptr(logits, torch.float32), _ptr(tokens, torch.int32), _ptr(parent, torch.int32), _ptr(qo_indptr, torch.int32),
        _ptr(accept_len, torch.int32), _ptr(out_tokens, torch.int32), _ptr(path, torch.int32), _ptr(rollback, torch.uint8),
        _ptr(stats, torch.int32), B, M, V, int(gamma_max), _ptr(status_flags, torch.int32),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def spec_kv_commit_tree(k_cache, v_cache, page_table, seq_lens, qo_indptr, accept_len, path, free_list, free_count,
                        status_flags):
    num_pages, Hkv, P, D = k_cache.shape
    B = seq_lens.shape[0]
    _check(_lib.spec_kv_commit_tree(
        _ptr(k_cache, torch.bfloat16), _ptr(v_cache, torch.bfloat16), _ptr(page_table, torch.int32), page_table.shape[1],
        num_pages, _ptr(seq_lens, torch.int32), _ptr(qo_indptr, torch.int32), _ptr(accept_len, torch.int32),
        _ptr(path, torch.int32), path.shape[1] - 1, _ptr(free_list, torch.int32), free_list.shape[0],
        _ptr(free_count, torch.int32), B, Hkv, D, P, _ptr(status_flags, torch.int32), _stream()))



def spec_probe_read(src, sink):
    """Linear read of the whole tensor `src`, once."""
    _check(_lib.spec_probe_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream()))


def spec_probe_read_pages(src, pages, sink):
    """Reads the 4 KB pages of `src` listed in `pages` (int32), each once."""
    assert src.numel() * src.element_size() >= (int(pages.max()) + 1) * 4096 if pages.numel() else True
    _check(_lib.spec_probe_read_pages(_ptr(src), _ptr(pages, torch.int32), pages.numel(), _ptr(sink), _stream()))


def spec_probe_mfma(iters, constant_operands, sink):
    """MFMA-only loop; returns the floating-point operations of the launch."""
    flops = float(_lib.spec_probe_mfma(int(iters), int(constant_operands), _ptr(sink), _stream()))
    _check(0 if flops > 0 else -1)
    return flops
