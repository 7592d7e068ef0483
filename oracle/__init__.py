"""ctypes front end of the CPU oracle (oracle/spec_oracle.c).

TEST INFRASTRUCTURE ONLY: importable from tests/, the smoke check and the
cpu_baseline leg of bench.py.  The GPU library and its Python binding never
import this package, and this package imports nothing of theirs.

All arrays are numpy, on the host.  bf16 tensors travel as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spec_oracle.c")
# ORACLE_LIB in the environment names an instrumented build of the same source (a test makes one with extra
# compiler checks and reruns the pins on it); it is loaded as it is and never rebuilt here.
_PREBUILT = os.environ.get("ORACLE_LIB", "")
_LIB = _PREBUILT or os.path.join(_HERE, "libspec_oracle.so")
CFLAGS = ["-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math: summation order is part of the definition)."""
    if _PREBUILT:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"], check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_uniform.restype = ctypes.c_float
        lib.oracle_uniform.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32]
        for name in ("oracle_thr_ordinary", "oracle_thr_parallel", "oracle_r_star"):
            getattr(lib, name).restype = ctypes.c_double
        lib.oracle_thr_ordinary.argtypes = [ctypes.c_double] * 5
        lib.oracle_thr_parallel.argtypes = [ctypes.c_double] * 4
        lib.oracle_r_star.argtypes = [ctypes.c_double] * 4
        lib.oracle_next_mode.restype = ctypes.c_int
        lib.oracle_next_mode.argtypes = [ctypes.c_int] * 3 + [ctypes.c_double] * 3 + [ctypes.POINTER(ctypes.c_double)] * 2
        _lib = lib
    return _lib


def _p(a, dtype):
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what} rejected its arguments (status {rc})")


def verify_attn(q, k_cache, v_cache, page_table, seq_lens, qo_indptr, scale, want_lse=False):
    """q [M,Hq,D] u16(bf16); caches [pages,Hkv,P,D] u16; returns fp32 out [M,Hq,D] (and lse [M,Hq])."""
    M, Hq, D = q.shape
    _, Hkv, P, D2 = k_cache.shape
    assert D2 == D and v_cache.shape == k_cache.shape
    B = seq_lens.shape[0]
    out = np.zeros((M, Hq, D), np.float32)
    lse = np.zeros((M, Hq), np.float32) if want_lse else None
    rc = _load().oracle_verify_attn(
        _p(q, np.uint16), _p(k_cache, np.uint16), _p(v_cache, np.uint16),
        _p(page_table, np.int32), ctypes.c_int(page_table.shape[1]),
        _p(seq_lens, np.int32), _p(qo_indptr, np.int32), _p(out, np.float32), _p(lse, np.float32),
        B, M, Hq, Hkv, D, P, ctypes.c_float(scale))
    _check(rc, "oracle_verify_attn")
    return (out, lse) if want_lse else out


def lm_head(hidden, W):
    """hidden [M,H] u16(bf16), W [V,H] u16(bf16) -> logits fp32 [M,V]."""
    M, H = hidden.shape
    V, H2 = W.shape
    assert H == H2
    logits = np.zeros((M, V), np.float32)
    _check(_load().oracle_lm_head(_p(hidden, np.uint16), _p(W, np.uint16), _p(logits, np.float32), M, H, V),
           "oracle_lm_head")
    return logits


def philox4x32_10(ctr, key):
    c = (ctypes.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (ctypes.c_uint32 * 4)()
    _load().oracle_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def uniform(seed, round_, j, tag):
    return float(_load().oracle_uniform(int(seed), int(round_), int(j), int(tag)))


def target_probs(logits_row, T):
    V = logits_row.shape[0]
    p = np.zeros(V, np.float32)
    _check(_load().oracle_target_probs(_p(logits_row, np.float32), V, ctypes.c_float(T), _p(p, np.float32)),
           "oracle_target_probs")
    return p


def accept(logits, tokens, draft_probs, temperature, seeds, round_, qo_indptr, gamma_max):
    """Returns dict(accept_len [B] i32, out_tokens [B,gamma_max+1] i32, rollback [B] u8, status int)."""
    M, V = logits.shape
    B = qo_indptr.shape[0] - 1
    accept_len = np.zeros(B, np.int32)
    out_tokens = np.zeros((B, gamma_max + 1), np.int32)
    rollback = np.zeros(B, np.uint8)
    status = np.zeros(1, np.int32)
    rc = _load().oracle_accept(
        _p(logits, np.float32), _p(tokens, np.int32), _p(draft_probs, np.float32),
        _p(temperature, np.float32), _p(seeds, np.uint64), ctypes.c_uint32(round_),
        _p(qo_indptr, np.int32), _p(accept_len, np.int32), _p(out_tokens, np.int32),
        _p(rollback, np.uint8), _p(status, np.int32), B, M, V, gamma_max)
    _check(rc, "oracle_accept")
    return dict(accept_len=accept_len, out_tokens=out_tokens, rollback=rollback, status=int(status[0]))


def kv_commit(page_table, seq_lens, qo_indptr, accept_len, free_list, free_count, page_size):
    """In place on page_table [B,max_pages], seq_lens [B], free_list [cap], free_count [1]."""
    B = seq_lens.shape[0]
    rc = _load().oracle_kv_commit(
        _p(page_table, np.int32), ctypes.c_int(page_table.shape[1]), _p(seq_lens, np.int32),
        _p(qo_indptr, np.int32), _p(accept_len, np.int32), _p(free_list, np.int32),
        ctypes.c_int32(free_list.shape[0]), _p(free_count, np.int32), B, page_size)
    _check(rc, "oracle_kv_commit")


def thr_ordinary(B, L, gamma, T_D, T_T):
    return float(_load().oracle_thr_ordinary(B, L, gamma, T_D, T_T))


def thr_parallel(B, L, r, T_T):
    return float(_load().oracle_thr_parallel(B, L, r, T_T))


def r_star(L, gamma, T_D, T_T):
    return float(_load().oracle_r_star(L, gamma, T_D, T_T))


def next_mode(rollback_count, emitted, B, gamma, T_D, T_T):
    """(mode, r_hat, r_star): mode 1 = PARALLEL, 0 = ORDINARY (Method, eq. mode_switch_batch)."""
    rh, rs = ctypes.c_double(), ctypes.c_double()
    mode = _load().oracle_next_mode(int(rollback_count), int(emitted), int(B), float(gamma), float(T_D), float(T_T),
                                    ctypes.byref(rh), ctypes.byref(rs))
    return int(mode), rh.value, rs.value


def assemble_next(accept_len, out_tokens, qo_indptr, cont, cont_len, repair, repair_len, mode, gamma_next):
    """Candidates of the next round (Method, eqs. ordinary_* / parallel_*; Appendix, eq. target_suffix_reuse).
    cont / repair: int32 [B, C] / [B, R] with per-request lengths, or None.  Returns a dict."""
    lib = _load()
    B = accept_len.shape[0]
    gamma_max = out_tokens.shape[1] - 1
    nt = np.full(B * (gamma_next + 1), -7, np.int32)
    nqo = np.zeros(B + 1, np.int32)
    rb = np.zeros(B, np.uint8)
    st = np.zeros(4, np.int32)
    null = ctypes.c_void_p(None)
    lib.oracle_assemble_next.restype = ctypes.c_int
    rows = lib.oracle_assemble_next(
        _p(accept_len, np.int32), _p(out_tokens, np.int32), ctypes.c_int(gamma_max), _p(qo_indptr, np.int32), ctypes.c_int(B),
        _p(cont, np.int32) if cont is not None else null, ctypes.c_int(cont.shape[1] if cont is not None else 0),
        _p(cont_len, np.int32) if cont is not None else null,
        _p(repair, np.int32) if repair is not None else null, ctypes.c_int(repair.shape[1] if repair is not None else 0),
        _p(repair_len, np.int32) if repair is not None else null,
        ctypes.c_int(mode), ctypes.c_int(gamma_next), _p(nt, np.int32), _p(nqo, np.int32),
        rb.ctypes.data_as(ctypes.c_void_p), _p(st, np.int32))
    _check(min(rows, 0), "oracle_assemble_next")
    return dict(tokens=nt[:rows].copy(), qo_indptr=nqo, rollback=rb, stats=st, rows=rows)


def divergence(p_tokens, p_indptr, h_tokens, h_indptr):
    """delta_i = first position where request i's verified prefix and the draft's own tokens differ
    (Appendix "Draft side", "Message handling and update")."""
    B = p_indptr.shape[0] - 1
    delta = np.zeros(B, np.int32)
    _check(_load().oracle_divergence(_p(p_tokens, np.int32), _p(p_indptr, np.int32), _p(h_tokens, np.int32),
                                     _p(h_indptr, np.int32), _p(delta, np.int32), ctypes.c_int(B)), "oracle_divergence")
    return delta


def kv_truncate(page_table, seq_lens, keep_len, free_list, free_count, page_size):
    """Rollback(S, delta) on the paged cache, in place (Appendix "Draft side", "State recovery")."""
    B = seq_lens.shape[0]
    rc = _load().oracle_kv_truncate(
        _p(page_table, np.int32), ctypes.c_int(page_table.shape[1]), _p(seq_lens, np.int32), _p(keep_len, np.int32),
        _p(free_list, np.int32), ctypes.c_int32(free_list.shape[0]), _p(free_count, np.int32), B, page_size)
    _check(rc, "oracle_kv_truncate")


def compress_prompts(tokens, indptr, p_num, p_den):
    """E(x) of eq. token_eviction on a ragged batch; returns (out_tokens, out_indptr, kept_index)."""
    lib = _load()
    lib.oracle_compress_prompts.restype = ctypes.c_long
    B = indptr.shape[0] - 1
    out = np.full(max(1, tokens.shape[0]), -7, np.int32)
    idx = np.full(max(1, tokens.shape[0]), -7, np.int32)
    oip = np.zeros(B + 1, np.int32)
    n = lib.oracle_compress_prompts(_p(tokens, np.int32), _p(indptr, np.int32), ctypes.c_int(B), ctypes.c_int(p_num),
                                    ctypes.c_int(p_den), _p(out, np.int32), _p(oip, np.int32), _p(idx, np.int32))
    _check(min(n, 0), "oracle_compress_prompts")
    return out[:n].copy(), oip, idx[:n].copy()


def verify_attn_tree(q, k_cache, v_cache, page_table, seq_lens, qo_indptr, parent, scale, want_lse=False):
    """Tree attention: row j sees the committed prefix and its own root path (Appendix, "Unified verification interface")."""
    M, Hq, D = q.shape
    _, Hkv, P, _ = k_cache.shape
    B = seq_lens.shape[0]
    out = np.zeros((M, Hq, D), np.float32)
    lse = np.zeros((M, Hq), np.float32) if want_lse else None
    rc = _load().oracle_verify_attn_tree(
        _p(q, np.uint16), _p(k_cache, np.uint16), _p(v_cache, np.uint16), _p(page_table, np.int32),
        ctypes.c_int(page_table.shape[1]), _p(seq_lens, np.int32), _p(qo_indptr, np.int32), _p(parent, np.int32),
        _p(out, np.float32), _p(lse, np.float32), B, M, Hq, Hkv, D, P, ctypes.c_float(scale))
    _check(rc, "oracle_verify_attn_tree")
    return (out, lse) if want_lse else out


def accept_tree(logits, tokens, parent, qo_indptr, gamma_max):
    M, V = logits.shape
    B = qo_indptr.shape[0] - 1
    accept_len = np.zeros(B, np.int32)
    out_tokens = np.zeros((B, gamma_max + 1), np.int32)
    path = np.zeros((B, gamma_max + 1), np.int32)
    rollback = np.zeros(B, np.uint8)
    status = np.zeros(1, np.int32)
    rc = _load().oracle_accept_tree(_p(logits, np.float32), _p(tokens, np.int32), _p(parent, np.int32), _p(qo_indptr, np.int32),
                                    _p(accept_len, np.int32), _p(out_tokens, np.int32), _p(path, np.int32),
                                    _p(rollback, np.uint8), _p(status, np.int32), B, M, V, gamma_max)
    _check(rc, "oracle_accept_tree")
    return dict(accept_len=accept_len, out_tokens=out_tokens, path=path, rollback=rollback, status=int(status[0]))


def kv_commit_tree(k_cache, v_cache, page_table, seq_lens, qo_indptr, accept_len, path, free_list, free_count, page_size):
    """In place: gathers the accepted path's K/V to positions c+1.., then commits as kv_commit."""
    B = seq_lens.shape[0]
    _, Hkv, P, D = k_cache.shape
    rc = _load().oracle_kv_commit_tree(
        _p(k_cache, np.uint16), _p(v_cache, np.uint16), _p(page_table, np.int32), ctypes.c_int(page_table.shape[1]),
        _p(seq_lens, np.int32), _p(qo_indptr, np.int32), _p(accept_len, np.int32), _p(path, np.int32),
        ctypes.c_int(path.shape[1] - 1), _p(free_list, np.int32), ctypes.c_int32(free_list.shape[0]),
        _p(free_count, np.int32), B, Hkv, D, page_size)
    _check(rc, "oracle_kv_commit_tree")

