"""Pins for oracle_verify_attn: closed forms, invariants, and the library attention routine on the
gathered (unpaged) special case.  None of these re-run the oracle's own formula."""
import math

import numpy as np
import pytest
import torch

P, D = 16, 128


def _bits(x):
    return torch.as_tensor(np.array(x), dtype=torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _f32(bits):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()


def _paged(rng, cs, gammas, Hq, Hkv, std=1.0, D_=D):
    B = len(cs)
    n = np.asarray(gammas) + 1
    qo = np.zeros(B + 1, np.int32)
    qo[1:] = np.cumsum(n)
    pages = (np.asarray(cs) + n + P - 1) // P
    total = int(pages.sum()) + 5
    perm = rng.permutation(total).astype(np.int32)
    pt = np.full((B, int(pages.max()) + 1), -1, np.int32)
    off = 0
    for i in range(B):
        pt[i, :pages[i]] = perm[off:off + pages[i]]
        off += pages[i]
    q = _bits(rng.normal(0, std, (int(qo[-1]), Hq, D_)))
    k = _bits(rng.normal(0, std, (total, Hkv, P, D_)))
    v = _bits(rng.normal(0, std, (total, Hkv, P, D_)))
    return q, k, v, pt, np.asarray(cs, np.int32), qo


def _gather(cache, pt, i, length, kvh):
    """contiguous [length, D] fp32 view of request i's kv head, by the page table"""
    x = _f32(cache)
    rows = [x[pt[i, t // P], kvh, t % P] for t in range(length)]
    return np.stack(rows)


def test_matches_library_sdpa_on_gathered_kv(oracle):
    rng = np.random.default_rng(0)
    cs, gammas, Hq, Hkv = [37, 5, 64, 130], [4, 0, 2, 8], 8, 2
    q, k, v, pt, sl, qo = _paged(rng, cs, gammas, Hq, Hkv)
    scale = 1 / math.sqrt(D)
    out, lse = oracle.verify_attn(q, k, v, pt, sl, qo, scale, want_lse=True)
    G = Hq // Hkv
    for i in range(len(cs)):
        n = gammas[i] + 1
        L = cs[i] + n
        qi = torch.from_numpy(_f32(q)[qo[i]:qo[i + 1]]).double().permute(1, 0, 2)             # [Hq,n,D]
        K = torch.stack([torch.from_numpy(_gather(k, pt, i, L, h // G)) for h in range(Hq)]).double()
        Vv = torch.stack([torch.from_numpy(_gather(v, pt, i, L, h // G)) for h in range(Hq)]).double()
        mask = torch.arange(L)[None, :] <= (cs[i] + torch.arange(n))[:, None]                   # row j sees t <= c+j
        ref = torch.nn.functional.scaled_dot_product_attention(qi, K, Vv, attn_mask=mask, scale=scale)
        got = torch.from_numpy(out[qo[i]:qo[i + 1]]).double().permute(1, 0, 2)
        assert torch.allclose(got, ref, rtol=1e-6, atol=1e-7)
        s = torch.einsum("hnd,htd->hnt", qi, K) * scale
        ref_lse = torch.logsumexp(s.masked_fill(~mask, -math.inf), -1)
        assert torch.allclose(torch.from_numpy(lse[qo[i]:qo[i + 1]]).double().T, ref_lse, rtol=1e-6, atol=1e-6)


def test_zero_query_gives_prefix_mean_of_v(oracle):
    """q = 0 => uniform weights over exactly c+j+1 keys: out = running mean of V, lse = log(c+j+1)."""
    rng = np.random.default_rng(1)
    cs, gammas = [20, 47], [4, 2]
    q, k, v, pt, sl, qo = _paged(rng, cs, gammas, 4, 1)
    q[:] = 0
    out, lse = oracle.verify_attn(q, k, v, pt, sl, qo, 0.3, want_lse=True)
    for i in range(2):
        Vi = _gather(v, pt, i, cs[i] + gammas[i] + 1, 0).astype(np.float64)
        for j in range(gammas[i] + 1):
            nk = cs[i] + j + 1
            np.testing.assert_allclose(out[qo[i] + j, 0], Vi[:nk].mean(0), rtol=1e-6, atol=1e-7)
            np.testing.assert_allclose(lse[qo[i] + j], math.log(nk), rtol=1e-6)


def test_constant_v_is_reproduced(oracle):
    rng = np.random.default_rng(2)
    q, k, v, pt, sl, qo = _paged(rng, [33], [4], 8, 2)
    row = _bits(rng.normal(0, 1, (2, 1, D)))
    v[:] = row[None]                                          # every slot of kv head h holds the same vector
    out = oracle.verify_attn(q, k, v, pt, sl, qo, 0.1)
    want = _f32(row)[:, 0]
    for h in range(8):
        np.testing.assert_allclose(out[:, h], np.broadcast_to(want[h // 4], out[:, h].shape), rtol=1e-6, atol=1e-7)


def test_two_key_closed_form(oracle):
    """c = 1, gamma = 0: two keys; weight of key 1 is the logistic of scale * q.(k1-k0)."""
    q = _bits(np.array([[[1.0] + [0.0] * (D - 1)]]))
    k = np.zeros((2, 1, P, D), np.uint16)
    v = np.zeros((2, 1, P, D), np.uint16)
    k[1, 0, 0] = _bits(np.array([0.5] + [0.0] * (D - 1)))
    k[1, 0, 1] = _bits(np.array([2.5] + [0.0] * (D - 1)))
    v[1, 0, 0] = _bits(np.array([1.0] * D))
    v[1, 0, 1] = _bits(np.array([3.0] * D))
    pt = np.array([[1, -1]], np.int32)
    out = oracle.verify_attn(q, k, v, pt, np.array([1], np.int32), np.array([0, 1], np.int32), 0.25)
    w1 = 1 / (1 + math.exp(-0.25 * 2.0))
    np.testing.assert_allclose(out[0, 0], (1 - w1) * 1.0 + w1 * 3.0, rtol=1e-6)


def test_needle_shows_causal_boundary_and_paging(oracle):
    """A key with a huge score at candidate position c+j' is seen by rows j >= j' only."""
    rng = np.random.default_rng(3)
    c, gamma, jn = 40, 4, 2
    q, k, v, pt, sl, qo = _paged(rng, [c], [gamma], 2, 1, std=0.02)
    direction = np.ones(D) / math.sqrt(D)
    q[:] = _bits(np.broadcast_to(8.0 * direction, (gamma + 1, 2, D)))
    t = c + jn
    k[pt[0, t // P], 0, t % P] = _bits(64.0 * direction)      # score = scale*8*64 = 45 >> everything else
    v[pt[0, t // P], 0, t % P] = _bits(np.full(D, 7.0))
    out = oracle.verify_attn(q, k, v, pt, sl, qo, 1 / math.sqrt(D))
    for j in range(gamma + 1):
        if j >= jn:
            np.testing.assert_allclose(out[j], 7.0, atol=1e-3)
        else:
            assert np.abs(out[j]).max() < 0.1


def test_page_permutation_is_bit_invariant(oracle):
    rng = np.random.default_rng(4)
    q, k, v, pt, sl, qo = _paged(rng, [50, 17], [4, 2], 8, 1)
    out = oracle.verify_attn(q, k, v, pt, sl, qo, 0.088)
    perm = rng.permutation(k.shape[0])
    inv = np.empty_like(perm)
    inv[perm] = np.arange(len(perm))
    k2, v2 = k[perm], v[perm]                                   # new physical page x holds old page perm[x]
    pt2 = np.where(pt >= 0, inv[np.maximum(pt, 0)], -1).astype(np.int32)
    out2 = oracle.verify_attn(q, k2, v2, pt2, sl, qo, 0.088)
    assert np.array_equal(out, out2)


def test_future_candidate_positions_do_not_leak(oracle):
    rng = np.random.default_rng(5)
    c, gamma = 21, 4
    q, k, v, pt, sl, qo = _paged(rng, [c], [gamma], 4, 1)
    out = oracle.verify_attn(q, k, v, pt, sl, qo, 0.088)
    for jp in range(1, gamma + 1):
        k2, v2 = k.copy(), v.copy()
        t = c + jp
        k2[pt[0, t // P], 0, t % P] = _bits(rng.normal(0, 1, D))
        v2[pt[0, t // P], 0, t % P] = _bits(rng.normal(0, 1, D))
        out2 = oracle.verify_attn(q, k2, v2, pt, sl, qo, 0.088)
        assert np.array_equal(out[:jp], out2[:jp])
        assert not np.array_equal(out[jp:], out2[jp:])


def test_gqa_equals_replicated_kv_heads(oracle):
    rng = np.random.default_rng(6)
    q, k, v, pt, sl, qo = _paged(rng, [30, 9], [2, 4], 8, 2)
    out = oracle.verify_attn(q, k, v, pt, sl, qo, 0.088)
    k8, v8 = np.repeat(k, 4, axis=1), np.repeat(v, 4, axis=1)
    out8 = oracle.verify_attn(q, k8, v8, pt, sl, qo, 0.088)
    assert np.array_equal(out, out8)


def test_gamma_zero_is_plain_decode(oracle):
    """gamma = 0 for every request: each row is single-query attention over its c+1 keys (library softmax)."""
    rng = np.random.default_rng(7)
    cs = [3, 16, 31, 100]
    q, k, v, pt, sl, qo = _paged(rng, cs, [0] * 4, 2, 1)
    out = oracle.verify_attn(q, k, v, pt, sl, qo, 0.1)
    assert list(qo) == [0, 1, 2, 3, 4]
    for i, c in enumerate(cs):
        K = torch.from_numpy(_gather(k, pt, i, c + 1, 0)).double()
        Vv = torch.from_numpy(_gather(v, pt, i, c + 1, 0)).double()
        for h in range(2):
            w = torch.softmax(0.1 * (K @ torch.from_numpy(_f32(q)[i, h]).double()), 0)
            np.testing.assert_allclose(out[i, h], (w @ Vv).numpy(), rtol=1e-6, atol=1e-7)


def test_rejects_bad_shapes(oracle):
    rng = np.random.default_rng(8)
    q, k, v, pt, sl, qo = _paged(rng, [10], [1], 3, 2)       # Hq not a multiple of Hkv
    with pytest.raises(ValueError):
        oracle.verify_attn(q, k, v, pt, sl, qo, 0.1)
