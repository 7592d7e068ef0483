"""Pins for the tree-structured verification routines of the oracle (Appendix "Target side", "Unified verification
interface"): the chain as the degenerate tree, the library attention routine with an ancestor mask, hand-worked
acceptance walks, and the K/V gather of an accepted path."""
import math

import numpy as np
import torch

from test_oracle_attn import D, P, _f32, _gather, _paged


def _random_parents(rng, gammas):
    """row-local parent of every candidate row: a random tree per request, rows in topological order"""
    out = []
    for g in gammas:
        out.append(-1)
        out += [int(rng.integers(0, j)) for j in range(1, g + 1)]
    return np.array(out, np.int32)


def _chain_parents(gammas):
    return np.concatenate([np.arange(-1, g, dtype=np.int32) for g in gammas])


def _ancestors(parent_local, j):
    s = set()
    while j >= 0:
        s.add(j)
        j = int(parent_local[j])
    return s


def test_chain_is_the_degenerate_tree(oracle):
    rng = np.random.default_rng(0)
    cs, gammas, Hq, Hkv = [37, 5, 64, 0], [4, 0, 2, 8], 8, 2
    q, k, v, pt, sl, qo = _paged(rng, cs, gammas, Hq, Hkv)
    scale = 1 / math.sqrt(D)
    a, la = oracle.verify_attn(q, k, v, pt, sl, qo, scale, want_lse=True)
    b, lb = oracle.verify_attn_tree(q, k, v, pt, sl, qo, _chain_parents(gammas), scale, want_lse=True)
    assert np.array_equal(a, b) and np.array_equal(la, lb)
    V = 50
    logits = rng.normal(0, 1, (int(qo[-1]), V)).astype(np.float32)
    tokens = rng.integers(0, V, int(qo[-1])).astype(np.int32)
    am = logits.argmax(1)
    for i, g in enumerate(gammas):                       # plant accepted prefixes of different lengths
        for j in range(1, min(g, i + 1) + 1):
            tokens[qo[i] + j] = am[qo[i] + j - 1]
    chain = oracle.accept(logits, tokens, None, np.zeros(len(cs), np.float32), None, 0, qo, 8)
    tree = oracle.accept_tree(logits, tokens, _chain_parents(gammas), qo, 8)
    assert np.array_equal(chain["accept_len"], tree["accept_len"]) and np.array_equal(chain["out_tokens"], tree["out_tokens"])
    assert np.array_equal(chain["rollback"], tree["rollback"])
    for i in range(len(cs)):
        a_i = tree["accept_len"][i]
        assert tree["path"][i, :a_i + 1].tolist() == list(range(a_i + 1)) and (tree["path"][i, a_i + 1:] == -1).all()


def test_tree_attention_matches_library_sdpa_with_an_ancestor_mask(oracle):
    rng = np.random.default_rng(1)
    cs, gammas, Hq, Hkv = [37, 5, 64, 130, 0], [6, 0, 3, 12, 4], 4, 2
    q, k, v, pt, sl, qo = _paged(rng, cs, gammas, Hq, Hkv)
    parent = _random_parents(rng, gammas)
    scale = 1 / math.sqrt(D)
    out, lse = oracle.verify_attn_tree(q, k, v, pt, sl, qo, parent, scale, want_lse=True)
    G = Hq // Hkv
    for i in range(len(cs)):
        n, c = gammas[i] + 1, cs[i]
        L = c + n
        pl = parent[qo[i]:qo[i + 1]]
        mask = torch.zeros((n, L), dtype=torch.bool)
        mask[:, :c] = True
        for j in range(n):
            for a in _ancestors(pl, j):
                mask[j, c + a] = True
        qi = torch.from_numpy(_f32(q)[qo[i]:qo[i + 1]]).double().permute(1, 0, 2)
        K = torch.stack([torch.from_numpy(_gather(k, pt, i, L, h // G)) for h in range(Hq)]).double()
        Vv = torch.stack([torch.from_numpy(_gather(v, pt, i, L, h // G)) for h in range(Hq)]).double()
        ref = torch.nn.functional.scaled_dot_product_attention(qi, K, Vv, attn_mask=mask, scale=scale)
        np.testing.assert_allclose(out[qo[i]:qo[i + 1]], ref.permute(1, 0, 2).numpy(), rtol=1e-6, atol=1e-7)
    # a sibling's key must not leak: changing the K/V of a row changes only the rows that have it on their path
    i = 3
    pl = parent[qo[i]:qo[i + 1]]
    victim = 5
    k2, v2 = k.copy(), v.copy()
    t = cs[i] + victim
    k2[pt[i, t // P], :, t % P] ^= 0x0101
    v2[pt[i, t // P], :, t % P] ^= 0x0101
    out2 = oracle.verify_attn_tree(q, k2, v2, pt, sl, qo, parent, scale)
    for j in range(gammas[i] + 1):
        same = np.array_equal(out2[qo[i] + j], out[qo[i] + j])
        assert same == (victim not in _ancestors(pl, j))


def test_tree_acceptance_hand_worked(oracle):
    # root 0; children 1 (token 5) and 2 (token 7); node 2 has children 3 (token 9) and 4 (token 11); node 1 has child 5 (token 11)
    parent = np.array([-1, 0, 0, 2, 2, 1], np.int32)
    tokens = np.array([0, 5, 7, 9, 11, 11], np.int32)
    qo = np.array([0, 6], np.int32)
    V = 16

    def run(argmax_per_row):
        logits = np.zeros((6, V), np.float32)
        for r, a in enumerate(argmax_per_row):
            logits[r, a] = 1.0
        return oracle.accept_tree(logits, tokens, parent, qo, 5)

    r = run([7, 0, 11, 0, 3, 0])                          # 0 -> 2 (token 7) -> 4 (token 11) -> leaf, bonus 3
    assert r["accept_len"][0] == 2 and r["out_tokens"][0].tolist() == [7, 11, 3, -1, -1, -1]
    assert r["path"][0].tolist() == [0, 2, 4, -1, -1, -1] and r["rollback"][0] == 0
    r = run([6, 0, 0, 0, 0, 0])                           # no child of the root carries token 6: bonus 6, rollback
    assert r["accept_len"][0] == 0 and r["out_tokens"][0].tolist() == [6, -1, -1, -1, -1, -1] and r["rollback"][0] == 1
    r = run([7, 0, 10, 0, 0, 0])                          # 0 -> 2, then neither 9 nor 11: bonus 10, node 2 had children
    assert r["accept_len"][0] == 1 and r["out_tokens"][0].tolist()[:2] == [7, 10] and r["path"][0].tolist()[:2] == [0, 2]
    assert r["rollback"][0] == 1
    r = run([5, 11, 0, 0, 0, 2])                          # the other branch: 0 -> 1 -> 5 (token 11 under node 1, not node 4)
    assert r["path"][0].tolist()[:3] == [0, 1, 5] and r["out_tokens"][0].tolist()[:3] == [5, 11, 2] and r["rollback"][0] == 0
    # two children with the same token: the lower row is taken
    parent2 = np.array([-1, 0, 0], np.int32)
    tokens2 = np.array([0, 4, 4], np.int32)
    logits = np.zeros((3, V), np.float32)
    logits[0, 4] = 1.0
    logits[1, 8] = 1.0
    logits[2, 9] = 1.0
    r = oracle.accept_tree(logits, tokens2, parent2, np.array([0, 3], np.int32), 2)
    assert r["path"][0].tolist() == [0, 1, -1] and r["out_tokens"][0].tolist() == [4, 8, -1]
    # a malformed tree (parent not before its child) is refused for that request only
    bad = oracle.accept_tree(logits, tokens2, np.array([-1, 2, 0], np.int32), np.array([0, 3], np.int32), 2)
    assert bad["accept_len"][0] == 0 and bad["out_tokens"][0].tolist() == [-1, -1, -1] and bad["status"] & 2


def test_tree_commit_gathers_the_accepted_path(oracle):
    rng = np.random.default_rng(2)
    cs, gammas, Hq, Hkv = [37, 5, 64, 14, 0], [6, 0, 3, 12, 4], 4, 2
    q, k, v, pt, sl, qo = _paged(rng, cs, gammas, Hq, Hkv)
    B = len(cs)
    parent = _random_parents(rng, gammas)
    gmax = max(gammas)
    # a valid root path per request
    path = np.full((B, gmax + 1), -1, np.int32)
    acc = np.zeros(B, np.int32)
    for i in range(B):
        pl = parent[qo[i]:qo[i + 1]]
        leaf = int(rng.integers(0, gammas[i] + 1))
        nodes = sorted(_ancestors(pl, leaf))
        path[i, :len(nodes)] = nodes
        acc[i] = len(nodes) - 1
    total = k.shape[0]
    free_list = np.full(total, -1, np.int32)
    fc = np.zeros(1, np.int32)
    k0, v0, pt0 = k.copy(), v.copy(), pt.copy()
    oracle.kv_commit_tree(k, v, pt, sl, qo, acc, path, free_list, fc, P)
    # the page bookkeeping is the chain commit's (pinned by the golden cases)
    pt1, sl1, fl1, fc1 = pt0.copy(), np.asarray(cs, np.int32).copy(), np.full(total, -1, np.int32), np.zeros(1, np.int32)
    oracle.kv_commit(pt1, sl1, qo, acc, fl1, fc1, P)
    assert np.array_equal(pt, pt1) and np.array_equal(sl, sl1) and np.array_equal(free_list, fl1) and fc[0] == fc1[0]
    for i in range(B):
        for h in range(Hkv):
            before_k, after_k = _gather(k0, pt0, i, cs[i] + gammas[i] + 1, h), _gather(k, pt0, i, cs[i] + gammas[i] + 1, h)
            before_v, after_v = _gather(v0, pt0, i, cs[i] + gammas[i] + 1, h), _gather(v, pt0, i, cs[i] + gammas[i] + 1, h)
            assert np.array_equal(after_k[:cs[i] + 1], before_k[:cs[i] + 1])             # prefix and root untouched
            for kk in range(1, acc[i] + 1):
                assert np.array_equal(after_k[cs[i] + kk], before_k[cs[i] + path[i, kk]])
                assert np.array_equal(after_v[cs[i] + kk], before_v[cs[i] + path[i, kk]])
