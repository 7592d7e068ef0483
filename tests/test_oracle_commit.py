"""Pins for oracle_kv_commit: hand-worked page arithmetic and conservation invariants."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "kv_commit_cases.txt")
P = 16


def _state(cs, gammas, rng, slack=3):
    B = len(cs)
    n = np.asarray(gammas) + 1
    pages = (np.asarray(cs) + n + P - 1) // P
    total = int(pages.sum()) + slack
    perm = rng.permutation(total).astype(np.int32)
    max_pages = int(pages.max()) + 2
    pt = np.full((B, max_pages), -1, np.int32)
    off = 0
    for i in range(B):
        pt[i, :pages[i]] = perm[off:off + pages[i]]
        off += pages[i]
    free_list = np.full(total, -1, np.int32)
    free_list[:total - off] = perm[off:]
    free_count = np.array([total - off], np.int32)
    qo = np.zeros(B + 1, np.int32)
    qo[1:] = np.cumsum(n)
    return pt, np.asarray(cs, np.int32).copy(), qo, free_list, free_count, total


def test_hand_worked_cases(oracle):
    rows = [list(map(int, l.split())) for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    rng = np.random.default_rng(0)
    cs, gs, acc = [r[0] for r in rows], [r[1] for r in rows], [r[2] for r in rows]
    pt, sl, qo, fl, fc, total = _state(cs, gs, rng)
    before = pt.copy()
    fc0 = int(fc[0])
    oracle.kv_commit(pt, sl, qo, np.asarray(acc, np.int32), fl, fc, P)
    expect_free = []
    for i, r in enumerate(rows):
        _, _, _, new_len, pages_before, kept, freed = r
        assert sl[i] == new_len
        assert (before[i] >= 0).sum() == pages_before
        assert (pt[i] >= 0).sum() == kept
        assert np.array_equal(pt[i, :kept], before[i, :kept])        # kept pages untouched, in place
        assert pages_before - kept == freed
        expect_free += list(before[i, kept:pages_before])            # request order, then logical order
    assert int(fc[0]) == fc0 + len(expect_free)
    assert list(fl[fc0:int(fc[0])]) == expect_free


def test_conservation_random(oracle):
    rng = np.random.default_rng(1)
    for trial in range(20):
        B = int(rng.integers(1, 40))
        cs = rng.integers(0, 300, B)
        gs = rng.choice([0, 2, 4, 8], B)
        acc = np.array([rng.integers(0, g + 1) for g in gs], np.int32)
        pt, sl, qo, fl, fc, total = _state(cs, gs, rng)
        oracle.kv_commit(pt, sl, qo, acc, fl, fc, P)
        used = pt[pt >= 0]
        free = fl[:int(fc[0])]
        both = np.concatenate([used, free])
        assert len(both) == total and len(np.unique(both)) == total       # disjoint, nothing lost
        assert np.array_equal(sl, cs + acc + 1)
        assert np.array_equal((pt >= 0).sum(1), (sl + P - 1) // P)


def test_gamma_zero_adds_exactly_one_token(oracle):
    rng = np.random.default_rng(2)
    cs = [5, 15, 16, 31, 32]
    pt, sl, qo, fl, fc, total = _state(cs, [0] * 5, rng)
    before, fc0 = pt.copy(), int(fc[0])
    oracle.kv_commit(pt, sl, qo, np.zeros(5, np.int32), fl, fc, P)
    assert list(sl) == [c + 1 for c in cs]
    assert np.array_equal(pt, before) and int(fc[0]) == fc0             # decode never frees a page
