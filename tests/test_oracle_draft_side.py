"""Pins for the draft-side primitives of the oracle: divergence point, KV rollback, prompt compression
(Appendix "Draft side"; Method, "Draft-side context compression", eq. token_eviction)."""
import numpy as np

from test_oracle_commit import P, _state


def _ragged(rows):
    ip = np.zeros(len(rows) + 1, np.int32)
    ip[1:] = np.cumsum([len(r) for r in rows])
    flat = np.array([t for r in rows for t in r] or [0], np.int32)
    return flat, ip


def test_divergence_hand_cases_and_brute_force(oracle):
    p_rows = [[1, 2, 3, 4], [1, 2, 3], [9], [], [5, 6, 7, 8, 9], [4, 4, 4]]
    h_rows = [[1, 2, 7, 4], [1, 2, 3, 4, 5], [8, 9], [1], [5, 6, 7, 8, 9], [4, 4]]
    pt, pi = _ragged(p_rows)
    ht, hi = _ragged(h_rows)
    # differ at 2; p is a prefix of h (keep all 3); differ at 0; empty prefix; identical; h is a prefix of p
    assert oracle.divergence(pt, pi, ht, hi).tolist() == [2, 3, 0, 0, 5, 2]
    rng = np.random.default_rng(0)
    p_rows, h_rows = [], []
    for _ in range(300):
        n = int(rng.integers(0, 400))
        base = rng.integers(0, 3, n).tolist()
        other = list(base)
        if n and rng.random() < 0.7:
            t = int(rng.integers(0, n))
            other[t] += 1
        cut = int(rng.integers(0, n + 1))
        p_rows.append(base)
        h_rows.append(other[:cut] if rng.random() < 0.3 else other)
    pt, pi = _ragged(p_rows)
    ht, hi = _ragged(h_rows)
    want = []
    for a, b in zip(p_rows, h_rows):
        m = min(len(a), len(b))
        neq = np.flatnonzero(np.asarray(a[:m]) != np.asarray(b[:m]))
        want.append(int(neq[0]) if len(neq) else m)
    assert oracle.divergence(pt, pi, ht, hi).tolist() == want


def test_truncate_hand_cases(oracle):
    # 40 tokens = 3 pages; keep 17 -> 2 pages kept, logical page 2 freed; keep 16 -> 1 page kept, pages 1 and 2 freed;
    # keep >= length: nothing happens; keep 0: everything goes; negative keep counts as 0
    rng = np.random.default_rng(1)
    cs = [40, 40, 40, 40, 33]
    pt, sl, qo, fl, fc, total = _state(cs, [0] * 5, rng)
    sl[:] = cs                                            # the lengths themselves (the helper adds a candidate row)
    before = pt.copy()
    keep = np.array([17, 16, 99, 0, -4], np.int32)
    fc0 = int(fc[0])
    oracle.kv_truncate(pt, sl, keep, fl, fc, P)
    assert sl.tolist() == [17, 16, 40, 0, 0]
    freed = [before[0, 2], before[1, 1], before[1, 2], before[3, 0], before[3, 1], before[3, 2], before[4, 0], before[4, 1], before[4, 2]]
    assert fl[fc0:int(fc[0])].tolist() == freed
    assert (pt[0, :2] == before[0, :2]).all() and pt[0, 2] == -1 and (pt[2] == before[2]).all() and (pt[3] == -1).all()


def test_truncate_agrees_with_commit(oracle):
    """Commit(p, y, L) is "write the candidate, then roll back to c + a + 1": the two oracle routines must leave the
    same page table, lengths and free list (the commit routine is pinned by the hand-worked golden cases)."""
    rng = np.random.default_rng(2)
    for trial in range(20):
        B = int(rng.integers(1, 60))
        cs = rng.integers(0, 300, B)
        gs = rng.choice([0, 2, 4, 8, 40], B)
        acc = np.array([rng.integers(0, g + 1) for g in gs], np.int32)
        pt, sl, qo, fl, fc, total = _state(cs, gs, rng)
        pt2, sl2, fl2, fc2 = pt.copy(), (sl + gs + 1).astype(np.int32), fl.copy(), fc.copy()
        oracle.kv_commit(pt, sl, qo, acc, fl, fc, P)
        oracle.kv_truncate(pt2, sl2, (np.asarray(cs) + acc + 1).astype(np.int32), fl2, fc2, P)
        assert np.array_equal(pt, pt2) and np.array_equal(sl, sl2) and int(fc[0]) == int(fc2[0])
        assert np.array_equal(fl[:int(fc[0])], fl2[:int(fc[0])])
        used = pt[pt >= 0]
        assert len(set(used.tolist()) | set(fl[:int(fc[0])].tolist())) == total      # pages conserved


def test_compression_hand_cases(oracle):
    x = np.arange(1, 21, dtype=np.int32)                 # a prompt x_1 .. x_20
    out, ip, idx = oracle.compress_prompts(x, np.array([0, 20], np.int32), 1, 2)      # p = 0.5: k = 5
    assert out.tolist() == [1, 2, 3, 4, 5, 16, 17, 18, 19, 20] and ip.tolist() == [0, 10]
    assert idx.tolist() == [0, 1, 2, 3, 4, 15, 16, 17, 18, 19]
    out, ip, _ = oracle.compress_prompts(x[:7].copy(), np.array([0, 7], np.int32), 3, 5)   # S = 7, p = 0.6: k = 2
    assert out.tolist() == [1, 2, 6, 7]
    out, ip, _ = oracle.compress_prompts(x[:10].copy(), np.array([0, 10], np.int32), 1, 10)  # p = 0.1 of 10 tokens: k = 0
    assert out.tolist() == [] and ip.tolist() == [0, 0]
    out, ip, _ = oracle.compress_prompts(x, np.array([0, 20], np.int32), 1, 1)             # p = 1: everything, once
    assert out.tolist() == x.tolist()
    # the paper's setting: p = 0.1 on a 4000-token prompt keeps 200 + 200 tokens
    big = np.arange(4000, dtype=np.int32)
    out, ip, idx = oracle.compress_prompts(big, np.array([0, 4000], np.int32), 1, 10)
    assert len(out) == 400 and out[:200].tolist() == list(range(200)) and out[200:].tolist() == list(range(3800, 4000))


def test_compression_matches_slicing_on_ragged_batches(oracle):
    rng = np.random.default_rng(4)
    for (pn, pd) in [(1, 10), (1, 4), (2, 3), (0, 1), (7, 5)]:
        rows = [rng.integers(0, 1000, int(rng.integers(0, 900))).tolist() for _ in range(70)]
        flat, ip = _ragged(rows)
        out, oip, idx = oracle.compress_prompts(flat, ip, pn, pd)
        want, widx = [], []
        for r in rows:
            S = len(r)
            k = pn * S // (2 * pd)
            assert 2 * k * pd <= pn * S                                       # at most p S tokens kept
            kept = list(range(S)) if 2 * k >= S else list(range(k)) + list(range(S - k, S))
            want.append([r[t] for t in kept])
            widx += kept
        assert out.tolist() == [t for w in want for t in w]
        assert oip.tolist() == np.concatenate([[0], np.cumsum([len(w) for w in want])]).tolist()
        assert idx.tolist() == widx
