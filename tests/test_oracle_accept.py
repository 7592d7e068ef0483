"""Pins for oracle_accept.

Greedy: longest prefix match against the library argmax.  Stochastic: the lossless property of
rejection sampling (the emitted token is distributed as the target p whatever the drafter q), checked by
brute force over ~10^6 Philox seeds on tiny vocabularies, plus the closed-form accept probability
min(1, p/q), the q == p and one-hot-q special cases, and the gamma = 0 reduction to plain sampling."""
import numpy as np
import torch


def _qo(gammas):
    qo = np.zeros(len(gammas) + 1, np.int32)
    qo[1:] = np.cumsum(np.asarray(gammas) + 1)
    return qo


def _softmax64(x, T=1.0):
    return torch.softmax(torch.from_numpy(np.asarray(x, np.float64)) / T, -1).numpy()


def _chi2(counts, probs):
    n = counts.sum()
    e = probs * n
    return float(((counts - e) ** 2 / e).sum())


# ---------------------------------------------------------------- greedy
def test_greedy_is_longest_prefix_match(oracle):
    rng = np.random.default_rng(0)
    V, gammas = 97, [4, 0, 8, 2, 4, 4, 8, 1]
    qo = _qo(gammas)
    logits = rng.normal(0, 1, (qo[-1], V)).astype(np.float32)
    am = logits.argmax(1)
    tokens = rng.integers(0, V, qo[-1]).astype(np.int32)
    planned = [2, 0, 8, 0, 4, 1, 3, 1]
    for i, g in enumerate(gammas):
        for j in range(1, g + 1):
            if j <= planned[i]:
                tokens[qo[i] + j] = am[qo[i] + j - 1]
            elif j == planned[i] + 1:
                tokens[qo[i] + j] = (am[qo[i] + j - 1] + 1 + rng.integers(0, V - 1)) % V     # any wrong token
            else:
                tokens[qo[i] + j] = am[qo[i] + j - 1]      # correct tokens AFTER a mismatch must not count
    res = oracle.accept(logits, tokens, None, np.zeros(len(gammas), np.float32), None, 0, qo, 8)
    assert list(res["accept_len"]) == planned
    for i, g in enumerate(gammas):
        a = planned[i]
        row = res["out_tokens"][i]
        assert list(row[:a]) == list(tokens[qo[i] + 1:qo[i] + 1 + a])
        assert row[a] == am[qo[i] + a]                       # bonus = target's own token at the first mismatch
        assert (row[a + 1:] == -1).all()
        assert res["rollback"][i] == (a < g)
    assert res["status"] == 0


def test_greedy_full_accept_when_drafts_are_the_greedy_continuation(oracle):
    rng = np.random.default_rng(1)
    V, gammas = 50, [4] * 6
    qo = _qo(gammas)
    logits = rng.normal(0, 1, (qo[-1], V)).astype(np.float32)
    tokens = np.zeros(qo[-1], np.int32)
    tokens[1:] = logits.argmax(1)[:-1]
    res = oracle.accept(logits, tokens, None, np.zeros(6, np.float32), None, 0, qo, 4)
    assert (res["accept_len"] == 4).all() and (res["rollback"] == 0).all()


def test_greedy_ties_take_lowest_index(oracle):
    logits = np.zeros((2, 9), np.float32)
    logits[0, [3, 7]] = 2.0
    logits[1, [5, 6]] = 1.0
    qo = _qo([1])
    for tok, a, bonus in [(3, 1, 5), (7, 0, 3)]:
        res = oracle.accept(logits, np.array([0, tok], np.int32), None, np.zeros(1, np.float32), None, 0, qo, 1)
        assert res["accept_len"][0] == a and res["out_tokens"][0, a] == bonus


def test_nonfinite_rows_are_flagged(oracle):
    logits = np.zeros((3, 5), np.float32)
    logits[1, 2] = np.nan
    qo = _qo([2])
    res = oracle.accept(logits, np.array([0, 0, 0], np.int32), None, np.zeros(1, np.float32), None, 0, qo, 2)
    assert res["status"] & 1 and res["accept_len"][0] == 0 and res["out_tokens"][0, 0] == -1
    assert res["rollback"][0] == 1
    logits[1, 2] = -np.inf                                    # a masked vocabulary entry is fine
    res = oracle.accept(logits, np.array([0, 0, 0], np.int32), None, np.zeros(1, np.float32), None, 0, qo, 2)
    assert res["status"] == 0 and res["accept_len"][0] == 2


# ---------------------------------------------------------------- stochastic
def test_target_probs_is_library_softmax(oracle):
    rng = np.random.default_rng(2)
    l = rng.normal(0, 3, 1000).astype(np.float32)
    for T in (0.7, 1.0, 2.5):
        p = oracle.target_probs(l, T)
        np.testing.assert_allclose(p, _softmax64(l, np.float64(np.float32(T))), rtol=2e-7)


def _run_many(oracle, logits_rows, q_rows, gamma, T, n, rng, seed0=0, one_hot=False):
    """n independent requests sharing the same gamma+1 logits rows; drafts d_j ~ q_j drawn by numpy."""
    V = logits_rows.shape[1]
    qo = _qo([gamma] * n)
    logits = np.tile(logits_rows, (n, 1)).astype(np.float32)
    tokens = np.zeros(qo[-1], np.int32).reshape(n, gamma + 1)
    for j in range(1, gamma + 1):
        tokens[:, j] = rng.choice(V, size=n, p=q_rows[j - 1].astype(np.float64) / q_rows[j - 1].astype(np.float64).sum())
    dp = None if one_hot else np.tile(q_rows.astype(np.float32), (n, 1))
    seeds = (np.arange(n, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15) + np.uint64(seed0))
    res = oracle.accept(logits, tokens.reshape(-1), dp, np.full(n, T, np.float32), seeds, 3, qo, gamma)
    return res, tokens


def test_emitted_tokens_follow_target_distribution_bruteforce(oracle):
    rng = np.random.default_rng(3)
    V, gamma, T, n = 5, 2, 0.8, 1_000_000
    logits_rows = rng.normal(0, 1.5, (gamma + 1, V))
    q_rows = np.stack([_softmax64(rng.normal(0, 1.5, V)) for _ in range(gamma)])
    p = np.stack([_softmax64(np.float32(logits_rows[j]).astype(np.float64), np.float64(np.float32(T))) for j in range(gamma + 1)])
    res, tokens = _run_many(oracle, logits_rows, q_rows, gamma, T, n, rng)
    out, a = res["out_tokens"], res["accept_len"]
    # first emitted token ~ p_0 regardless of q_1
    c0 = np.bincount(out[:, 0], minlength=V)
    assert _chi2(c0, p[0]) < 40.0                              # 4 dof: P(chi2 > 40) ~ 4e-8
    # given the first draft was accepted, the second emitted token ~ p_1; given two accepted, third ~ p_2
    c1 = np.bincount(out[a >= 1, 1], minlength=V)
    assert _chi2(c1, p[1]) < 40.0
    c2 = np.bincount(out[a >= 2, 2], minlength=V)
    assert _chi2(c2, p[2]) < 40.0
    # accept probability of draft 1 is sum_d q(d) min(1, p(d)/q(d)) = sum_d min(p, q)
    want = np.minimum(p[0], q_rows[0]).sum()
    got = (a >= 1).mean()
    assert abs(got - want) < 5 * np.sqrt(want * (1 - want) / n)
    # per-token accept rate is min(1, p(d)/q(d))
    for d in range(V):
        sel = tokens[:, 1] == d
        rate = (a[sel] >= 1).mean()
        w = min(1.0, p[0, d] / q_rows[0, d])
        assert abs(rate - w) < 5 * np.sqrt(max(w * (1 - w), 1e-4) / sel.sum())
    # a rejected draft is replaced by a draw from norm(max(0, p - q))
    rej = a == 0
    resid = np.maximum(p[0] - q_rows[0], 0)
    resid /= resid.sum()
    cr = np.bincount(out[rej, 0], minlength=V)
    keep = resid > 0
    assert cr[~keep].sum() == 0
    assert _chi2(cr[keep], resid[keep]) < 40.0


def test_draft_equal_to_target_accepts_everything(oracle):
    rng = np.random.default_rng(4)
    V, gamma, T, n = 6, 2, 0.7, 50_000
    logits_rows = rng.normal(0, 2, (gamma + 1, V)).astype(np.float32)
    q_rows = np.stack([oracle.target_probs(logits_rows[j], T) for j in range(gamma)])
    res, _ = _run_many(oracle, logits_rows, q_rows, gamma, T, n, rng)
    assert (res["accept_len"] == gamma).all() and (res["rollback"] == 0).all()
    p_last = oracle.target_probs(logits_rows[gamma], T).astype(np.float64)
    assert _chi2(np.bincount(res["out_tokens"][:, gamma], minlength=V), p_last / p_last.sum()) < 45.0


def test_one_hot_drafter(oracle):
    """draft_probs == NULL: accept w.p. p(d); on rejection the bonus is never d and follows p with d removed."""
    rng = np.random.default_rng(5)
    V, T, n = 4, 1.0, 400_000
    logits_rows = rng.normal(0, 1, (2, V)).astype(np.float32)
    p0 = oracle.target_probs(logits_rows[0], T).astype(np.float64)
    q_rows = np.full((1, V), 1.0 / V)
    res, tokens = _run_many(oracle, logits_rows, q_rows, 1, T, n, rng, one_hot=True)
    a, out = res["accept_len"], res["out_tokens"]
    for d in range(V):
        sel = tokens[:, 1] == d
        assert abs((a[sel] == 1).mean() - p0[d]) < 5 * np.sqrt(p0[d] * (1 - p0[d]) / sel.sum())
        rej = sel & (a == 0)
        assert (out[rej, 0] != d).all()
        rest = p0.copy()
        rest[d] = 0
        cnt = np.bincount(out[rej, 0], minlength=V)
        k = rest > 0
        assert _chi2(cnt[k], rest[k] / rest.sum()) < 40.0


def test_gamma_zero_is_plain_sampling(oracle):
    rng = np.random.default_rng(6)
    V, n = 7, 300_000
    row = rng.normal(0, 1, (1, V)).astype(np.float32)
    res, _ = _run_many(oracle, row, np.zeros((0, V)), 0, 1.3, n, rng)
    assert (res["accept_len"] == 0).all() and (res["rollback"] == 0).all()
    p = oracle.target_probs(row[0], 1.3).astype(np.float64)
    assert _chi2(np.bincount(res["out_tokens"][:, 0], minlength=V), p / p.sum()) < 45.0
    # greedy gamma = 0 emits the argmax
    res = oracle.accept(row, np.zeros(1, np.int32), None, np.zeros(1, np.float32), None, 0, _qo([0]), 0)
    assert res["out_tokens"][0, 0] == row[0].argmax() and res["accept_len"][0] == 0


def test_bonus_is_the_inverse_cdf_bucket_of_its_uniform(oracle):
    """gamma = 0 at T = 1 with p = (.5, .25, .25) exactly: the bonus is the bucket of u' = U(seed, round, 1, 1)."""
    row = np.log(np.array([[2.0, 1.0, 1.0]])).astype(np.float32)
    hits = set()
    for seed in range(2000):
        u = oracle.uniform(seed, 9, 1, 1)
        res = oracle.accept(row, np.zeros(1, np.int32), None, np.ones(1, np.float32),
                            np.array([seed], np.uint64), 9, _qo([0]), 0)
        want = 0 if u < 0.5 - 1e-6 else 1 if 0.5 + 1e-6 < u < 0.75 - 1e-6 else 2 if u > 0.75 + 1e-6 else None
        if want is not None:
            assert res["out_tokens"][0, 0] == want
            hits.add(want)
    assert hits == {0, 1, 2}


def test_accept_test_uses_uniform_j_tag0(oracle):
    """One draft, q(d) = 1, p(d) = 1/2 exactly (two equal logits): accepted iff U(seed, round, 1, 0) < 1/2."""
    logits = np.zeros((2, 2), np.float32)
    n_acc = 0
    for seed in range(500):
        u = oracle.uniform(seed, 4, 1, 0)
        res = oracle.accept(logits, np.array([0, 1], np.int32), None, np.ones(1, np.float32),
                            np.array([seed], np.uint64), 4, _qo([1]), 1)
        assert res["accept_len"][0] == int(u < 0.5)
        n_acc += int(u < 0.5)
        if u >= 0.5:
            assert res["out_tokens"][0, 0] == 0               # residual removes the rejected token
    assert 150 < n_acc < 350


def _bucket(u, edges):
    """Index of the inverse-CDF bucket of u, or None when u is within 1e-6 of an edge."""
    for k, e in enumerate(edges):
        if abs(u - e) < 1e-6:
            return None
        if u < e:
            return k
    return len(edges)


def test_zero_residual_falls_back_to_the_target_distribution(oracle):
    """p = (1/2, 1/4, 1/4, 0) exactly, the draft is the masked entry 3 and q = p there and elsewhere: the accept
    test 0 < 0 fails, max(0, p - q) is zero everywhere, so the bonus is the inverse-CDF bucket of
    U(seed, round, 1, 1) in p itself: never the rejected token, never -1."""
    row = np.log(np.array([2.0, 1.0, 1.0, 1.0])).astype(np.float32)
    row[3] = -np.inf
    logits = np.stack([row, np.zeros(4, np.float32)])
    q = oracle.target_probs(row, 1.0)[None, :].copy()
    assert list(q[0]) == [0.5, 0.25, 0.25, 0.0]
    hits = set()
    for seed in range(1500):
        res = oracle.accept(logits, np.array([0, 3], np.int32), q, np.ones(1, np.float32),
                            np.array([seed], np.uint64), 7, _qo([1]), 1)
        assert res["accept_len"][0] == 0 and res["rollback"][0] == 1 and res["status"] == 0
        want = _bucket(oracle.uniform(seed, 7, 1, 1), [0.5, 0.75])
        if want is not None:
            assert res["out_tokens"][0, 0] == want
            hits.add(want)
        assert list(res["out_tokens"][0, 1:]) == [-1]
    assert hits == {0, 1, 2}


def test_drafter_above_target_everywhere_rejects_into_the_target_distribution(oracle):
    """q = 2p (a drafter whose stated probabilities exceed the target's at every token): draft d is accepted
    iff U(seed, round, 1, 0) < 1/2; a rejection leaves no positive residual, and the bonus is then the bucket
    of U(seed, round, 1, 1) in p = (1/2, 1/4, 1/4)."""
    row = np.log(np.array([2.0, 1.0, 1.0])).astype(np.float32)
    logits = np.stack([row, row])
    q = (2.0 * oracle.target_probs(row, 1.0))[None, :].astype(np.float32)
    n_rej = 0
    for seed in range(1200):
        d = seed % 3
        res = oracle.accept(logits, np.array([0, d], np.int32), q, np.ones(1, np.float32),
                            np.array([seed], np.uint64), 2, _qo([1]), 1)
        u = oracle.uniform(seed, 2, 1, 0)
        if abs(u - 0.5) < 1e-6:
            continue
        assert res["accept_len"][0] == int(u < 0.5)
        if u >= 0.5:
            n_rej += 1
            want = _bucket(oracle.uniform(seed, 2, 1, 1), [0.5, 0.75])
            if want is not None:
                assert res["out_tokens"][0, 0] == want
    assert 400 < n_rej < 800
