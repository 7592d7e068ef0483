"""Pins for oracle_assemble_next: candidates of round n+1 worked by hand from the paper's equations
(tests/golden/assemble_next_cases.txt) and invariants on random batches."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "assemble_next_cases.txt")
GAMMA_NEXT = 4


def _ints(field):
    field = field.strip()
    return [] if field == "-" else [int(x) for x in field.split()]


def _cases():
    out = []
    for line in open(GOLDEN):
        if not line.strip() or line.startswith("#"):
            continue
        lhs, rhs = line.split("->")
        mode, gamma, a, b, cont, repair = [f.strip() for f in lhs.split("|")]
        rb, cand = [f.strip() for f in rhs.split("|")]
        out.append(dict(mode=0 if mode == "O" else 1, gamma=int(gamma), a=int(a), b=int(b), cont=_ints(cont),
                        repair=_ints(repair), rollback=int(rb), cand=_ints(cand)))
    return out


def _pack(rows, width):
    arr = np.full((len(rows), max(1, width)), -3, np.int32)
    for i, r in enumerate(rows):
        arr[i, :len(r)] = r
    return arr, np.array([len(r) for r in rows], np.int32)


def _batch(cases, gamma_max=8):
    B = len(cases)
    qo = np.zeros(B + 1, np.int32)
    qo[1:] = np.cumsum([c["gamma"] + 1 for c in cases])
    al = np.array([c["a"] for c in cases], np.int32)
    ot = np.full((B, gamma_max + 1), -1, np.int32)
    for i, c in enumerate(cases):
        ot[i, :c["a"]] = 1000 + np.arange(c["a"])        # the accepted drafts (not used by the assembly)
        ot[i, c["a"]] = c["b"]
    cont, cl = _pack([c["cont"] for c in cases], 8)
    rep, rl = _pack([c["repair"] for c in cases], 8)
    return al, ot, qo, cont, cl, rep, rl


def test_hand_worked_cases(oracle):
    cases = _cases()
    assert len(cases) >= 12
    for mode in (0, 1):
        sub = [c for c in cases if c["mode"] == mode]
        al, ot, qo, cont, cl, rep, rl = _batch(sub)
        r = oracle.assemble_next(al, ot, qo, cont, cl, rep if mode == 0 else None, rl if mode == 0 else None, mode, GAMMA_NEXT)
        for i, c in enumerate(sub):
            got = r["tokens"][r["qo_indptr"][i]:r["qo_indptr"][i + 1]].tolist()
            assert got == c["cand"], (c, got)
            assert int(r["rollback"][i]) == c["rollback"], c
        assert r["stats"].tolist() == [sum(c["rollback"] for c in sub), sum(c["a"] + 1 for c in sub), len(sub), r["rows"]]


def test_invariants_on_random_batches(oracle):
    rng = np.random.default_rng(3)
    for mode in (0, 1):
        for trial in range(20):
            B = int(rng.integers(1, 200))
            gam = rng.choice([0, 2, 4, 8], B)
            qo = np.zeros(B + 1, np.int32)
            qo[1:] = np.cumsum(gam + 1)
            al = np.array([rng.integers(0, g + 1) for g in gam], np.int32)
            ot = np.full((B, 9), -1, np.int32)
            bonus = rng.integers(0, 50, B).astype(np.int32)
            for i in range(B):
                ot[i, al[i]] = bonus[i]
            cont = rng.integers(0, 50, (B, 10)).astype(np.int32)
            agree = rng.random(B) < 0.6
            cont[agree, 0] = bonus[agree]
            cl = rng.integers(0, 11, B).astype(np.int32)
            rep = rng.integers(100, 150, (B, 6)).astype(np.int32)
            rl = rng.integers(0, 7, B).astype(np.int32)
            gn = int(rng.integers(0, 9))
            r = oracle.assemble_next(al, ot, qo, cont, cl, rep if mode == 0 else None, rl if mode == 0 else None, mode, gn)
            nqo = r["qo_indptr"]
            assert nqo[0] == 0 and (np.diff(nqo) >= 1).all() and (np.diff(nqo) <= gn + 1).all() and nqo[-1] == r["rows"]
            assert (r["tokens"][nqo[:-1]] == bonus).all()                       # row 0 is always the bonus
            stable = (al == gam) & (cl >= 1) & (cont[:, 0] == bonus)
            assert (r["rollback"] == (~stable)).all()                           # rollback set: rejected prefix or invalidated continuation
            for i in range(B):
                rows = r["tokens"][nqo[i] + 1:nqo[i + 1]]
                if stable[i]:
                    assert rows.tolist() == cont[i, 1:1 + min(cl[i] - 1, gn)].tolist()
                elif mode == 1:
                    assert len(rows) == 0                                       # parallel mode: the padded candidate
                else:
                    assert rows.tolist() == rep[i, :min(rl[i], gn)].tolist()
            assert r["stats"].tolist() == [int((~stable).sum()), int((al + 1).sum()), B, r["rows"]]


def test_undecided_request_gets_a_single_invalid_row(oracle):
    al = np.array([0, 2], np.int32)
    ot = np.array([[-1, -1, -1], [7, 8, 9]], np.int32)            # request 0: spec_accept could not decide (bonus -1)
    qo = np.array([0, 3, 6], np.int32)
    cont = np.array([[5, 6], [9, 4]], np.int32)
    r = oracle.assemble_next(al, ot, qo, cont, np.array([2, 2], np.int32), None, None, 1, 4)
    assert r["tokens"].tolist() == [-1, 9, 4] and r["qo_indptr"].tolist() == [0, 1, 3]
    assert r["rollback"].tolist() == [1, 0] and r["stats"].tolist() == [1, 3, 2, 3]
