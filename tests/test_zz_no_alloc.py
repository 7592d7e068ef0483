"""spec_accept_static (the entry point that allocates nothing: its scratch is an array inside the library image)
against spec_accept on the same inputs, through the C ABI: two calls in a row, the second on a smaller batch, so
that whatever the first call left in the shared array cannot leak into the second.  Integers, bit-exact."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2605_08151_amd import workloads as wl  # noqa: E402


def _qo(gammas):
    qo = np.zeros(len(gammas) + 1, np.int32)
    qo[1:] = np.cumsum(np.asarray(gammas) + 1)
    return qo


def _inputs(seed, B, V):
    rng = np.random.default_rng(seed)
    gammas = rng.choice([0, 2, 4, 8], B)
    qo = _qo(gammas)
    logits = rng.normal(0, 1.0, (qo[-1], V)).astype(np.float32)
    cfg = wl.VerifyConfig("na", seed, B, (4,), ("const", 1), 8, 1, 64, V)
    dp, tokens = wl.draft_probs_noisy(cfg, torch.from_numpy(qo), torch.from_numpy(logits), noise_std=1.0)
    tg, _ = wl.draft_tokens_greedy(cfg, torch.from_numpy(qo), torch.from_numpy(logits.argmax(1)))
    temp = np.where(np.arange(B) % 3 == 0, 0.0, 0.8).astype(np.float32)        # greedy and sampled requests mixed
    per_row_T = np.repeat(temp, np.diff(qo))
    tokens = np.where(per_row_T > 0, tokens.numpy(), tg.numpy()).astype(np.int32)
    seeds = rng.integers(0, 2 ** 63, B, dtype=np.uint64)
    return gammas, qo, logits, tokens, dp.numpy(), temp, seeds


def _run(sv, fn_static, qo, logits, tokens, dp, temp, seeds, round_, gamma_max):
    B, (M, V) = len(qo) - 1, logits.shape
    dev = lambda a: torch.from_numpy(a).cuda()
    al = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    ot = torch.full((B, gamma_max + 1), -9, dtype=torch.int32, device="cuda")
    rb = torch.full((B,), 9, dtype=torch.uint8, device="cuda")
    stats = torch.full((4,), -9, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    args = (dev(logits), dev(tokens), dev(dp), dev(temp), dev(seeds.view(np.int64)), round_, dev(qo), al, ot, rb, stats,
            gamma_max, status)
    if fn_static:
        sv.spec_accept_static(*args)
    else:
        ws = torch.empty(max(256, sv.spec_accept_workspace_bytes(B, M, V, gamma_max)), dtype=torch.uint8, device="cuda")
        sv.spec_accept(*args, ws)
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in (al, ot, rb, stats, status)]


def test_accept_without_allocation_matches_spec_accept_twice_in_a_row():
    import paper_2605_08151_amd.binding as sv
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    for seed, B, V in ((71, 48, 20011), (72, 9, 5000)):             # the second call is the smaller one
        gammas, qo, logits, tokens, dp, temp, seeds = _inputs(seed, B, V)
        got = _run(sv, True, qo, logits, tokens, dp, temp, seeds, 6, 8)
        want = _run(sv, False, qo, logits, tokens, dp, temp, seeds, 6, 8)
        for g, w in zip(got, want):
            assert np.array_equal(g, w)
        assert got[4][0] == 0 and (got[1][np.arange(B), got[0]] >= 0).all()
        assert 0 < got[0].sum() < gammas.sum()                      # accepts and rejections both occur


def test_accept_without_allocation_rejects_what_does_not_fit():
    import paper_2605_08151_amd.binding as sv
    B, M, V = 4, 8000, 151936                                       # 8000 rows x 38 segments: beyond the 4 MiB array
    assert sv.spec_accept_workspace_bytes(B, M, V, 8) > (4 << 20)
    z = lambda n, dt: torch.zeros(n, dtype=dt, device="cuda")
    logits = torch.zeros((8, 16), dtype=torch.float32, device="cuda")
    with pytest.raises(sv.SpecError) as e:
        # the sizes alone decide: the pointers are never dereferenced
        sv._check(sv._lib.spec_accept_static(sv._ptr(logits), sv._ptr(z(8, torch.int32)), None, sv._ptr(z(4, torch.float32)), None, 0,
                                             sv._ptr(z(5, torch.int32)), sv._ptr(z(4, torch.int32)), sv._ptr(z(36, torch.int32)), None, None,
                                             B, M, V, 8, None, None))
    assert e.value.code == -3 and "4194304" in str(e.value)
