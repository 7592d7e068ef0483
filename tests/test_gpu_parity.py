"""GPU parity: every library call against the CPU oracle on the same seeded inputs, through the C ABI.

Tolerances (written here; derived from bf16 inputs, fp32 accumulation and bf16 outputs): attention and logits |err| <= 1e-2 + 2e-2*|ref| (bf16 inputs,
fp32 accumulation) and, because N(0, 0.02) data would make that check vacuous, also
|err| <= 1e-2 * (|ref| + rms of the element's own output vector) on unit-variance ("sharp") data, 2e-2 otherwise.  Acceptance and commit outputs are integers and must be bit-exact.
"""
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2605_08151_amd import workloads as wl  # noqa: E402


@pytest.fixture(scope="module")
def sv():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2605_08151_amd.binding as b
    return b


def _step(b, cfg):
    from paper_2605_08151_amd.step import VerifyStep
    return VerifyStep(b["B"], b["M"], cfg.Hq, cfg.Hkv, cfg.D, cfg.H, cfg.V, b["gamma_max"], b["max_kv_len"])


def _close(got, ref, what, sharp=False):
    """The contract's bound, plus a scale-aware one: every element within 1e-2 (sharp data) of
    |ref| + rms of its own output vector (last axis), so a wrong mask or a dropped page cannot hide
    behind an absolute tolerance that is larger than the data."""
    got, ref = got.astype(np.float64), ref.astype(np.float64)
    err = np.abs(got - ref)
    assert (err <= 1e-2 + 2e-2 * np.abs(ref)).all(), f"{what}: max err {err.max():.3e}"
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    rel = err / (np.abs(ref) + rms + 1e-30)
    assert rel.max() <= (1e-2 if sharp else 2e-2), f"{what}: max scaled err {rel.max():.3e}"


def _oracle_attn(oracle, b, want_lse=False):
    return oracle.verify_attn(wl.bf16_bits(b["q"]), wl.bf16_bits(b["k_cache"]), wl.bf16_bits(b["v_cache"]),
                              b["page_table"].cpu().numpy(), b["seq_lens"].cpu().numpy(),
                              b["qo_indptr"].cpu().numpy(), b["scale"], want_lse=want_lse)


# --------------------------------------------------------------------------- attention
ATTN_CASES = [
    # name, B, gammas, ctx, Hq, Hkv, sigma_qkv
    ("tiny_cfg", 4, (4,), ("uniform", 128, 512), 8, 1, None),
    ("sharp_g8", 5, (0, 2, 4, 8), ("uniform", 1, 700), 8, 1, 1.0),
    ("sharp_g4", 6, (4,), ("uniform", 100, 1500), 32, 8, 1.0),
    ("sharp_mha", 3, (0, 1, 3), ("uniform", 1, 300), 4, 4, 1.0),
    ("decode_only", 7, (0,), ("uniform", 1, 400), 8, 2, 1.0),
    ("short_ctx", 8, (0, 4, 8), ("uniform", 0, 20), 8, 1, 1.0),
    ("max_rows", 2, (15,), ("uniform", 200, 600), 8, 1, 1.0),       # 8 * 16 = 128 rows per kv head
    ("g16", 2, (3, 7), ("uniform", 50, 900), 16, 1, 1.0),
]


@pytest.mark.parametrize("case", ATTN_CASES, ids=[c[0] for c in ATTN_CASES])
def test_attention_matches_oracle(sv, oracle, case):
    name, B, gammas, ctx, Hq, Hkv, sq = case
    cfg = wl.VerifyConfig(name, 11, B, gammas, ctx, Hq, Hkv, 64, 64, sigma_qkv=sq)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    step = _step(b, cfg)
    step.attn_out.fill_(7.0)
    out = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"])
    torch.cuda.synchronize()
    ref, ref_lse = _oracle_attn(oracle, b, want_lse=True)
    _close(out.float().cpu().numpy(), ref, name, sharp=sq is not None)
    np.testing.assert_allclose(step.lse.cpu().numpy(), ref_lse, rtol=2e-3, atol=2e-3)
    assert int(step.status.cpu()) == 0


@pytest.mark.parametrize("chunk", [128, 256, 1024, 100000])
def test_attention_is_split_invariant(sv, oracle, chunk):
    cfg = wl.VerifyConfig("split", 12, 4, (0, 4, 8), ("uniform", 900, 2500), 8, 1, 64, 64, sigma_qkv=1.0)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    sv.spec_set_tuning("attn_chunk", chunk)
    try:
        step = _step(b, cfg)
        out = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"])
        torch.cuda.synchronize()
    finally:
        sv.spec_set_tuning("attn_chunk", 0)
    _close(out.float().cpu().numpy(), _oracle_attn(oracle, b), f"chunk {chunk}", sharp=True)


@pytest.mark.parametrize("tuning", [{"attn_rows": 1}, {"attn_rows": 2}, {"attn_rows_ring": 4}, {"attn_rows": 2, "attn_rows_ring": 4}],
                         ids=["wave_per_key_block", "row_split_from_2_tiles", "ring_of_4", "both"])
@pytest.mark.parametrize("case", [c for c in ATTN_CASES if c[0] in ("sharp_g8", "sharp_g4", "max_rows", "g16", "short_ctx")],
                         ids=lambda c: c[0])
def test_attention_kernel_variants_match_oracle(sv, oracle, case, tuning):
    """The two decompositions of the attention kernel (one wave per key block and all rows; one wave per row tile and shared
    K/V stages) and the ring depths of the latter, each forced where it is not the default, split into several chunks."""
    name, B, gammas, ctx, Hq, Hkv, sq = case
    cfg = wl.VerifyConfig(name, 21, B, gammas, ctx, Hq, Hkv, 64, 64, sigma_qkv=sq)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    keys = dict(tuning, attn_chunk=256)
    for k, v in keys.items():
        sv.spec_set_tuning(k, v)
    try:
        step = _step(b, cfg)
        out = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"])
        torch.cuda.synchronize()
    finally:
        for k in keys:
            sv.spec_set_tuning(k, 0)
    ref, ref_lse = _oracle_attn(oracle, b, want_lse=True)
    _close(out.float().cpu().numpy(), ref, f"{name} {tuning}", sharp=True)
    np.testing.assert_allclose(step.lse.cpu().numpy(), ref_lse, rtol=2e-3, atol=2e-3)
    assert int(step.status.cpu()) == 0


PLAN_CASES = ATTN_CASES + [
    ("plan_split", 4, (0, 4, 8), ("uniform", 900, 2500), 8, 1, 1.0),
    ("plan_long_few", 2, (4,), ("uniform", 5000, 9000), 8, 1, 1.0),
    ("plan_gqa", 3, (2, 4), ("uniform", 600, 3000), 16, 4, 1.0),
]


@pytest.mark.parametrize("waves", [0, 3])
@pytest.mark.parametrize("case", PLAN_CASES, ids=[c[0] for c in PLAN_CASES])
def test_attention_with_balanced_work_list(sv, oracle, case, waves):
    """The device-built work list (chunks sized from the real lengths, longest first) gives the same attention."""
    name, B, gammas, ctx, Hq, Hkv, sq = case
    cfg = wl.VerifyConfig(name, 21, B, gammas, ctx, Hq, Hkv, 64, 64, sigma_qkv=sq)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    sv.spec_set_tuning("attn_plan", 1)
    sv.spec_set_tuning("attn_plan_waves", waves)
    try:
        step = _step(b, cfg)
        step.attn_out.fill_(7.0)
        out = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"])
        torch.cuda.synchronize()
    finally:
        sv.spec_set_tuning("attn_plan", 0)
        sv.spec_set_tuning("attn_plan_waves", 0)
    ref, ref_lse = _oracle_attn(oracle, b, want_lse=True)
    _close(out.float().cpu().numpy(), ref, name, sharp=sq is not None)
    np.testing.assert_allclose(step.lse.cpu().numpy(), ref_lse, rtol=2e-3, atol=2e-3)
    assert int(step.status.cpu()) == 0


def test_balanced_work_list_skips_and_flags_bad_requests(sv, oracle):
    cfg = wl.VerifyConfig("bad_plan", 22, 4, (2,), ("uniform", 300, 1400), 8, 1, 64, 64, sigma_qkv=1.0)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    sv.spec_set_tuning("attn_plan", 1)
    try:
        step = _step(b, cfg)
        sl = b["seq_lens"].clone()
        sl[1] = b["max_kv_len"] + 100                  # longer than the bound the launch was sized for
        step.attn_out.fill_(5.0)
        out = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], sl, b["qo_indptr"], b["scale"])
        torch.cuda.synchronize()
        assert int(step.status.cpu()) & sv.FLAG_BAD_LENGTH
        qo = b["qo_indptr"].cpu().numpy()
        assert (out[qo[1]:qo[2]].float() == 5.0).all()
        ref = _oracle_attn(oracle, b)
        keep = np.r_[0:qo[1], qo[2]:qo[4]]
        _close(out.float().cpu().numpy()[keep], ref[keep], "others unaffected", sharp=True)
        step.status.zero_()
        pt = b["page_table"].clone()
        pt[2, 3] = -1                                   # unmapped page inside request 2's range
        step.attn(b["q"], b["k_cache"], b["v_cache"], pt, b["seq_lens"], b["qo_indptr"], b["scale"])
        torch.cuda.synchronize()
        assert int(step.status.cpu()) & sv.FLAG_BAD_PAGE
    finally:
        sv.spec_set_tuning("attn_plan", 0)


def test_attention_needle_and_causality(sv, oracle):
    """A dominant key at candidate position c+2 must be seen by rows j >= 2 only (mask and page mapping)."""
    cfg = wl.VerifyConfig("needle", 13, 3, (4,), ("uniform", 100, 400), 8, 1, 64, 64)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    direction = torch.ones(cfg.D, device="cuda") / math.sqrt(cfg.D)
    b["q"][:] = (8.0 * direction).to(torch.bfloat16)
    ctx = b["ctx"].tolist()
    pt = b["page_table"].cpu()
    for i, c in enumerate(ctx):
        t = c + 2
        page = int(pt[i, t // 16])
        b["k_cache"][page, 0, t % 16] = (64.0 * direction).to(torch.bfloat16)
        b["v_cache"][page, 0, t % 16] = 7.0
    step = _step(b, cfg)
    out = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"])
    torch.cuda.synchronize()
    o = out.float().cpu().numpy().reshape(3, 5, 8, cfg.D)
    assert np.abs(o[:, :2]).max() < 0.1
    np.testing.assert_allclose(o[:, 2:], 7.0, atol=0.05)
    _close(out.float().cpu().numpy(), _oracle_attn(oracle, b), "needle")


@pytest.mark.parametrize("gammas", [(8,), (0, 2, 4)], ids=["row_split_kernel", "wave_per_key_block_kernel"])
def test_attention_with_an_overwhelming_key_in_every_key_group(sv, oracle, gammas):
    """One committed key per request whose score exceeds every other by ~200 in log2 units, at slot 1, 6, 9 or 14 of its
    page (one of the four groups of keys a 16-lane row of the wave owns): the running maximum has to come from all
    four groups, or the exponentials overflow.  The output is then that key's value row."""
    cfg = wl.VerifyConfig("dominant", 17, 8, gammas, ("uniform", 150, 600), 8, 1, 64, 64, sigma_qkv=1.0)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    direction = torch.ones(cfg.D, device="cuda") / math.sqrt(cfg.D)
    b["q"][:] = (8.0 * direction).to(torch.bfloat16)
    pt = b["page_table"].cpu()
    for i, c in enumerate(b["ctx"].tolist()):
        t = 16 * (3 + i) + (1, 6, 9, 14)[i % 4]             # inside the committed prefix (>= 150 keys): every row sees it
        page = int(pt[i, t // 16])
        b["k_cache"][page, 0, t % 16] = (200.0 * direction).to(torch.bfloat16)
        b["v_cache"][page, 0, t % 16] = 7.0
    step = _step(b, cfg)
    out = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"])
    torch.cuda.synchronize()
    o = out.float().cpu().numpy()
    assert np.isfinite(o).all()
    np.testing.assert_allclose(o, 7.0, atol=0.05)
    _close(o, _oracle_attn(oracle, b), "dominant key")
    assert int(step.status.cpu()) == 0


def _split_geometry(length, target):
    """(splits, keys per split) of a request of `length` keys when splits are at most `target` keys long."""
    ns = -(-length // target)
    return ns, (-(-length // ns) + 15) // 16 * 16


@pytest.mark.parametrize("mode", ["fixed_4096", "work_list"])
def test_long_context_sharp_data_and_needles(sv, oracle, mode):
    """Contexts of 32k-40k keys on permuted pages, unit-variance Q/K/V (a peaked softmax: one page is visible),
    with the fixed 4096-key split (256 page ids staged per workgroup) and with the device-built work list.
    Then the same batch with a handful of dominant keys, each carrying its own value pattern, placed in
    several splits, on both sides of a split boundary, at the end of a split, in the last partial page and inside
    the candidate block: a page fetched from the wrong place or left out changes the mean of the patterns."""
    cfg = wl.VerifyConfig("long_sharp", 61, 2, (4,), ("uniform", 32768, 40000), 8, 1, 64, 64, sigma_qkv=1.0)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    tuning = {"attn_plan": 2, "attn_chunk": 4096} if mode == "fixed_4096" else {"attn_plan": 1}
    for k, v in tuning.items():
        sv.spec_set_tuning(k, v)
    try:
        step = _step(b, cfg)
        run = lambda: step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"])
        out = run()
        torch.cuda.synchronize()
        ref, ref_lse = _oracle_attn(oracle, b, want_lse=True)
        _close(out.float().cpu().numpy(), ref, f"{mode} sharp", sharp=True)
        np.testing.assert_allclose(step.lse.cpu().numpy(), ref_lse, rtol=2e-3, atol=2e-3)

        # needles
        direction = torch.ones(cfg.D, device="cuda") / math.sqrt(cfg.D)
        b["q"][:] = (8.0 * direction).to(torch.bfloat16)
        gen = torch.Generator().manual_seed(5)
        pt = b["page_table"].cpu()
        placed = []
        for i, c in enumerate(b["ctx"].tolist()):
            length = c + 5
            spots = {5, c - 1, c + 1, length - 1}                   # first page, last committed key, a candidate, the last key
            for target in (4096, 512):
                ns, chunk = _split_geometry(length, target)
                for sp in (1, ns // 2, ns - 1):
                    kbeg, kend = sp * chunk, min(length, (sp + 1) * chunk)
                    if 0 < kbeg < kend:
                        spots |= {kbeg - 1, kbeg, kend - 1}
            for t in sorted(spots):
                page = int(pt[i, t // 16])
                pattern = (torch.randint(0, 2, (cfg.D,), generator=gen) * 2 - 1).to(torch.float32) * 4.0
                b["k_cache"][page, 0, t % 16] = (64.0 * direction).to(torch.bfloat16)
                b["v_cache"][page, 0, t % 16] = pattern.to(torch.bfloat16).cuda()
                placed.append((i, t, pattern.numpy()))
        out = run()
        torch.cuda.synchronize()
        got = out.float().cpu().numpy()
        ref = _oracle_attn(oracle, b)
        _close(got, ref, f"{mode} needles", sharp=True)
        # independent of the oracle: every row is the plain mean of the patterns it may see
        qo = b["qo_indptr"].cpu().numpy()
        for i, c in enumerate(b["ctx"].tolist()):
            for j in range(5):
                seen = np.stack([pat for (ii, t, pat) in placed if ii == i and t <= c + j])
                np.testing.assert_allclose(got[qo[i] + j], np.broadcast_to(seen.mean(0), (8, cfg.D)), atol=0.04)
        assert int(step.status.cpu()) == 0
    finally:
        for k in tuning:
            sv.spec_set_tuning(k, 0)


def test_attention_flags_bad_inputs_without_faulting(sv, oracle):
    cfg = wl.VerifyConfig("bad", 14, 3, (2,), ("uniform", 40, 90), 8, 1, 64, 64, sigma_qkv=1.0)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    step = _step(b, cfg)
    pt = b["page_table"].clone()
    pt[1, 1] = b["num_pages"] + 5                      # out-of-range page id inside request 1's range
    step.attn(b["q"], b["k_cache"], b["v_cache"], pt, b["seq_lens"], b["qo_indptr"], b["scale"])
    torch.cuda.synchronize()
    assert int(step.status.cpu()) & sv.FLAG_BAD_PAGE
    step.status.zero_()
    sl = b["seq_lens"].clone()
    sl[2] = b["max_kv_len"] + 100                      # longer than the bound the launch was sized for
    step.attn_out.fill_(5.0)
    out = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], sl, b["qo_indptr"], b["scale"])
    torch.cuda.synchronize()
    assert int(step.status.cpu()) & sv.FLAG_BAD_LENGTH
    qo = b["qo_indptr"].cpu().numpy()
    assert (out[qo[2]:qo[3]].float() == 5.0).all()      # skipped request's rows untouched
    ref = _oracle_attn(oracle, b)
    _close(out[:qo[2]].float().cpu().numpy(), ref[:qo[2]], "others unaffected", sharp=True)


def test_host_side_rejections(sv):
    cfg = wl.VerifyConfig("rej", 15, 2, (2,), ("uniform", 40, 90), 8, 1, 64, 64)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    step = _step(b, cfg)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(sv.SpecError) as e:
        sv.spec_verify_attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"],
                            step.attn_out, None, b["max_kv_len"], 3, b["scale"], None, small)
    assert e.value.code == -3
    with pytest.raises(sv.SpecError) as e:                 # 8 heads * 17 rows > 128 rows per kv head
        sv.spec_verify_attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"],
                            step.attn_out, None, b["max_kv_len"], 17, b["scale"], None, step.attn_ws)
    assert e.value.code == -2
    h = torch.zeros((4, 100), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sv.SpecError):
        sv.spec_lm_head(h, torch.zeros((8, 100), dtype=torch.bfloat16, device="cuda"),
                        torch.zeros((4, 8), dtype=torch.float32, device="cuda"))


# --------------------------------------------------------------------------- LM head
@pytest.mark.parametrize("M,H,V,std", [(20, 1024, 32000, 0.02), (7, 192, 1013, 1.0), (160, 512, 4100, 1.0), (45, 768, 3001, 1.0),
                                       (300, 256, 777, 1.0), (1, 64, 5, 1.0), (64, 128, 128, 1.0)])
def test_lm_head_matches_oracle(sv, oracle, M, H, V, std):
    g = torch.Generator(device="cuda").manual_seed(M * 7 + V)
    hs, ws = (1.0, 1.0 / math.sqrt(H)) if std == 1.0 else (std, std)      # unit-variance logits, or the paper-like scale
    hidden = (torch.randn((M, H), generator=g, device="cuda") * hs).to(torch.bfloat16)
    W = (torch.randn((V, H), generator=g, device="cuda") * ws).to(torch.bfloat16)
    logits = torch.full((M, V), 3.0, dtype=torch.float32, device="cuda")
    sv.spec_lm_head(hidden, W, logits)
    torch.cuda.synchronize()
    ref = oracle.lm_head(wl.bf16_bits(hidden), wl.bf16_bits(W))
    got = logits.cpu().numpy()
    _close(got, ref, f"lm_head {M}x{H}x{V}", sharp=std == 1.0)
    # fp32 accumulation of exact bf16 products: far tighter than the contract
    assert np.abs(got - ref).max() <= 1e-5 * max(1.0, np.abs(ref).max()) * math.sqrt(H)


def _packed_layout(wbits: np.ndarray) -> np.ndarray:
    """The packed vocabulary matrix as the header defines it, by index arithmetic on the host."""
    V, H = wbits.shape
    panels = (V + 15) // 16
    padded = np.zeros((panels * 16, H), dtype=np.uint16)
    padded[:V] = wbits
    # [panel, entry-in-panel, k-tile, k-group, j] -> [panel, k-tile, k-group, entry-in-panel, j]; lane = 16 * k-group + entry
    return padded.reshape(panels, 16, H // 32, 4, 8).transpose(0, 2, 3, 1, 4).reshape(-1).copy()


@pytest.mark.parametrize("V,H", [(1013, 256), (4096, 512), (5, 32), (16, 64), (3001, 768)])
def test_lm_head_pack_is_the_documented_permutation(sv, V, H):
    g = torch.Generator(device="cuda").manual_seed(V + H)
    W = torch.randn((V, H), generator=g, device="cuda").to(torch.bfloat16)
    nbytes = sv.spec_lm_head_packed_bytes(V, H)
    assert nbytes == (V + 15) // 16 * 16 * H * 2
    Wp = torch.full((nbytes // 2,), 7.0, dtype=torch.bfloat16, device="cuda")
    sv.spec_lm_head_pack(W, Wp)
    torch.cuda.synchronize()
    assert np.array_equal(wl.bf16_bits(Wp), _packed_layout(wl.bf16_bits(W)))


@pytest.mark.parametrize("M,H,V,std", [(20, 1024, 32000, 0.02), (7, 256, 1013, 1.0), (160, 512, 4100, 1.0), (45, 768, 3001, 1.0),
                                       (300, 256, 777, 1.0), (1, 256, 5, 1.0), (64, 256, 128, 1.0), (97, 512, 70001, 1.0),
                                       (130, 256, 16 * 256 * 16 + 4, 1.0), (161, 256, 2049, 1.0), (576, 512, 9000, 1.0), (1153, 256, 4104, 1.0),
                                       (3, 256, 1000004, 1.0)])                  # a million entries: 16 passes per workgroup
def test_lm_head_packed_matches_oracle(sv, oracle, M, H, V, std):
    g = torch.Generator(device="cuda").manual_seed(M * 7 + V)
    hs, ws = (1.0, 1.0 / math.sqrt(H)) if std == 1.0 else (std, std)
    hidden = (torch.randn((M, H), generator=g, device="cuda") * hs).to(torch.bfloat16)
    W = (torch.randn((V, H), generator=g, device="cuda") * ws).to(torch.bfloat16)
    Wp = torch.empty((sv.spec_lm_head_packed_bytes(V, H) // 2,), dtype=torch.bfloat16, device="cuda")
    sv.spec_lm_head_pack(W, Wp)
    logits = torch.full((M, V), 3.0, dtype=torch.float32, device="cuda")
    sv.spec_lm_head_packed(hidden, Wp, logits)
    torch.cuda.synchronize()
    ref = oracle.lm_head(wl.bf16_bits(hidden), wl.bf16_bits(W))
    got = logits.cpu().numpy()
    _close(got, ref, f"lm_head_packed {M}x{H}x{V}", sharp=std == 1.0)
    assert np.abs(got - ref).max() <= 1e-5 * max(1.0, np.abs(ref).max()) * math.sqrt(H)
    # the other launch variants (4 waves; passes of 512 entries over row groups of at most 80) add in the same order
    try:
        for key, value, back in (("lm_packed_waves", 4, 8), ("lm_packed_wide", 1, 0), ("lm_packed_wide", 2, 0)):
            sv.spec_set_tuning(key, value)
            again = torch.zeros_like(logits)
            sv.spec_lm_head_packed(hidden, Wp, again)
            torch.cuda.synchronize()
            assert torch.equal(again, logits), key
            sv.spec_set_tuning(key, back)
    finally:
        sv.spec_set_tuning("lm_packed_waves", 8)
        sv.spec_set_tuning("lm_packed_wide", 0)


@pytest.mark.parametrize("M,cap", [(161, 0), (200, 0), (224, 0), (240, 0), (256, 0), (270, 0), (300, 0), (418, 0), (576, 0), (1206, 0),
                                   (1206, 256), (500, 144), (700, 240)])
def test_lm_head_large_tile_kernel(sv, oracle, M, cap):
    """The MFMA-bound kernel behind spec_lm_head_packed for M > 160, at every row-tile count per group it is built for
    (9..16, even and uneven groups, a last group with a ragged tile), vocabulary sizes with ragged panels and passes:
    every logit against the oracle, and the same bits as the weight-streaming kernel (same k order per output)."""
    H, V = 512, 4104 + 16 * (M % 7)
    g = torch.Generator(device="cuda").manual_seed(M + cap)
    hidden = torch.randn((M, H), generator=g, device="cuda").to(torch.bfloat16)
    W = (torch.randn((V, H), generator=g, device="cuda") / math.sqrt(H)).to(torch.bfloat16)
    Wp = torch.empty(sv.spec_lm_head_packed_bytes(V, H) // 2, dtype=torch.bfloat16, device="cuda")
    sv.spec_lm_head_pack(W, Wp)
    guard = 256
    flat = torch.full((M * V + 2 * guard,), 9.0, dtype=torch.float32, device="cuda")
    logits = flat[guard:guard + M * V].view(M, V)
    other = torch.empty((M, V), dtype=torch.float32, device="cuda")
    sv.spec_set_tuning("lm_mfma_rows", cap)
    try:
        sv.spec_lm_head_packed(hidden, Wp, logits)
        sv.spec_set_tuning("lm_packed_tile", 1)
        sv.spec_lm_head_packed(hidden, Wp, other)
        torch.cuda.synchronize()
    finally:
        sv.spec_set_tuning("lm_mfma_rows", 0)
        sv.spec_set_tuning("lm_packed_tile", 0)
    assert (flat[:guard] == 9.0).all() and (flat[-guard:] == 9.0).all()
    assert torch.equal(logits, other)
    ref = oracle.lm_head(wl.bf16_bits(hidden), wl.bf16_bits(W))
    _close(logits.cpu().numpy(), ref, f"large tile M={M}", sharp=True)


def test_lm_head_packed_rejects_bad_shapes(sv):
    hidden = torch.zeros((4, 192), dtype=torch.bfloat16, device="cuda")
    Wp = torch.zeros((sv.spec_lm_head_packed_bytes(40, 192) // 2,), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sv.SpecError) as e:
        sv.spec_lm_head_packed(hidden, Wp, torch.zeros((4, 40), dtype=torch.float32, device="cuda"))
    assert e.value.code == -2
    with pytest.raises(sv.SpecError) as e:
        sv.spec_lm_head_pack(torch.zeros((40, 48), dtype=torch.bfloat16, device="cuda"),
                             torch.zeros((sv.spec_lm_head_packed_bytes(40, 48) // 2,), dtype=torch.bfloat16, device="cuda"))
    assert e.value.code == -2
    assert sv.spec_lm_head_packed_bytes(0, 256) == 0


# --------------------------------------------------------------------------- acceptance
def _accept_both(sv, oracle, logits, tokens, dp, temp, seeds, round_, qo, gamma_max):
    B, (M, V) = len(qo) - 1, logits.shape
    dev = lambda a, dt=None: None if a is None else torch.from_numpy(a).cuda()
    ws = torch.empty(max(256, sv.spec_accept_workspace_bytes(B, M, V, gamma_max)), dtype=torch.uint8, device="cuda")
    al = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    ot = torch.full((B, gamma_max + 1), -9, dtype=torch.int32, device="cuda")
    rb = torch.full((B,), 9, dtype=torch.uint8, device="cuda")
    stats = torch.full((4,), -9, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    seeds_dev = None if seeds is None else torch.from_numpy(seeds.view(np.int64)).cuda()
    sv.spec_accept(dev(logits), dev(tokens), dev(dp), dev(temp), seeds_dev, round_, dev(qo), al, ot, rb, stats,
                   gamma_max, status, ws)
    torch.cuda.synchronize()
    ref = oracle.accept(logits, tokens, dp, temp, seeds, round_, qo, gamma_max)
    got = dict(accept_len=al.cpu().numpy(), out_tokens=ot.cpu().numpy(), rollback=rb.cpu().numpy(),
               stats=stats.cpu().numpy(), status=int(status.cpu()))
    return got, ref


def _assert_same(got, ref, gammas):
    assert np.array_equal(got["accept_len"], ref["accept_len"])
    assert np.array_equal(got["out_tokens"], ref["out_tokens"])
    assert np.array_equal(got["rollback"], ref["rollback"])
    assert got["stats"][0] == int(ref["rollback"].sum())
    assert got["stats"][2] == len(gammas)


def _qo(gammas):
    qo = np.zeros(len(gammas) + 1, np.int32)
    qo[1:] = np.cumsum(np.asarray(gammas) + 1)
    return qo


@pytest.mark.parametrize("V", [5, 1000, 4096, 4097, 32000, 151936])
def test_greedy_accept_is_bit_exact(sv, oracle, V):
    rng = np.random.default_rng(V)
    gammas = rng.choice([0, 2, 4, 8], 24)
    qo = _qo(gammas)
    logits = rng.normal(0, 0.03, (qo[-1], V)).astype(np.float32)
    cfg = wl.VerifyConfig("g", V, len(gammas), (4,), ("const", 1), 8, 1, 64, V, rho=0.7)
    tokens, planned = wl.draft_tokens_greedy(cfg, torch.from_numpy(qo), torch.from_numpy(logits.argmax(1)))
    got, ref = _accept_both(sv, oracle, logits, tokens.numpy(), None, np.zeros(len(gammas), np.float32), None, 0, qo, 8)
    _assert_same(got, ref, gammas)
    if V > 1:
        assert np.array_equal(ref["accept_len"], planned.numpy())
    assert got["status"] == 0
    assert got["stats"][1] == int((ref["accept_len"] + 1).sum())


@pytest.mark.parametrize("rho", [0.2, 0.6, 0.95])
def test_mode_rule_from_device_counters(sv, oracle, rho):
    # eq. mode_switch_batch: the counters spec_accept leaves on the device give the same mode, r_hat and r* as
    # the oracle's rule applied to the oracle's own acceptance result
    V = 4097
    rng = np.random.default_rng(int(rho * 100))
    gammas = np.full(48, 4)
    qo = _qo(gammas)
    logits = rng.normal(0, 0.03, (qo[-1], V)).astype(np.float32)
    cfg = wl.VerifyConfig("g", V, len(gammas), (4,), ("const", 1), 8, 1, 64, V, rho=rho)
    tokens, _ = wl.draft_tokens_greedy(cfg, torch.from_numpy(qo), torch.from_numpy(logits.argmax(1)))
    got, ref = _accept_both(sv, oracle, logits, tokens.numpy(), None, np.zeros(len(gammas), np.float32), None, 0, qo, 4)
    _assert_same(got, ref, gammas)
    for (t_d, t_t) in [(1.0, 10.0), (3.0, 40.0), (0.2, 47.0)]:
        want = oracle.next_mode(int(ref["rollback"].sum()), int((ref["accept_len"] + 1).sum()), len(gammas), 5, t_d, t_t)
        have = sv.spec_next_mode(got["stats"], 5, t_d, t_t)
        assert have[0] == want[0] and have[1] == want[1] and math.isclose(have[2], want[2], rel_tol=1e-15)


def test_greedy_ties_and_duplicates_across_segments(sv, oracle):
    V = 10000
    logits = np.zeros((3, V), np.float32)
    logits[0, [4095, 4096, 9000]] = 1.0          # tie straddling a segment boundary: lowest index wins
    logits[1, [8191, 70]] = 2.0
    logits[2, :] = -1.0
    qo = _qo([2])
    tokens = np.array([0, 4095, 70], np.int32)
    got, ref = _accept_both(sv, oracle, logits, tokens, None, np.zeros(1, np.float32), None, 0, qo, 2)
    _assert_same(got, ref, [2])
    assert got["accept_len"][0] == 2 and got["out_tokens"][0, 2] == 0


@pytest.fixture(params=[0, 2, 3], ids=["interval_test", "fp64_sums_on_every_row", "interval_left_open"])
def accept_filter(request, sv):
    """How sampled requests get their normalisers: fp32 bulk sums + interval test + fp64 on the bonus row (default),
    fp64 sums on every row, or an interval so wide that nearly every test falls through to the exact fallback.
    The integers must be the oracle's in all three."""
    sv.spec_set_tuning("accept_filter", request.param)
    yield request.param
    sv.spec_set_tuning("accept_filter", 0)


@pytest.mark.parametrize("V,T,sigma", [(5, 0.8, 1.5), (1000, 0.7, 1.0), (4097, 1.0, 2.0), (32000, 0.7, 0.03), (151936, 1.0, 0.03),
                                       (20000, 0.3, 6.0)])      # the last: sharp rows, exponents down to -200
def test_stochastic_accept_is_bit_exact(sv, oracle, V, T, sigma, accept_filter):
    rng = np.random.default_rng(V + 1)
    B = 48
    gammas = rng.choice([0, 2, 4, 8], B)
    qo = _qo(gammas)
    logits = rng.normal(0, sigma, (qo[-1], V)).astype(np.float32)
    cfg = wl.VerifyConfig("s", V, B, (4,), ("const", 1), 8, 1, 64, V)
    dp, tokens = wl.draft_probs_noisy(cfg, torch.from_numpy(qo), torch.from_numpy(logits), noise_std=1.0)
    seeds = rng.integers(0, 2 ** 63, B, dtype=np.uint64)
    temp = np.full(B, T, np.float32)
    temp[::5] = 0.0                                        # a few greedy requests in the same batch
    got, ref = _accept_both(sv, oracle, logits, tokens.numpy(), dp.numpy(), temp, seeds, 3, qo, 8)
    _assert_same(got, ref, gammas)
    assert got["status"] == 0
    assert 0 < ref["accept_len"].sum() < gammas.sum()       # both accepts and rejections occur


@pytest.mark.parametrize("V,B,gamma", [(270000, 6, 3), (2200000, 3, 2), (1000, 5, 63), (4100, 4, 40)],
                         ids=["66_segments", "538_segments_unstaged", "64_rows", "41_rows_2_segments"])
def test_stochastic_accept_wide_vocabularies_and_deep_drafts(sv, oracle, V, B, gamma, accept_filter):
    """More than 64 segments per row (the segment walks go round their 64-lane loops more than once), more than 512 (the
    draw reads the segment sums in place), and up to 64 candidate rows per request (every lane of the decision wave holds
    a draft; rows beyond the sixteenth are merged in a second turn of the waves)."""
    rng = np.random.default_rng(V + gamma)
    gammas = np.full(B, gamma)
    gammas[0] = max(1, gamma // 2)
    qo = _qo(gammas)
    logits = rng.normal(0, 1.0, (qo[-1], V)).astype(np.float32)
    cfg = wl.VerifyConfig("w", V % 1000, B, (gamma,), ("const", 1), 8, 1, 64, V)
    dp, tokens = wl.draft_probs_noisy(cfg, torch.from_numpy(qo), torch.from_numpy(logits), noise_std=0.3)
    seeds = rng.integers(0, 2 ** 63, B, dtype=np.uint64)
    temp = np.full(B, 0.8, np.float32)
    if B > 3:
        temp[1] = 0.0
    got, ref = _accept_both(sv, oracle, logits, tokens.numpy(), dp.numpy(), temp, seeds, 5, qo, gamma)
    _assert_same(got, ref, gammas)
    assert got["status"] == 0
    assert ref["accept_len"].sum() > 0


def test_stochastic_one_hot_drafter_and_q_equal_p(sv, oracle, accept_filter):
    rng = np.random.default_rng(5)
    V, B = 3000, 32
    gammas = np.full(B, 4)
    qo = _qo(gammas)
    logits = rng.normal(0, 2.0, (qo[-1], V)).astype(np.float32)
    tokens = rng.integers(0, V, qo[-1]).astype(np.int32)
    tokens.reshape(B, 5)[:, 1:] = logits.reshape(B, 5, V)[:, :4].argmax(2)      # likely-accepted drafts
    seeds = rng.integers(0, 2 ** 63, B, dtype=np.uint64)
    temp = np.full(B, 0.9, np.float32)
    got, ref = _accept_both(sv, oracle, logits, tokens, None, temp, seeds, 1, qo, 4)      # draft_probs == NULL
    _assert_same(got, ref, gammas)
    # q == p: every draft accepted
    dp = np.stack([oracle.target_probs(logits[qo[i] + j], 0.9) for i in range(B) for j in range(4)])
    got, ref = _accept_both(sv, oracle, logits, tokens, dp, temp, seeds, 1, qo, 4)
    _assert_same(got, ref, gammas)
    assert (got["accept_len"] == 4).all()


@pytest.mark.parametrize("V", [5, 10000, 151936])
def test_sampler_without_positive_residual_draws_from_the_target(sv, oracle, V, accept_filter):
    """A rejected draft whose residual max(0, p - q) is zero everywhere: (a) the draft is a masked entry (-inf logit)
    and q equals p, so 0 < 0 rejects it; (b) q = 2p, rejected whenever u >= 1/2.  The bonus then comes from p
    itself.  One and several 4096-entry segments; integers identical to the oracle's."""
    rng = np.random.default_rng(V + 17)
    B = 40
    gammas = np.full(B, 2)
    qo = _qo(gammas)
    logits = rng.normal(0, 1.5, (qo[-1], V)).astype(np.float32)
    tokens = rng.integers(0, V, qo[-1]).astype(np.int32)
    dp = np.zeros((qo[-1] - B, V), np.float32)
    for i in range(B):
        r0 = qo[i]
        masked_at = 1 + (i % 2)                                  # the draft that hits the masked entry (even i: the first)
        d = int(tokens[r0 + masked_at])
        logits[r0 + masked_at - 1, d] = -np.inf
        for j in (1, 2):
            p = oracle.target_probs(logits[r0 + j - 1], 0.9)
            dp[r0 - i + j - 1] = p if i % 4 < 2 else 2.0 * p       # (b) for half of the requests
        if masked_at == 2:                                       # a first draft that q == p accepts: any token with p > 0
            tokens[r0 + 1] = int(np.argmax(logits[r0]))
    seeds = rng.integers(0, 2 ** 63, B, dtype=np.uint64)
    temp = np.full(B, 0.9, np.float32)
    got, ref = _accept_both(sv, oracle, logits, tokens, dp, temp, seeds, 11, qo, 2)
    _assert_same(got, ref, gammas)
    assert got["status"] == 0
    al = ref["accept_len"]
    assert (al[0::4] == 0).all() and (al[1::4] == 1).all()      # q == p: rejected exactly at the masked draft
    assert (al < 2).all() and (ref["out_tokens"][np.arange(B), al] >= 0).all()
    for i in range(B):                                           # rejected at the masked draft: the bonus is never that entry
        if al[i] == i % 2:
            assert ref["out_tokens"][i, al[i]] != tokens[qo[i] + 1 + (i % 2)]


def test_sampler_fallback_bucket_across_segments(sv, oracle, accept_filter):
    """p = (1/2, 1/4, 1/4) on entries 10, 5000 and 9000 of a 10000-entry row (three different segments), every
    other entry masked; the draft is a masked entry and q = p: the bonus is the bucket of U(seed, round, 1, 1)."""
    V, B = 10000, 64
    row = np.full(V, -np.inf, np.float32)
    row[[10, 5000, 9000]] = np.log(np.array([2.0, 1.0, 1.0])).astype(np.float32)
    qo = _qo(np.full(B, 1))
    logits = np.tile(np.stack([row, row]), (B, 1))
    tokens = np.tile(np.array([0, 7777], np.int32), B)
    dp = np.tile(oracle.target_probs(row, 1.0)[None, :], (B, 1))
    seeds = np.arange(100, 100 + B, dtype=np.uint64)
    got, ref = _accept_both(sv, oracle, logits, tokens, dp, np.ones(B, np.float32), seeds, 4, qo, 1)
    _assert_same(got, ref, np.full(B, 1))
    assert (got["accept_len"] == 0).all()
    hits = set()
    for i in range(B):
        u = oracle.uniform(int(seeds[i]), 4, 1, 1)
        want = None if min(abs(u - 0.5), abs(u - 0.75)) < 1e-6 else 10 if u < 0.5 else 5000 if u < 0.75 else 9000
        if want is not None:
            assert got["out_tokens"][i, 0] == want
            hits.add(want)
    assert hits == {10, 5000, 9000}


def test_accept_flags_bad_rows_and_tokens(sv, oracle):
    rng = np.random.default_rng(6)
    V = 5000
    gammas = [2, 2, 2, 0]
    qo = _qo(gammas)
    logits = rng.normal(0, 1, (qo[-1], V)).astype(np.float32)
    logits[1, 4500] = np.nan                                 # request 0
    logits[4, 17] = -np.inf                                  # request 1: fine
    tokens = rng.integers(0, V, qo[-1]).astype(np.int32)
    tokens[7] = V + 3                                        # request 2: token out of range
    temp = np.array([0.0, 0.0, 1.0, 1.0], np.float32)
    seeds = rng.integers(0, 2 ** 63, 4, dtype=np.uint64)
    got, ref = _accept_both(sv, oracle, logits, tokens, None, temp, seeds, 0, qo, 2)
    assert np.array_equal(got["accept_len"], ref["accept_len"])
    assert np.array_equal(got["out_tokens"], ref["out_tokens"])
    assert np.array_equal(got["rollback"], ref["rollback"])
    assert got["status"] & sv.FLAG_BAD_LOGITS and got["status"] & sv.FLAG_BAD_TOKEN
    assert got["out_tokens"][0, 0] == -1 and got["out_tokens"][2, 0] == -1 and got["out_tokens"][3, 0] >= 0


# --------------------------------------------------------------------------- commit
def test_kv_commit_is_bit_exact(sv, oracle):
    rng = np.random.default_rng(7)
    for B in (1, 5, 257, 1500):
        cfg = wl.VerifyConfig("c", B, B, (0, 2, 4, 8), ("uniform", 0, 200), 8, 1, 64, 64)
        b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
        gam = b["gammas"].numpy()
        acc = np.array([rng.integers(0, g + 1) for g in gam], np.int32)
        pt, sl = b["page_table"].cpu().numpy().copy(), b["seq_lens"].cpu().numpy().copy()
        fl, fc = b["free_list"].cpu().numpy().copy(), b["free_count"].cpu().numpy().copy()
        qo = b["qo_indptr"].cpu().numpy()
        oracle.kv_commit(pt, sl, qo, acc, fl, fc, 16)
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        sv.spec_kv_commit(b["page_table"], b["seq_lens"], b["qo_indptr"], torch.from_numpy(acc).cuda(), b["free_list"],
                          b["free_count"], 16, status)
        torch.cuda.synchronize()
        assert np.array_equal(b["page_table"].cpu().numpy(), pt)
        assert np.array_equal(b["seq_lens"].cpu().numpy(), sl)
        assert int(b["free_count"].cpu()) == int(fc[0])
        assert np.array_equal(b["free_list"].cpu().numpy()[:int(fc[0])], fl[:int(fc[0])])
        assert int(status.cpu()) == 0


def test_empty_batch_calls_are_noops(sv):
    z32 = torch.zeros(1, dtype=torch.int32, device="cuda")
    sv.spec_kv_commit(z32.view(1, 1), z32[:0], z32, z32[:0], z32, z32.clone(), 16, None)
    # no rows: the LM heads launch nothing and leave the (empty) logits alone; no entries: nothing to pack
    W = torch.ones((48, 256), dtype=torch.bfloat16, device="cuda")
    Wp = torch.full((sv.spec_lm_head_packed_bytes(48, 256) // 2,), 5.0, dtype=torch.bfloat16, device="cuda")
    none = torch.zeros((0, 256), dtype=torch.bfloat16, device="cuda")
    sv.spec_lm_head(none, W, torch.zeros((0, 48), dtype=torch.float32, device="cuda"))
    sv.spec_lm_head_packed(none, Wp, torch.zeros((0, 48), dtype=torch.float32, device="cuda"))
    sv.spec_lm_head_pack(W[:0], Wp[:0])
    torch.cuda.synchronize()
    assert (Wp == 5.0).all()


# --------------------------------------------------------------------------- candidates of the next round
def _assemble_both(sv, oracle, al, ot, qo, cont, cl, rep, rl, mode, gn):
    B = al.shape[0]
    dev = lambda a: None if a is None else torch.from_numpy(a).cuda()
    nt = torch.full((max(1, B * (gn + 1)),), -9, dtype=torch.int32, device="cuda")
    nqo = torch.full((B + 1,), -9, dtype=torch.int32, device="cuda")
    rb = torch.full((max(1, B),), 9, dtype=torch.uint8, device="cuda")
    st = torch.full((4,), -9, dtype=torch.int32, device="cuda")
    sv.spec_assemble_next(dev(al), dev(ot), dev(qo), dev(cont), dev(cl), dev(rep), dev(rl), mode, gn, nt, nqo, rb[:B], st)
    torch.cuda.synchronize()
    ref = oracle.assemble_next(al, ot, qo, cont, cl, rep, rl, mode, gn)
    assert np.array_equal(nqo.cpu().numpy(), ref["qo_indptr"])
    assert np.array_equal(nt.cpu().numpy()[:ref["rows"]], ref["tokens"])
    assert (nt.cpu().numpy()[ref["rows"]:] == -9).all()                        # nothing written past the last row
    assert np.array_equal(rb.cpu().numpy()[:B], ref["rollback"])
    assert np.array_equal(st.cpu().numpy(), ref["stats"])
    return ref


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("B", [1, 7, 64, 1024, 1025, 3000])
def test_next_round_candidates_are_bit_exact(sv, oracle, B, mode):
    rng = np.random.default_rng(B + mode)
    gam = rng.choice([0, 2, 4, 8], B)
    qo = np.zeros(B + 1, np.int32)
    qo[1:] = np.cumsum(gam + 1)
    al = np.array([rng.integers(0, g + 1) for g in gam], np.int32)
    ot = np.full((B, 9), -1, np.int32)
    bonus = rng.integers(0, 1000, B).astype(np.int32)
    ot[np.arange(B), al] = bonus
    undecided = rng.random(B) < 0.03                                            # requests spec_accept flagged
    ot[undecided] = -1
    al[undecided] = 0
    cont = rng.integers(0, 1000, (B, 10)).astype(np.int32)
    agree = rng.random(B) < 0.6
    cont[agree, 0] = bonus[agree]
    cl = rng.integers(0, 11, B).astype(np.int32)
    rep = rng.integers(1000, 2000, (B, 6)).astype(np.int32)
    rl = rng.integers(0, 7, B).astype(np.int32)
    for gn in (0, 4, 8):
        _assemble_both(sv, oracle, al, ot, qo, cont, cl, rep if mode == 0 else None, rl if mode == 0 else None, mode, gn)
    _assemble_both(sv, oracle, al, ot, qo, None, None, None, None, mode, 4)       # no drafter output at all: every request decodes


def test_next_round_follows_acceptance_on_the_device(sv, oracle):
    """spec_accept -> spec_assemble_next -> spec_next_mode without a host round trip in between; the rollback set now
    counts continuations invalidated by the bonus as well (Method, "Rollback-Based Mode Selection")."""
    V = 4097
    rng = np.random.default_rng(5)
    gammas = np.full(40, 4)
    qo = _qo(gammas)
    logits = rng.normal(0, 0.03, (qo[-1], V)).astype(np.float32)
    cfg = wl.VerifyConfig("g", V, len(gammas), (4,), ("const", 1), 8, 1, 64, V, rho=0.8)
    tokens, _ = wl.draft_tokens_greedy(cfg, torch.from_numpy(qo), torch.from_numpy(logits.argmax(1)))
    got, ref = _accept_both(sv, oracle, logits, tokens.numpy(), None, np.zeros(len(gammas), np.float32), None, 0, qo, 4)
    _assert_same(got, ref, gammas)
    bonus = ref["out_tokens"][np.arange(len(gammas)), ref["accept_len"]]
    cont = rng.integers(0, V, (len(gammas), 5)).astype(np.int32)
    right = rng.random(len(gammas)) < 0.7
    cont[right, 0] = bonus[right]                                                 # the drafter guessed the bonus
    cl = np.full(len(gammas), 5, np.int32)
    r = _assemble_both(sv, oracle, got["accept_len"], got["out_tokens"], qo, cont, cl, None, None, 1, 4)
    stable = (ref["accept_len"] == gammas) & right
    assert np.array_equal(r["rollback"], (~stable).astype(np.uint8))
    assert r["stats"][0] >= int(ref["rollback"].sum())                            # a superset of "prefix rejected"
    mode = sv.spec_next_mode(r["stats"], 5, 1.0, 10.0)
    assert mode[0] == oracle.next_mode(int(r["stats"][0]), int(r["stats"][1]), len(gammas), 5, 1.0, 10.0)[0]


def test_four_rounds_chained_on_the_device(sv, oracle):
    """Verify -> accept -> commit -> next round's candidates, four rounds in a row with the state (lengths, page table,
    free list, candidates) carried from call to call on the device; the oracle runs the same loop.  Only the page
    allocation for the new candidate rows is done on the host (the library frees pages, it does not hand them out)."""
    from paper_2605_08151_amd.step import VerifyStep
    rng = np.random.default_rng(11)
    B, Hq, Hkv, D, P, H, V, gmax = 6, 8, 1, 128, 16, 256, 997, 4
    num_pages, max_pages = 96, 12
    g = torch.Generator(device="cuda").manual_seed(3)
    kc = torch.randn((num_pages, Hkv, P, D), generator=g, device="cuda").to(torch.bfloat16)   # every page holds "some" K/V
    vc = torch.randn((num_pages, Hkv, P, D), generator=g, device="cuda").to(torch.bfloat16)
    W = (torch.randn((V, H), generator=g, device="cuda") / math.sqrt(H)).to(torch.bfloat16)
    Wp = torch.empty((sv.spec_lm_head_packed_bytes(V, H) // 2,), dtype=torch.bfloat16, device="cuda")
    sv.spec_lm_head_pack(W, Wp)
    # host mirror of the state; the device copies are compared with it after every call that changes them
    seq = rng.integers(20, 100, B).astype(np.int32)
    pt = np.full((B, max_pages), -1, np.int32)
    perm = rng.permutation(num_pages).astype(np.int32)
    used = 0
    for i in range(B):
        n = (seq[i] + P - 1) // P
        pt[i, :n] = perm[used:used + n]
        used += n
    fl = np.full(num_pages, -1, np.int32)
    fc = np.array([num_pages - used], np.int32)
    fl[:fc[0]] = perm[used:]
    gam = rng.integers(0, gmax + 1, B)
    qo = np.zeros(B + 1, np.int32)
    qo[1:] = np.cumsum(gam + 1)
    tokens = rng.integers(0, V, qo[-1]).astype(np.int32)
    temp = np.array([0.0, 0.8] * (B // 2), np.float32)
    seeds = rng.integers(0, 2 ** 62, B).astype(np.uint64)
    d_pt, d_seq = torch.from_numpy(pt).cuda(), torch.from_numpy(seq).cuda()
    d_fl, d_fc = torch.from_numpy(fl).cuda(), torch.from_numpy(fc).cuda()
    d_temp, d_seeds = torch.from_numpy(temp).cuda(), torch.from_numpy(seeds.view(np.int64)).cuda()
    modes = []
    for rnd in range(4):
        M = int(qo[-1])
        # pages for the candidate rows (positions c_i .. c_i + gamma_i): taken from the top of the free list, on both sides
        for i in range(B):
            for pg in range((seq[i] + P - 1) // P, (seq[i] + gam[i] + 1 + P - 1) // P):
                fc[0] -= 1
                pt[i, pg] = fl[fc[0]]
                fl[fc[0]] = -1
        d_pt.copy_(torch.from_numpy(pt)); d_fl.copy_(torch.from_numpy(fl)); d_fc.copy_(torch.from_numpy(fc))
        d_qo, d_tok = torch.from_numpy(qo).cuda(), torch.from_numpy(tokens).cuda()
        q = torch.randn((M, Hq, D), generator=g, device="cuda").to(torch.bfloat16)
        hidden = torch.randn((M, H), generator=g, device="cuda").to(torch.bfloat16)
        step = VerifyStep(B, M, Hq, Hkv, D, H, V, gmax, int((seq + gam + 1).max()))
        scale = 1.0 / math.sqrt(D)
        out = step.attn(q, kc, vc, d_pt, d_seq, d_qo, scale)
        logits = step.lm_head_packed(hidden, Wp)
        step.accept(d_tok, None, d_temp, d_seeds, rnd, d_qo)
        torch.cuda.synchronize()
        _close(out.float().cpu().numpy(), oracle.verify_attn(wl.bf16_bits(q), wl.bf16_bits(kc), wl.bf16_bits(vc), pt, seq, qo, scale),
               f"round {rnd} attention", sharp=True)
        gl = logits.cpu().numpy()
        _close(gl, oracle.lm_head(wl.bf16_bits(hidden), wl.bf16_bits(W)), f"round {rnd} logits", sharp=True)
        ref = oracle.accept(gl, tokens, None, temp, seeds, rnd, qo, gmax)
        assert np.array_equal(step.accept_len.cpu().numpy(), ref["accept_len"]), rnd
        assert np.array_equal(step.out_tokens.cpu().numpy(), ref["out_tokens"]), rnd
        step.commit(d_pt, d_seq, d_qo, d_fl, d_fc, P)
        oracle.kv_commit(pt, seq, qo, ref["accept_len"], fl, fc, P)
        torch.cuda.synchronize()
        assert np.array_equal(d_pt.cpu().numpy(), pt) and np.array_equal(d_seq.cpu().numpy(), seq), rnd
        assert int(d_fc.cpu()) == int(fc[0]) and np.array_equal(d_fl.cpu().numpy()[:fc[0]], fl[:fc[0]]), rnd
        assert int(step.status.cpu()) == 0
        # the drafter's continuation: right about the bonus for two requests in three
        bonus = ref["out_tokens"][np.arange(B), ref["accept_len"]]
        cont = rng.integers(0, V, (B, gmax + 1)).astype(np.int32)
        right = rng.random(B) < 0.67
        cont[right, 0] = bonus[right]
        cl = np.full(B, gmax + 1, np.int32)
        mode, _, _ = sv.spec_next_mode(step.stats.cpu().numpy(), gmax + 1, 1.0, 12.0)
        assert mode == oracle.next_mode(int(ref["rollback"].sum()), int((ref["accept_len"] + 1).sum()), B, gmax + 1, 1.0, 12.0)[0]
        modes.append(mode)
        nxt = _assemble_both(sv, oracle, step.accept_len.cpu().numpy(), step.out_tokens.cpu().numpy(), qo, cont, cl, None, None,
                             mode, gmax)
        qo, tokens = nxt["qo_indptr"].copy(), nxt["tokens"].copy()
        gam = np.diff(qo) - 1
        fl[fc[0]:] = -1                                   # entries above the count are unspecified on the device
    assert (seq >= 24).all() and len(modes) == 4


def test_next_round_host_rejections(sv):
    z = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(sv.SpecError):                  # unknown mode
        sv.spec_assemble_next(z[:1], z[:1].view(1, 1), z[:2], None, None, None, None, 7, 4, z.clone(), z[:2].clone(), None, None)
    with pytest.raises(sv.SpecError):                  # negative gamma_next
        sv.spec_assemble_next(z[:1], z[:1].view(1, 1), z[:2], None, None, None, None, 1, -1, z.clone(), z[:2].clone(), None, None)
    nqo = torch.full((1,), 5, dtype=torch.int32, device="cuda")
    sv.spec_assemble_next(z[:0], z[:0].view(0, 1), z[:1], None, None, None, None, 1, 4, z.clone(), nqo, None, None)   # empty batch
    torch.cuda.synchronize()
    assert int(nqo.cpu()) == 0


# --------------------------------------------------------------------------- draft-side primitives
def _ragged(rows):
    ip = np.zeros(len(rows) + 1, np.int32)
    ip[1:] = np.cumsum([len(r) for r in rows])
    flat = np.array([t for r in rows for t in r] or [0], np.int32)
    return flat, ip


def test_divergence_point_is_bit_exact(sv, oracle):
    rng = np.random.default_rng(8)
    p_rows, h_rows = [], []
    for _ in range(500):
        n = int(rng.integers(0, 3000)) if rng.random() < 0.9 else 0
        base = rng.integers(0, 4, n).tolist()
        other = list(base)
        if n and rng.random() < 0.7:
            other[int(rng.integers(0, n))] += 1
        if n and rng.random() < 0.1:
            other[0] += 1                                                     # differ at the very first token
        cut = int(rng.integers(0, n + 1))
        p_rows.append(base)
        h_rows.append(other[:cut] if rng.random() < 0.3 else other + [7] * int(rng.integers(0, 3)))
    pt, pi = _ragged(p_rows)
    ht, hi = _ragged(h_rows)
    delta = torch.full((len(p_rows),), -9, dtype=torch.int32, device="cuda")
    sv.spec_divergence(torch.from_numpy(pt).cuda(), torch.from_numpy(pi).cuda(), torch.from_numpy(ht).cuda(),
                       torch.from_numpy(hi).cuda(), delta)
    torch.cuda.synchronize()
    assert np.array_equal(delta.cpu().numpy(), oracle.divergence(pt, pi, ht, hi))


def test_kv_rollback_is_bit_exact(sv, oracle):
    rng = np.random.default_rng(9)
    for B in (1, 5, 257, 1500):
        cfg = wl.VerifyConfig("t", B, B, (0, 2, 4, 8), ("uniform", 0, 300), 8, 1, 64, 64)
        b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
        lens = (b["seq_lens"].cpu().numpy() + b["gammas"].numpy() + 1).astype(np.int32)   # candidates written: full lengths
        keep = np.array([rng.integers(-2, l + 5) for l in lens], np.int32)
        pt, sl = b["page_table"].cpu().numpy().copy(), lens.copy()
        fl, fc = b["free_list"].cpu().numpy().copy(), b["free_count"].cpu().numpy().copy()
        oracle.kv_truncate(pt, sl, keep, fl, fc, 16)
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        sl_d = torch.from_numpy(lens).cuda()
        sv.spec_kv_truncate(b["page_table"], sl_d, torch.from_numpy(keep).cuda(), b["free_list"], b["free_count"], 16, status)
        torch.cuda.synchronize()
        assert np.array_equal(b["page_table"].cpu().numpy(), pt) and np.array_equal(sl_d.cpu().numpy(), sl)
        assert int(b["free_count"].cpu()) == int(fc[0])
        assert np.array_equal(b["free_list"].cpu().numpy()[:int(fc[0])], fl[:int(fc[0])])
        assert int(status.cpu()) == 0


@pytest.mark.parametrize("p_num,p_den", [(1, 10), (1, 4), (2, 3), (0, 1), (7, 5)])
def test_prompt_compression_is_bit_exact(sv, oracle, p_num, p_den):
    rng = np.random.default_rng(p_num * 10 + p_den)
    rows = [rng.integers(0, 50000, int(rng.integers(0, 9000))).tolist() for _ in range(90)]
    rows[3] = []
    flat, ip = _ragged(rows)
    out = torch.full((len(flat) + 8,), -9, dtype=torch.int32, device="cuda")
    idx = torch.full((len(flat) + 8,), -9, dtype=torch.int32, device="cuda")
    oip = torch.full((len(rows) + 1,), -9, dtype=torch.int32, device="cuda")
    sv.spec_compress_prompts(torch.from_numpy(flat).cuda(), torch.from_numpy(ip).cuda(), p_num, p_den, out, oip, idx)
    torch.cuda.synchronize()
    want, woip, widx = oracle.compress_prompts(flat, ip, p_num, p_den)
    n = len(want)
    assert np.array_equal(oip.cpu().numpy(), woip)
    assert np.array_equal(out.cpu().numpy()[:n], want) and (out.cpu().numpy()[n:] == -9).all()
    assert np.array_equal(idx.cpu().numpy()[:n], widx)


# --------------------------------------------------------------------------- tree-structured verification
def _random_parents(rng, gammas):
    out = []
    for g in gammas:
        out.append(-1)
        out += [int(rng.integers(0, j)) for j in range(1, int(g) + 1)]
    return np.array(out, np.int32)


TREE_CASES = [
    # name, B, gammas, ctx, Hq, Hkv
    ("tree_g8", 5, (0, 2, 4, 8), ("uniform", 1, 700), 8, 1),
    ("tree_gqa", 6, (4, 7), ("uniform", 100, 1500), 32, 8),
    ("tree_15", 3, (15,), ("uniform", 200, 600), 8, 1),
    ("tree_short", 8, (0, 3, 8), ("uniform", 0, 20), 8, 2),
    ("tree_split", 4, (4, 8), ("uniform", 900, 2500), 8, 1),
]


@pytest.mark.parametrize("plan", [0, 1])
@pytest.mark.parametrize("case", TREE_CASES, ids=[c[0] for c in TREE_CASES])
def test_tree_attention_matches_oracle(sv, oracle, case, plan):
    name, B, gammas, ctx, Hq, Hkv = case
    cfg = wl.VerifyConfig(name, 61, B, gammas, ctx, Hq, Hkv, 64, 64, sigma_qkv=1.0)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    rng = np.random.default_rng(len(name))
    parent = _random_parents(rng, b["gammas"].numpy())
    sv.spec_set_tuning("attn_plan", 1 if plan else 2)
    if name == "tree_split":
        sv.spec_set_tuning("attn_chunk", 256)
    try:
        step = _step(b, cfg)
        step.attn_out.fill_(7.0)
        sv.spec_verify_attn_tree(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"],
                                 torch.from_numpy(parent).cuda(), step.attn_out, step.lse, b["max_kv_len"],
                                 b["gamma_max"] + 1, b["scale"], step.status, step.attn_ws)
        torch.cuda.synchronize()
    finally:
        sv.spec_set_tuning("attn_plan", 0)
        sv.spec_set_tuning("attn_chunk", 0)
    ref, ref_lse = oracle.verify_attn_tree(wl.bf16_bits(b["q"]), wl.bf16_bits(b["k_cache"]), wl.bf16_bits(b["v_cache"]),
                                           b["page_table"].cpu().numpy(), b["seq_lens"].cpu().numpy(),
                                           b["qo_indptr"].cpu().numpy(), parent, b["scale"], want_lse=True)
    _close(step.attn_out.float().cpu().numpy(), ref, name, sharp=True)
    np.testing.assert_allclose(step.lse.cpu().numpy(), ref_lse, rtol=2e-3, atol=2e-3)
    assert int(step.status.cpu()) == 0


def test_tree_attention_chain_parents_and_bad_trees(sv, oracle):
    cfg = wl.VerifyConfig("treechain", 62, 4, (3, 6), ("uniform", 50, 400), 8, 1, 64, 64, sigma_qkv=1.0)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    gam = b["gammas"].numpy()
    chain = np.concatenate([np.arange(-1, g, dtype=np.int32) for g in gam])
    step = _step(b, cfg)
    plain = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"]).clone()
    lse_plain = step.lse.clone()
    sv.spec_verify_attn_tree(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"],
                             torch.from_numpy(chain).cuda(), step.attn_out, step.lse, b["max_kv_len"], b["gamma_max"] + 1,
                             b["scale"], step.status, step.attn_ws)
    torch.cuda.synchronize()
    assert torch.equal(step.attn_out, plain) and torch.equal(step.lse, lse_plain)     # the chain is the degenerate tree
    bad = chain.copy()
    qo = b["qo_indptr"].cpu().numpy()
    bad[qo[2] + 1] = 3                                                                 # a parent after its child, request 2
    step.attn_out.fill_(5.0)
    sv.spec_verify_attn_tree(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"],
                             torch.from_numpy(bad).cuda(), step.attn_out, step.lse, b["max_kv_len"], b["gamma_max"] + 1,
                             b["scale"], step.status, step.attn_ws)
    torch.cuda.synchronize()
    assert int(step.status.cpu()) & sv.FLAG_BAD_TREE
    assert (step.attn_out[qo[2]:qo[3]].float() == 5.0).all()                           # skipped
    keep = np.r_[0:qo[2], qo[3]:qo[4]]
    assert torch.equal(step.attn_out[keep], plain[keep])


def test_tree_acceptance_and_commit_are_bit_exact(sv, oracle):
    rng = np.random.default_rng(63)
    cfg = wl.VerifyConfig("treeacc", 63, 40, (0, 3, 6, 12), ("uniform", 0, 300), 8, 2, 64, 64)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    gam = b["gammas"].numpy()
    qo = b["qo_indptr"].cpu().numpy()
    B, M, V, gmax = len(gam), int(qo[-1]), 4099, int(gam.max())
    parent = _random_parents(rng, gam)
    logits = rng.normal(0, 1, (M, V)).astype(np.float32)
    am = logits.argmax(1)
    tokens = rng.integers(0, V, M).astype(np.int32)
    for i in range(B):                                    # let most nodes carry their parent's argmax: deep walks
        for j in range(1, gam[i] + 1):
            if rng.random() < 0.7:
                tokens[qo[i] + j] = am[qo[i] + parent[qo[i] + j]]
    dev = lambda a: torch.from_numpy(a).cuda()
    ws = torch.empty(max(256, sv.spec_accept_workspace_bytes(B, M, V, gmax)), dtype=torch.uint8, device="cuda")
    al = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    ot = torch.full((B, gmax + 1), -9, dtype=torch.int32, device="cuda")
    pth = torch.full((B, gmax + 1), -9, dtype=torch.int32, device="cuda")
    rb = torch.full((B,), 9, dtype=torch.uint8, device="cuda")
    st = torch.full((4,), -9, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    sv.spec_accept_tree(dev(logits), dev(tokens), dev(parent), b["qo_indptr"], al, ot, pth, rb, st, gmax, status, ws)
    torch.cuda.synchronize()
    ref = oracle.accept_tree(logits, tokens, parent, qo, gmax)
    assert np.array_equal(al.cpu().numpy(), ref["accept_len"]) and np.array_equal(ot.cpu().numpy(), ref["out_tokens"])
    assert np.array_equal(pth.cpu().numpy(), ref["path"]) and np.array_equal(rb.cpu().numpy(), ref["rollback"])
    assert st.cpu().numpy().tolist() == [int(ref["rollback"].sum()), int((ref["accept_len"] + 1).sum()), B, 0]
    assert int(status.cpu()) == 0 and ref["accept_len"].max() >= 3
    # commit: gather the accepted paths, then the page bookkeeping
    kc, vc = wl.bf16_bits(b["k_cache"]).copy(), wl.bf16_bits(b["v_cache"]).copy()
    pt, sl = b["page_table"].cpu().numpy().copy(), b["seq_lens"].cpu().numpy().copy()
    fl, fc = b["free_list"].cpu().numpy().copy(), b["free_count"].cpu().numpy().copy()
    oracle.kv_commit_tree(kc, vc, pt, sl, qo, ref["accept_len"], ref["path"], fl, fc, 16)
    sv.spec_kv_commit_tree(b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], al, pth,
                           b["free_list"], b["free_count"], status)
    torch.cuda.synchronize()
    assert np.array_equal(wl.bf16_bits(b["k_cache"]), kc) and np.array_equal(wl.bf16_bits(b["v_cache"]), vc)
    assert np.array_equal(b["page_table"].cpu().numpy(), pt) and np.array_equal(b["seq_lens"].cpu().numpy(), sl)
    assert int(b["free_count"].cpu()) == int(fc[0])
    assert np.array_equal(b["free_list"].cpu().numpy()[:int(fc[0])], fl[:int(fc[0])])
    assert int(status.cpu()) == 0


def test_tree_acceptance_flags_bad_trees_and_tokens(sv, oracle):
    V = 1000
    qo = np.array([0, 3, 6, 9], np.int32)
    parent = np.array([-1, 0, 0, -1, 2, 0, -1, 0, 1], np.int32)      # request 1: node 1's parent is after it
    tokens = np.array([0, 4, 4, 0, 1, 2, 0, V + 5, 3], np.int32)       # request 2: a token outside the vocabulary
    logits = np.random.default_rng(1).normal(0, 1, (9, V)).astype(np.float32)
    dev = lambda a: torch.from_numpy(a).cuda()
    ws = torch.empty(max(256, sv.spec_accept_workspace_bytes(3, 9, V, 2)), dtype=torch.uint8, device="cuda")
    al = torch.full((3,), -9, dtype=torch.int32, device="cuda")
    ot = torch.full((3, 3), -9, dtype=torch.int32, device="cuda")
    pth = torch.full((3, 3), -9, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    sv.spec_accept_tree(dev(logits), dev(tokens), dev(parent), dev(qo), al, ot, pth, None, None, 2, status, ws)
    torch.cuda.synchronize()
    ref = oracle.accept_tree(logits, tokens, parent, qo, 2)
    assert np.array_equal(al.cpu().numpy(), ref["accept_len"]) and np.array_equal(ot.cpu().numpy(), ref["out_tokens"])
    assert np.array_equal(pth.cpu().numpy(), ref["path"])
    assert int(status.cpu()) & sv.FLAG_BAD_TREE and int(status.cpu()) & sv.FLAG_BAD_TOKEN
    assert ot.cpu().numpy()[1].tolist() == [-1, -1, -1] and ot.cpu().numpy()[2].tolist() == [-1, -1, -1]


# --------------------------------------------------------------------------- whole step
def _run_step(sv, oracle, cfg, stochastic, fused=False, packed=True):
    """One step as bench.py launches it (packed vocabulary matrix unless `packed` is False or `fused`)."""
    b = wl.make_batch(cfg, device="cuda")
    step = _step(b, cfg)
    qo = b["qo_indptr"].cpu().numpy()
    out = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"])
    packed = packed and cfg.H % 256 == 0
    if fused and packed:
        logits = step.lm_head_packed_stats(b["hidden"], step.pack_weights(b["W"]))
    elif fused:
        logits = step.lm_head_stats(b["hidden"], b["W"])
    elif packed:
        logits = step.lm_head_packed(b["hidden"], step.pack_weights(b["W"]))
    else:
        logits = step.lm_head(b["hidden"], b["W"])
    torch.cuda.synchronize()
    ref_attn = _oracle_attn(oracle, b)                   # before the commit changes lengths and pages
    gl = logits.cpu().numpy()
    temp = b["temperature"].cpu().numpy()
    tokens_g, _ = wl.draft_tokens_greedy(cfg, b["qo_indptr"], torch.from_numpy(gl.argmax(1)))
    dp = None
    tokens = tokens_g
    if stochastic:
        dp, tokens_s = wl.draft_probs_noisy(cfg, b["qo_indptr"], logits)
        per_row_T = np.repeat(temp, np.diff(qo))
        tokens = torch.where(torch.from_numpy(per_row_T > 0), tokens_s, tokens_g)
    seeds = b["seeds"]
    if fused:
        # an all-greedy batch may pass no seeds: then no logits are read at all
        (step.accept_packed_stats if packed else step.accept_stats)(
            tokens.cuda(), dp, b["temperature"], seeds if stochastic else None, 5, b["qo_indptr"])
    else:
        step.accept(tokens.cuda(), dp, b["temperature"], seeds, 5, b["qo_indptr"])
    torch.cuda.synchronize()
    ref = oracle.accept(gl, tokens.numpy(), None if dp is None else dp.cpu().numpy(), temp,
                        seeds.cpu().numpy().view(np.uint64), 5, qo, b["gamma_max"])
    assert np.array_equal(step.accept_len.cpu().numpy(), ref["accept_len"])
    assert np.array_equal(step.out_tokens.cpu().numpy(), ref["out_tokens"])
    assert np.array_equal(step.rollback.cpu().numpy(), ref["rollback"])
    pt, sl = b["page_table"].cpu().numpy().copy(), b["seq_lens"].cpu().numpy().copy()
    fl, fc = b["free_list"].cpu().numpy().copy(), b["free_count"].cpu().numpy().copy()
    oracle.kv_commit(pt, sl, qo, ref["accept_len"], fl, fc, cfg.P)
    step.commit(b["page_table"], b["seq_lens"], b["qo_indptr"], b["free_list"], b["free_count"], cfg.P)
    torch.cuda.synchronize()
    assert np.array_equal(b["page_table"].cpu().numpy(), pt) and np.array_equal(b["seq_lens"].cpu().numpy(), sl)
    assert np.array_equal(b["free_list"].cpu().numpy()[:int(fc[0])], fl[:int(fc[0])])
    assert int(step.status.cpu()) == 0
    return b, step, out, gl, ref_attn


@pytest.mark.parametrize("packed", [True, False], ids=["packed", "rowmajor"])
def test_whole_step_tiny_config(sv, oracle, packed):
    """The smallest workload (4 requests, 5 rows each, short contexts) end to end."""
    cfg = wl.CONFIGS["tiny"]
    b, step, out, gl, ref_attn = _run_step(sv, oracle, cfg, stochastic=False, packed=packed)
    _close(out.float().cpu().numpy(), ref_attn, "tiny attn")
    _close(gl, oracle.lm_head(wl.bf16_bits(b["hidden"]), wl.bf16_bits(b["W"])), "tiny logits")


def test_whole_step_small_hybrid_mix(sv, oracle):
    """The hybrid ordinary-parallel mix (gamma in {0,2,4,8}, alternating greedy / sampled) at reduced size."""
    cfg = wl.VerifyConfig("hybrid_small", 21, 24, (0, 2, 4, 8), ("lognormal", 600, 1.0, 32, 4000), 8, 1, 512, 20000,
                          temperature=("alternate", 0.0, 1.0), sigma_qkv=1.0)
    b, step, out, gl, ref_attn = _run_step(sv, oracle, cfg, stochastic=True)
    _close(out.float().cpu().numpy(), ref_attn, "hybrid attn", sharp=True)
    _close(gl, oracle.lm_head(wl.bf16_bits(b["hidden"]), wl.bf16_bits(b["W"])), "hybrid logits")


@pytest.mark.parametrize("layout", ["rowmajor", "packed"])
@pytest.mark.parametrize("M,H,V", [(20, 1024, 32000), (7, 512, 1013), (33, 512, 4097), (160, 512, 20011), (128, 1024, 9000),
                                   (300, 256, 5000), (700, 256, 4100)])
def test_fused_lm_head_statistics(sv, oracle, M, H, V, layout):
    """The LM head with block statistics writes the same logits as the plain one, and every block holds its range's
    maximum and its lowest index."""
    if layout == "rowmajor" and M > 160:
        pytest.skip("the row-major statistics kernel takes at most 160 rows")
    g = torch.Generator(device="cuda").manual_seed(M + V)
    hidden = torch.randn((M, H), generator=g, device="cuda").to(torch.bfloat16)
    W = (torch.randn((V, H), generator=g, device="cuda") / math.sqrt(H)).to(torch.bfloat16)
    W[V // 3] = W[V // 2]                                  # an exact tie between two vocabulary entries
    packed = layout == "packed"
    blocks = (sv.spec_lm_head_packed_stats_blocks if packed else sv.spec_lm_head_stats_blocks)(M, H, V)
    assert blocks > 0
    plain = torch.empty((M, V), dtype=torch.float32, device="cuda")
    fused = torch.full((M, V), 3.0, dtype=torch.float32, device="cuda")
    bm = torch.full((M, blocks), 7.0, dtype=torch.float32, device="cuda")
    ba = torch.full((M, blocks), -5, dtype=torch.int32, device="cuda")
    sv.spec_lm_head(hidden, W, plain)
    if packed:
        Wp = torch.empty((sv.spec_lm_head_packed_bytes(V, H) // 2,), dtype=torch.bfloat16, device="cuda")
        sv.spec_lm_head_pack(W, Wp)
        sv.spec_lm_head_packed_stats(hidden, Wp, fused, bm, ba)
    else:
        sv.spec_lm_head_stats(hidden, W, fused, bm, ba)
    torch.cuda.synchronize()
    assert torch.equal(plain, fused)
    gl, bmn, ban = fused.cpu().numpy(), bm.cpu().numpy(), ba.cpu().numpy()
    assert not np.isnan(bmn).any()
    np.testing.assert_array_equal(bmn.max(axis=1), gl.max(axis=1))
    for r in range(M):
        best = bmn[r].max()
        assert ban[r][bmn[r] == best].min() == int(np.flatnonzero(gl[r] == best)[0])   # lowest index among ties
        real = bmn[r] > -np.inf
        assert (gl[r][ban[r][real]] == bmn[r][real]).all()                               # every block names its own maximum
        assert (np.diff(ban[r][real]) > 0).all()                                          # blocks cover increasing ranges
    ref = oracle.lm_head(wl.bf16_bits(hidden), wl.bf16_bits(W))
    _close(gl, ref, "fused logits", sharp=True)


def _summary_batch(M, B, seed):
    """qo_indptr of B requests over M rows and a temperature per request (every third greedy)."""
    rng = np.random.default_rng(seed)
    cuts = np.sort(rng.choice(np.arange(1, M), B - 1, replace=False))
    qo = np.concatenate([[0], cuts, [M]]).astype(np.int32)
    temp = rng.choice([0.5, 0.8, 1.0, 1.3], B).astype(np.float32)
    temp[::3] = 0.0
    return qo, temp


@pytest.mark.parametrize("M,H,V,sigma", [(300, 256, 5000, 1.0), (161, 256, 151936 // 8 + 4, 1.0), (700, 512, 4100, 3.0),
                                         (1206, 256, 20012, 1.0), (256, 256, 1016, 1.0)])
def test_lm_head_block_summaries(sv, oracle, M, H, V, sigma):
    """spec_lm_head_packed_summary: the logits of spec_lm_head_packed bit for bit; the blocks tile [0, V) in increasing order;
    every block holds the maximum of its range exactly and, on the rows of sampled requests, the sum of
    2^((l - max) log2(e)/T) to fp32 accuracy (0 on greedy rows)."""
    g = torch.Generator(device="cuda").manual_seed(M + V)
    hidden = (torch.randn((M, H), generator=g, device="cuda") * sigma).to(torch.bfloat16)
    W = (torch.randn((V, H), generator=g, device="cuda") / math.sqrt(H)).to(torch.bfloat16)
    W[V // 3] = W[V // 2]                                  # an exact tie between two vocabulary entries
    B = 24
    qo, temp = _summary_batch(M, B, M + V)
    blocks = sv.spec_lm_head_packed_summary_blocks(M, H, V)
    assert blocks > 0
    Wp = torch.empty((sv.spec_lm_head_packed_bytes(V, H) // 2,), dtype=torch.bfloat16, device="cuda")
    sv.spec_lm_head_pack(W, Wp)
    plain = torch.empty((M, V), dtype=torch.float32, device="cuda")
    fused = torch.full((M, V), 3.0, dtype=torch.float32, device="cuda")
    bm = torch.full((M, blocks), 7.0, dtype=torch.float32, device="cuda")
    bs = torch.full((M, blocks), -7.0, dtype=torch.float32, device="cuda")
    span = torch.full((blocks, 2), -9, dtype=torch.int32, device="cuda")
    sv.spec_lm_head_packed(hidden, Wp, plain)
    sv.spec_lm_head_packed_summary(hidden, Wp, fused, torch.from_numpy(temp).cuda(), torch.from_numpy(qo).cuda(), bm, bs, span)
    torch.cuda.synchronize()
    assert torch.equal(plain, fused)
    gl, bmn, bsn, sp = fused.cpu().numpy().astype(np.float64), bm.cpu().numpy(), bs.cpu().numpy(), span.cpu().numpy()
    used = sp[:, 1] > 0
    assert (sp[:, 1] >= 0).all() and (sp[used, 1] <= 64).all()
    first, count = sp[used, 0], sp[used, 1]
    assert first[0] == 0 and (first[1:] == first[:-1] + count[:-1]).all() and first[-1] + count[-1] == V   # a partition, in order
    row_T = np.repeat(temp, np.diff(qo)).astype(np.float64)
    for b_idx, f, c in zip(np.flatnonzero(used), first, count):
        seg = gl[:, f:f + c]
        mx = seg.max(axis=1)
        np.testing.assert_array_equal(bmn[:, b_idx].astype(np.float64), mx)
        sampled = row_T > 0
        want = np.exp2((seg[sampled] - mx[sampled, None]) * (1.4426950408889634 / row_T[sampled, None])).sum(axis=1)
        np.testing.assert_allclose(bsn[sampled, b_idx], want, rtol=1.0e-5)
        assert (bsn[~sampled, b_idx] == 0.0).all()
    _close(gl, oracle.lm_head(wl.bf16_bits(hidden), wl.bf16_bits(W)), "logits beside the summaries", sharp=True)


@pytest.mark.parametrize("V,M,sigma", [(5000, 300, 2.0), (20012, 420, 1.0), (151936, 200, 1.0)])
def test_accept_from_block_summaries_is_bit_exact(sv, oracle, V, M, sigma, accept_filter):
    """LM head with summaries, then acceptance that never scans a row: integers identical to the oracle's on the same logits,
    greedy and sampled requests mixed, ties and a NaN row included."""
    H, B = 256, 40
    g = torch.Generator(device="cuda").manual_seed(V + M)
    hidden = (torch.randn((M, H), generator=g, device="cuda") * sigma).to(torch.bfloat16)
    W = (torch.randn((V, H), generator=g, device="cuda") / math.sqrt(H)).to(torch.bfloat16)
    W[V // 3] = W[V // 2]
    rng = np.random.default_rng(V)
    gammas = rng.integers(0, 9, B)
    while gammas.sum() + B != M:                           # adjust to exactly M rows
        k = rng.integers(0, B)
        gammas[k] += 1 if gammas.sum() + B < M else (-1 if gammas[k] > 0 else 0)
    qo = _qo(gammas)
    temp = rng.choice([0.6, 0.9, 1.0], B).astype(np.float32)
    temp[::2] = 0.0
    hidden[qo[5] + 1, 7] = float("nan")                     # request 5 (sampled): one poisoned row
    hidden[qo[8], 3] = float("nan")                         # request 8 (greedy)
    blocks = sv.spec_lm_head_packed_summary_blocks(M, H, V)
    Wp = torch.empty((sv.spec_lm_head_packed_bytes(V, H) // 2,), dtype=torch.bfloat16, device="cuda")
    sv.spec_lm_head_pack(W, Wp)
    logits = torch.empty((M, V), dtype=torch.float32, device="cuda")
    bm = torch.empty((M, blocks), dtype=torch.float32, device="cuda")
    bs = torch.empty((M, blocks), dtype=torch.float32, device="cuda")
    span = torch.empty((blocks, 2), dtype=torch.int32, device="cuda")
    temp_d, qo_d = torch.from_numpy(temp).cuda(), torch.from_numpy(qo).cuda()
    sv.spec_lm_head_packed_summary(hidden, Wp, logits, temp_d, qo_d, bm, bs, span)
    torch.cuda.synchronize()
    gl = logits.cpu().numpy()
    cfg = wl.VerifyConfig("s", V % 977, B, (4,), ("const", 1), 8, 1, 64, V)
    clean = torch.nan_to_num(logits, nan=0.0)
    dp, tokens_s = wl.draft_probs_noisy(cfg, qo_d, clean, noise_std=0.7)
    tokens_g, _ = wl.draft_tokens_greedy(cfg, qo_d, clean.argmax(1).cpu())
    per_row_T = np.repeat(temp, np.diff(qo))
    tokens = torch.where(torch.from_numpy(per_row_T > 0), tokens_s, tokens_g).to(torch.int32)
    seeds = rng.integers(0, 2 ** 63, B, dtype=np.uint64)
    gmax = int(gammas.max())
    ws = torch.empty(max(256, sv.spec_accept_workspace_bytes(B, M, V, gmax)), dtype=torch.uint8, device="cuda")
    al = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    ot = torch.full((B, gmax + 1), -9, dtype=torch.int32, device="cuda")
    rb = torch.full((B,), 9, dtype=torch.uint8, device="cuda")
    stats = torch.full((4,), -9, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    sv.spec_accept_summary(logits, tokens.cuda(), dp, temp_d, torch.from_numpy(seeds.view(np.int64)).cuda(), 9, qo_d, al, ot, rb,
                           stats, gmax, bm, bs, span, blocks, status, ws)
    torch.cuda.synchronize()
    ref = oracle.accept(gl, tokens.numpy(), dp.cpu().numpy(), temp, seeds, 9, qo, gmax)
    got = dict(accept_len=al.cpu().numpy(), out_tokens=ot.cpu().numpy(), rollback=rb.cpu().numpy(), stats=stats.cpu().numpy())
    _assert_same(got, ref, gammas)
    assert int(status.cpu()) == sv.FLAG_BAD_LOGITS and ref["status"] != 0      # both sides flag the poisoned rows
    bad = [i for i in range(B) if np.isnan(gl[qo[i]:qo[i + 1]]).any()]
    assert len(bad) >= 2 and (got["accept_len"][bad] == 0).all() and (got["out_tokens"][bad] == -1).all()
    assert 0 < ref["accept_len"].sum() < gammas.sum()


@pytest.mark.parametrize("layout", ["rowmajor", "packed"])
def test_fused_statistics_carry_nan_rows(sv, oracle, layout):
    """A NaN in a hidden row makes that row's logits NaN: flagged through the block statistics exactly as by the scan."""
    cfg = wl.VerifyConfig("nanrow", 31, 6, (2,), ("const", 40), 8, 1, 512, 5003)
    b = wl.make_batch(cfg, device="cuda")
    b["hidden"][4, 7] = float("nan")                      # request 1, row 1
    results = []
    for fused in (False, True):
        step = _step(b, cfg)
        if fused and layout == "packed":
            logits = step.lm_head_packed_stats(b["hidden"], step.pack_weights(b["W"]))
            accept = step.accept_packed_stats
        elif fused:
            logits = step.lm_head_stats(b["hidden"], b["W"])
            accept = step.accept_stats
        else:
            logits = step.lm_head(b["hidden"], b["W"])
            accept = step.accept
        torch.cuda.synchronize()
        tokens, _ = wl.draft_tokens_greedy(cfg, b["qo_indptr"], torch.nan_to_num(logits).argmax(1).cpu())
        accept(tokens.cuda(), None, b["temperature"], None, 0, b["qo_indptr"])
        torch.cuda.synchronize()
        assert int(step.status.cpu()) & sv.FLAG_BAD_LOGITS
        results.append((step.accept_len.cpu().numpy(), step.out_tokens.cpu().numpy(), step.rollback.cpu().numpy(),
                        step.stats.cpu().numpy()))
    for x, y in zip(*results):
        assert np.array_equal(x, y)
    assert results[1][0][1] == 0 and (results[1][1][1] == -1).all()
    ref = oracle.accept(logits.cpu().numpy(), tokens.numpy(), None, b["temperature"].cpu().numpy(), None, 0,
                        b["qo_indptr"].cpu().numpy(), b["gamma_max"])
    assert np.array_equal(results[1][0], ref["accept_len"]) and np.array_equal(results[1][1], ref["out_tokens"])


@pytest.mark.parametrize("packed", [True, False], ids=["packed", "rowmajor"])
@pytest.mark.parametrize("name,stochastic", [("tiny", False), ("mid", False), ("hybrid_small", True)])
def test_whole_step_with_fused_statistics(sv, oracle, name, stochastic, packed):
    """The step through spec_lm_head_stats + spec_accept_stats: same integers as the oracle on the GPU's logits
    (greedy requests decided from block maxima, sampled ones from the scan, in one batch for the mix)."""
    cfg = wl.CONFIGS[name] if name in wl.CONFIGS else wl.VerifyConfig(
        "hybrid_small", 21, 24, (0, 2, 4, 8), ("lognormal", 600, 1.0, 32, 4000), 8, 1, 512, 20000,
        temperature=("alternate", 0.0, 1.0), sigma_qkv=1.0)
    b, step, out, gl, ref_attn = _run_step(sv, oracle, cfg, stochastic=stochastic, fused=True, packed=packed)
    assert (step.pblocks if packed else step.blocks) > 0
    _close(out.float().cpu().numpy(), ref_attn, f"{name} attn", sharp=name == "hybrid_small")


# --------------------------------------------------------------------------- determinism, bounds, large batches
def test_results_are_bitwise_repeatable_and_stay_inside_their_buffers(sv, oracle):
    """Three runs of attention (split, work list and unsplit), LM head and stochastic acceptance give identical bits,
    and guard bands around every output keep their fill pattern (no write outside the tensors handed in)."""
    cfg = wl.VerifyConfig("rep", 41, 12, (0, 2, 4, 8), ("uniform", 300, 3000), 8, 1, 512, 20011,
                          temperature=("alternate", 0.0, 0.8), sigma_qkv=1.0)
    b = wl.make_batch(cfg, device="cuda")
    M, V, B = b["M"], cfg.V, b["B"]
    guard = 64

    def guarded(shape, dtype, fill):
        n = int(np.prod(shape))
        flat = torch.full((n + 2 * guard,), fill, dtype=dtype, device="cuda")
        return flat, flat[guard:guard + n].view(shape)

    runs = []
    for tuning in ({"attn_plan": 2, "attn_chunk": 0}, {"attn_plan": 1}, {"attn_plan": 2, "attn_chunk": 100000}):
        for k, v in tuning.items():
            sv.spec_set_tuning(k, v)
        try:
            outs = []
            for rep in range(3):
                step = _step(b, cfg)
                of, step.attn_out = guarded((M, cfg.Hq, cfg.D), torch.bfloat16, 9.0)
                lf, step.logits = guarded((M, V), torch.float32, 9.0)
                af, step.accept_len = guarded((B,), torch.int32, -77)
                tf, step.out_tokens = guarded((B, b["gamma_max"] + 1), torch.int32, -77)
                step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"])
                if rep == 1:                         # the packed kernel gives the same bits as the row-major one
                    step.lm_head_packed(b["hidden"], step.pack_weights(b["W"]))
                else:
                    step.lm_head(b["hidden"], b["W"])
                torch.cuda.synchronize()
                if rep == 0 and not runs:
                    dp, tokens_s = wl.draft_probs_noisy(cfg, b["qo_indptr"], step.logits)
                step.accept(tokens_s.cuda(), dp, b["temperature"], b["seeds"], 3, b["qo_indptr"])
                torch.cuda.synchronize()
                for flat, fill in ((of, 9.0), (lf, 9.0), (af, -77), (tf, -77)):
                    assert (flat[:guard] == fill).all() and (flat[-guard:] == fill).all()
                outs.append((step.attn_out.clone(), step.lse.clone(), step.logits.clone(), step.accept_len.clone(),
                             step.out_tokens.clone()))
            for other in outs[1:]:
                for x, y in zip(outs[0], other):
                    assert torch.equal(x, y)
            runs.append(outs[0])
        finally:
            for k in tuning:
                sv.spec_set_tuning(k, 0)
    # the three decompositions agree to the tolerance, the integer results exactly
    ref = _oracle_attn(oracle, b)
    for r in runs:
        _close(r[0].float().cpu().numpy(), ref, "decomposition", sharp=True)
        assert torch.equal(r[3], runs[0][3]) and torch.equal(r[4], runs[0][4])


def test_attention_with_more_requests_than_the_work_list_takes(sv, oracle):
    """B > 1024: the fixed-chunk path serves it even when the work list is asked for."""
    cfg = wl.VerifyConfig("manyreq", 42, 1100, (0, 1), ("uniform", 1, 60), 8, 1, 64, 64, sigma_qkv=1.0)
    b = wl.make_batch(cfg, device="cuda", with_lm_head=False)
    sv.spec_set_tuning("attn_plan", 1)
    try:
        step = _step(b, cfg)
        out = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"])
        torch.cuda.synchronize()
    finally:
        sv.spec_set_tuning("attn_plan", 0)
    _close(out.float().cpu().numpy(), _oracle_attn(oracle, b), "many requests", sharp=True)
    assert int(step.status.cpu()) == 0


def test_step_can_be_captured_in_a_graph_and_replayed(sv, oracle):
    """The four calls never allocate or synchronise, so a stream capture takes them; three replays, with eager
    work and synchronisations in between, reproduce the eager step bit for bit (work-list attention included)."""
    cfg = wl.VerifyConfig("graph", 51, 12, (0, 2, 4), ("uniform", 200, 2500), 8, 1, 512, 9001,
                          temperature=("alternate", 0.0, 0.9), sigma_qkv=1.0)
    b = wl.make_batch(cfg, device="cuda")
    qo = b["qo_indptr"]
    sv.spec_set_tuning("attn_plan", 1)
    try:
        step = _step(b, cfg)
        Wp = step.pack_weights(b["W"])
        logits = step.lm_head_packed(b["hidden"], Wp)
        torch.cuda.synchronize()
        dp, tokens = wl.draft_probs_noisy(cfg, qo, logits)
        tokens = tokens.cuda()
        pristine = (b["page_table"].clone(), b["seq_lens"].clone(), b["free_list"].clone(), b["free_count"].clone())
        pt, sl, fl, fc = [t.clone() for t in pristine]

        def one():
            for dst, src in zip((pt, sl, fl, fc), pristine):
                dst.copy_(src)
            step.attn(b["q"], b["k_cache"], b["v_cache"], pt, sl, qo, b["scale"])
            step.lm_head_packed(b["hidden"], Wp)
            step.accept(tokens, dp, b["temperature"], b["seeds"], 2, qo)
            step.commit(pt, sl, qo, fl, fc, cfg.P)

        one()
        torch.cuda.synchronize()
        outputs = lambda: (step.attn_out, step.lse, step.logits, step.accept_len, step.out_tokens, step.rollback,
                           step.stats, pt, sl, fl, fc)
        ref = [t.clone() for t in outputs()]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            one()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            one()
        torch.cuda.synchronize()
        for rep in range(3):
            step.accept_len.fill_(-5)
            step.logits.zero_()
            step.attn_out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            for x, y in zip(outputs(), ref):
                assert torch.equal(x, y)
            one()                                        # eager work between the replays
            torch.cuda.synchronize()
        assert int(step.status.cpu()) == 0
    finally:
        sv.spec_set_tuning("attn_plan", 0)


# --------------------------------------------------------------------------- the benchmark workloads at full size
def _sampled_logits_check(oracle, b, gl, n_cols=192, seed=0):
    """LM head at full size: the oracle recomputes all rows for a random sample of vocabulary entries
    (plus the first and last 32, which sit in the ragged tiles)."""
    V = b["W"].shape[0]
    rng = np.random.default_rng(seed)
    cols = np.unique(np.concatenate([rng.integers(0, V, n_cols), np.arange(32), np.arange(V - 32, V)]))
    ref = oracle.lm_head(wl.bf16_bits(b["hidden"]), wl.bf16_bits(b["W"][torch.from_numpy(cols).cuda()]))
    _close(gl[:, cols], ref, "sampled logits")


def _all_logits_check(oracle, b, gl, what):
    """Every logit against the oracle, 256 rows at a time: the contract's bound, the scaled bound, and the bound that
    fp32 accumulation over H products allows (1e-5 sqrt(H) max|ref|)."""
    H = b["hidden"].shape[1]
    Wb = wl.bf16_bits(b["W"])
    for lo in range(0, gl.shape[0], 256):
        ref = oracle.lm_head(wl.bf16_bits(b["hidden"][lo:lo + 256]), Wb)
        _close(gl[lo:lo + 256], ref, f"{what}, rows {lo}..")
        assert np.abs(gl[lo:lo + 256] - ref).max() <= 1e-5 * np.sqrt(H) * np.abs(ref).max(), what


@pytest.mark.parametrize("name", ["mid", "stochastic", "long"])
def test_full_size_configuration(sv, oracle, name):
    """The mid, stochastic and long workloads at full size, in the launch configuration bench.py times:
    attention against the oracle on every row, every logit against the oracle, acceptance and
    commit bit-exact on the GPU's own logits."""
    cfg = wl.CONFIGS[name]
    stochastic = cfg.temperature != ("const", 0.0)
    b, step, out, gl, ref_attn = _run_step(sv, oracle, cfg, stochastic=stochastic)
    _close(out.float().cpu().numpy(), ref_attn, f"{name} attn")
    _sampled_logits_check(oracle, b, gl)
    # every logit, against the independent row-major kernels: both add a row's products in the same order
    packed_logits = step.logits.clone()
    assert torch.equal(step.lm_head(b["hidden"], b["W"]), packed_logits)
    # and every one of the M x 151936 logits against the oracle (mid, long: a few seconds of host time; stochastic: ~15 s)
    _all_logits_check(oracle, b, gl, f"{name} logits, all of them")


def test_full_size_hybrid_mix_properties(sv, oracle):
    """The hybrid workload (B=256, gamma in {0,2,4,8}, lognormal contexts up to 32k, half sampled):
    attention of the whole batch against the oracle (the device-built work list at full size), every logit
    against the oracle, acceptance and commit bit-exact on the whole batch."""
    cfg = wl.CONFIGS["hybrid"]
    b = wl.make_batch(cfg, device="cuda")
    step = _step(b, cfg)
    out = step.attn(b["q"], b["k_cache"], b["v_cache"], b["page_table"], b["seq_lens"], b["qo_indptr"], b["scale"])
    torch.cuda.synchronize()
    qo = b["qo_indptr"].cpu().numpy()
    ref = _oracle_attn(oracle, b)                        # all 256 requests, every row and head (a few seconds of host time)
    _close(out.float().cpu().numpy(), ref, "hybrid attn, whole batch")
    assert int(step.status.cpu()) == 0
    del ref, out
    # acceptance + commit on the whole batch
    logits = step.lm_head_packed(b["hidden"], step.pack_weights(b["W"]))
    torch.cuda.synchronize()
    gl = logits.cpu().numpy()
    _sampled_logits_check(oracle, b, gl, n_cols=64)
    # all 1206 x 151936 logits of the large-tile kernel against the oracle (~30 s of host time on 16 cores)
    _all_logits_check(oracle, b, gl, "hybrid logits, all of them")
    temp = b["temperature"].cpu().numpy()
    tokens_g, _ = wl.draft_tokens_greedy(cfg, b["qo_indptr"], torch.from_numpy(gl.argmax(1)))
    dp, tokens_s = wl.draft_probs_noisy(cfg, b["qo_indptr"], logits)
    per_row_T = np.repeat(temp, np.diff(qo))
    tokens = torch.where(torch.from_numpy(per_row_T > 0), tokens_s, tokens_g)
    step.accept(tokens.cuda(), dp, b["temperature"], b["seeds"], 2, b["qo_indptr"])
    torch.cuda.synchronize()
    ref = oracle.accept(gl, tokens.numpy(), dp.cpu().numpy(), temp, b["seeds"].cpu().numpy().view(np.uint64), 2, qo,
                        b["gamma_max"])
    assert np.array_equal(step.accept_len.cpu().numpy(), ref["accept_len"])
    assert np.array_equal(step.out_tokens.cpu().numpy(), ref["out_tokens"])
    assert np.array_equal(step.rollback.cpu().numpy(), ref["rollback"])
    # the same batch through the LM head that leaves block summaries and the acceptance that scans no logits
    Wp = step.pack_weights(b["W"])
    kept = step.logits.clone()
    step.logits.zero_()
    step.lm_head_packed_summary(b["hidden"], Wp, b["temperature"], b["qo_indptr"])
    assert torch.equal(step.logits, kept)
    step.accept_len.fill_(-7); step.out_tokens.fill_(-7); step.rollback.fill_(7)
    step.accept_summary(tokens.cuda(), dp, b["temperature"], b["seeds"], 2, b["qo_indptr"])
    torch.cuda.synchronize()
    assert np.array_equal(step.accept_len.cpu().numpy(), ref["accept_len"])
    assert np.array_equal(step.out_tokens.cpu().numpy(), ref["out_tokens"])
    assert np.array_equal(step.rollback.cpu().numpy(), ref["rollback"])
    assert int(step.status.cpu()) == 0
    # gamma = 0 requests (the padded parallel-mode candidates) emit exactly one token and never roll back
    g0 = b["gammas"].numpy() == 0
    assert (ref["accept_len"][g0] == 0).all() and (ref["rollback"][g0] == 0).all() and (ref["out_tokens"][g0, 0] >= 0).all()
    pt, sl = b["page_table"].cpu().numpy().copy(), b["seq_lens"].cpu().numpy().copy()
    fl, fc = b["free_list"].cpu().numpy().copy(), b["free_count"].cpu().numpy().copy()
    oracle.kv_commit(pt, sl, qo, ref["accept_len"], fl, fc, cfg.P)
    step.commit(b["page_table"], b["seq_lens"], b["qo_indptr"], b["free_list"], b["free_count"], cfg.P)
    torch.cuda.synchronize()
    assert np.array_equal(b["page_table"].cpu().numpy(), pt) and np.array_equal(b["seq_lens"].cpu().numpy(), sl)
    assert np.array_equal(b["free_list"].cpu().numpy()[:int(fc[0])], fl[:int(fc[0])])
