"""GPU parity tests: every entry point of the HIP library against the CPU oracle, through the
C ABI, on seeded synthetic caches (several tiles, ragged tails, every regime)."""
import dataclasses

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2604_10900_amd as cask  # noqa: E402
from oracle import ref  # noqa: E402
from synth import caches  # noqa: E402
from tests import parity  # noqa: E402

W = caches.WORKLOADS


def _note(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ whole-path parity

def test_cfg1_tiny_fp32():
    _note("cfg1 fp32 d=64 N=1088")
    c = caches.make(W["cfg1"])
    st = parity.full_check(c, parity.params_of(W["cfg1"]))
    _note(st)


def test_cfg1_all_donors_merge_fp32():
    c = caches.make(W["cfg1"], seed=7)
    st = parity.full_check(c, parity.params_of(W["cfg1"], sim_threshold=-1.0), expect_folds=True)
    assert st["folded_rows"] >= 30
    _note(st)


def test_fp32_d128_gqa_ragged():
    w = caches.scaled(W["cfg1"], head_dim=128, q_per_kv=3, n_layers=2, n_kv_heads=2, decode=700,
                      decode_hi=1900, n_seqs=3, window=20, recent=16, budget=150, core=-1,
                      fixed_clusters=None, cluster_lo=4, cluster_hi=9)
    c = caches.make(w)
    st = parity.full_check(c, parity.params_of(w, sim_threshold=0.8), expect_folds=True)
    _note(st)


def test_bf16_d64_plain_path():
    w = caches.scaled(W["cfg2"], head_dim=64, n_layers=1, n_kv_heads=3, q_per_kv=2, decode=900,
                      prefix=100, window=48, budget=160)
    c = caches.make(w)
    st = parity.full_check(c, parity.params_of(w, sim_threshold=0.85))
    _note(st)


def _ragged_bf16(lens, prefixes, G=7, Wn=128, seed=3):
    """Hand-built ragged batch: one generator group per unit."""
    parts = []
    for i, (n, pfx) in enumerate(zip(lens, prefixes)):
        w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=1, q_per_kv=G, window=Wn, prefix=pfx,
                          decode=n - pfx, wid=100 + i)
        parts.append(caches.make(w, seed=seed))
    K = torch.cat([p["K"] for p in parts])
    V = torch.cat([p["V"] for p in parts])
    Q = torch.cat([p["Q"] for p in parts])
    row_off = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int64)
    return dict(K=K, V=V, Q=Q, row_off=row_off, prefix_len=torch.tensor(prefixes, dtype=torch.int32))


@pytest.mark.parametrize("rows", ["chosen", "narrow_rows", "wide_rows"])
def test_bf16_mfma_ragged_units_all_regimes(rows, monkeypatch):
    """N == W, N just above W, identity (N <= B), merge-inactive, active, several key tiles with
    ragged tails, and prefix lengths from 0 to almost N.  W*G = 896 takes the first sweep's
    wide form (128 resident window rows per wave) by itself, the second sweep only in large
    batches: the library's choice, both sweeps narrow, both sweeps wide."""
    monkeypatch.setenv("CASK_NARROW_ROWS", "1" if rows == "narrow_rows" else "0")
    monkeypatch.setenv("CASK_WIDE_ROWS", "1" if rows == "wide_rows" else "0")
    lens = [128, 129, 200, 257, 300, 1000, 2177, 5000, 2304, 640]
    pref = [0, 1, 0, 100, 290, 0, 50, 300, 2048, 512]
    c = _ragged_bf16(lens, pref)
    p = cask.Params(dtype=cask.BF16, head_dim=128, q_per_kv=7, window=128, budget=256,
                    sim_threshold=0.9)
    st = parity.full_check(c, p)
    _note(st)


@pytest.mark.parametrize("rows", ["chosen", "wide_rows"])
def test_bf16_mfma_odd_window_noncausal_and_custom_scale(rows, monkeypatch):
    monkeypatch.setenv("CASK_WIDE_ROWS", "1" if rows == "wide_rows" else "0")
    lens = [100, 333, 1500, 3001]
    pref = [0, 33, 200, 0]
    c = _ragged_bf16(lens, pref, G=4, Wn=100, seed=5)
    for causal, scale in ((0, 0.0), (1, 0.05)):
        p = cask.Params(dtype=cask.BF16, head_dim=128, q_per_kv=4, window=100, recent=37, budget=190,
                        core=60, prefix_budget=25, sim_threshold=0.7, causal=causal,
                        softmax_scale=scale)
        st = parity.full_check(c, p)
        _note((causal, scale, st))


@pytest.mark.parametrize("G,Wn,causal", [(4, 128, 1), (2, 128, 1), (4, 128, 0), (3, 100, 1), (1, 64, 1), (4, 72, 1)])
def test_both_sweeps_in_one_launch_for_long_units(G, Wn, causal):
    """W*G <= 512: the two scoring sweeps of long units as one launch, the four waves' column sums
    added in LDS (one row block: stored; two: added onto cleared scores).  Forced here on a small
    batch (the library takes the path by itself from about a thousand (unit, row block) pairs);
    ragged units shorter than, equal to and far longer than a stage, keys inside the window,
    against the oracle, against the two-launch path, and bit-identical when run again."""
    lens = [Wn, Wn + 1, 300, 777, 1900, 4097, 2048]
    pref = [0, 0, 100, 333, 40, 1000, 0]
    c = _ragged_bf16(lens, pref, G=G, Wn=Wn, seed=11)
    kw = dict(dtype=cask.BF16, head_dim=128, q_per_kv=G, window=Wn, recent=min(Wn, 40), budget=Wn + 60,
              sim_threshold=0.8, causal=causal)
    row_off, prefix_len, K, V, Q = parity.host_arrays(c)
    p1 = cask.Params(path_flags=cask.binding.PATH_FORCE_FUSED_SWEEPS, **kw)
    p2 = cask.Params(path_flags=cask.binding.PATH_NO_FUSED_SWEEPS, **kw)
    want = ref.score(parity.ref_params(p1), row_off, K, Q)
    b1, b2 = parity.to_device(c, p1), parity.to_device(c, p2)
    s1 = cask.score(b1)
    s1b = cask.score(b1, torch.full_like(s1, 7.0))          # whatever the buffer held before
    s2 = cask.score(b2)
    torch.cuda.synchronize()
    e1 = parity.check_scores(s1.cpu().numpy(), want, row_off)
    e2 = parity.check_scores(s2.cpu().numpy(), want, row_off)
    assert torch.equal(s1, s1b), "one-launch scoring is not deterministic"
    np.testing.assert_allclose(np.add.reduceat(s1.cpu().numpy().astype(np.float64), row_off[:-1]), 1.0, atol=2e-5)
    _note((G, Wn, causal, "score error / max: one launch", e1, "two launches", e2))
    st = parity.full_check(c, p1)          # the whole event through the one-launch scoring
    _note(st)


def test_score_error_does_not_grow_with_unit_length():
    """A 48k-row unit: the row statistics sum tens of thousands of terms per window row.  Summed
    tile by tile the error stays at a few 1e-6 of the largest score (a single fp32 running sum
    per lane would be ten times off that and keep growing with the length); the bar itself is 1e-4."""
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=1, prefix=512, decode=48000 - 512)
    c = caches.make(w, seed=23)
    p = parity.params_of(w)
    row_off, prefix_len, K, V, Q = parity.host_arrays(c)
    want = ref.score(parity.ref_params(p), row_off, K, Q, n_threads=8)
    got = cask.score(parity.to_device(c, p))
    torch.cuda.synchronize()
    err = parity.check_scores(got.cpu().numpy(), want, row_off)
    _note(("48k rows: score error / max", err))
    assert err <= 5e-6


def test_nonpositive_softmax_scale_is_the_default_scale():
    """softmax_scale <= 0 means 1/sqrt(d) in cask_score and in cask_attend, as in the oracle."""
    dev = torch.device("cuda:0")
    c = _ragged_bf16([700, 1300], [0, 100], G=4, Wn=64, seed=9)
    outs = []
    for sc in (0.0, -1.0, float(np.float32(1.0 / np.sqrt(128.0)))):
        p = cask.Params(dtype=cask.BF16, head_dim=128, q_per_kv=4, window=64, budget=200, softmax_scale=sc)
        b = parity.to_device(c, p)
        outs.append(cask.score(b).cpu().numpy())
        if sc < 0:
            row_off, prefix_len, K, V, Q = parity.host_arrays(c)
            parity.check_scores(outs[-1], ref.score(parity.ref_params(p), row_off, K, Q), row_off)
    assert np.array_equal(outs[0], outs[1])
    # (1/sqrt(128) is not an fp32 number: the explicit value differs from the default in the last bit)
    np.testing.assert_allclose(outs[2], outs[0], rtol=1e-5, atol=0)
    n, G, d, stride = 3, 4, 128, 96
    Q = torch.randn(n, G, d, generator=torch.Generator().manual_seed(1)).to(torch.bfloat16).to(dev)
    Kc = torch.randn(n, stride, d, generator=torch.Generator().manual_seed(2)).to(torch.bfloat16).to(dev)
    Vc = torch.randn(n, stride, d, generator=torch.Generator().manual_seed(3)).to(torch.bfloat16).to(dev)
    lens = torch.tensor([96, 40, 7], dtype=torch.int32, device=dev)
    res = []
    for sc in (0.0, -1.0):
        p = cask.Params(dtype=cask.BF16, head_dim=d, q_per_kv=G, window=1, budget=stride, softmax_scale=sc)
        res.append(cask.attend(p, Q, Kc, Vc, lens))
        if sc < 0:
            rp = parity.ref_params(p)
            Qh, Kh, Vh = caches.host_bits(Q), caches.host_bits(Kc), caches.host_bits(Vc)
            _attend_check(p, rp, res[-1], ref.attend(rp, Qh, Kh, Vh, lens.cpu().numpy()), Qh, Kh, Vh,
                          lens.cpu().numpy(), None)
    torch.cuda.synchronize()
    assert torch.equal(res[0], res[1])


@pytest.mark.parametrize("causal", [1, 0])
def test_bf16_window_rows_shared_by_two_workgroups(causal):
    """Few key tiles and at least 512 window rows: two workgroups of the second scoring sweep
    share a key tile, half of the window rows each.  W * G = 525 is no multiple of the 64-row
    stage or of the halves; units shorter than, equal to and longer than a key tile."""
    lens = [75, 256, 300, 777, 1900]
    pref = [0, 100, 0, 333, 40]
    c = _ragged_bf16(lens, pref, G=7, Wn=75, seed=13)
    p = cask.Params(dtype=cask.BF16, head_dim=128, q_per_kv=7, window=75, recent=20, budget=160,
                    sim_threshold=0.5, causal=causal)
    st = parity.full_check(c, p)
    _note((causal, st))
    # the same window on short units only: both sweeps in one launch, nine 64-row parts of
    # which the last is partly empty
    c = _ragged_bf16([75, 256, 300, 777, 1000], [0, 100, 0, 333, 40], G=7, Wn=75, seed=14)
    st = parity.full_check(c, p)
    _note((causal, "short", st))


def test_bf16_single_query_head_small_window():
    c = _ragged_bf16([64, 700, 4100], [0, 10, 100], G=1, Wn=8, seed=9)
    p = cask.Params(dtype=cask.BF16, head_dim=128, q_per_kv=1, window=8, budget=96)
    _note(parity.full_check(c, p))


@pytest.mark.parametrize("rows", ["chosen", "narrow_rows", "wide_rows"])
def test_cfg2_two_layers_full_length(rows, monkeypatch):
    monkeypatch.setenv("CASK_NARROW_ROWS", "1" if rows == "narrow_rows" else "0")
    monkeypatch.setenv("CASK_WIDE_ROWS", "1" if rows == "wide_rows" else "0")
    w = caches.scaled(W["cfg2"], n_layers=2)
    c = caches.make(w)
    st = parity.full_check(c, parity.params_of(w))
    _note(st)


def test_cfg2_heavy_merging():
    w = caches.scaled(W["cfg2"], n_layers=1, decode=3000)
    c = caches.make(w, seed=11)
    for tau in (-1.0, 0.3):
        st = parity.full_check(c, parity.params_of(w, sim_threshold=tau), expect_folds=True)
        _note((tau, st))


def test_prompt_heavy_two_stage_and_exhausted():
    w = caches.scaled(W["cfg4"], n_layers=1, n_kv_heads=2, prefix=4096, decode=1024, budget=1024)
    c = caches.make(w)
    p = parity.params_of(w)
    pl = cask.plan(p, 4096, 5120)
    assert pl["status"] == 0 and pl["p_keep"] == 256 and pl["seeds"] > 64
    _note(parity.full_check(c, p))
    # same cache, budget so small that the prefix floor eats it: consolidation must not run
    w2 = caches.scaled(w, prefix=16384, decode=512, budget=300)
    c2 = caches.make(w2)
    p2 = parity.params_of(w2)
    assert cask.plan(p2, 16384, 16896)["status"] == cask.binding.ST_PREFIX_BUDGET_EXHAUSTED
    st = parity.full_check(c2, p2)
    b = parity.to_device(c2, p2)
    out = cask.compress(b)
    torch.cuda.synchronize()
    assert (out.status.cpu().numpy() == cask.binding.ST_PREFIX_BUDGET_EXHAUSTED).all()
    assert (out.out_len.cpu().numpy() == 300).all()
    a = out.assign.cpu().numpy().reshape(2, -1)
    assert (a[:, 16384:16896 - 128] == -1).all()
    _note(st)


def test_many_seeds_take_several_lds_blocks():
    """A small explicit core leaves hundreds of seeds per unit: the similarity kernel then walks
    the seeds block by block for every donor tile."""
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=2, prefix=64, decode=2500, budget=900)
    c = caches.make(w, seed=5)
    p = parity.params_of(w, core=100, sim_threshold=0.3)
    pl = cask.plan(p, 64, 2564)
    assert pl["seeds"] > 384
    st = parity.full_check(c, p, expect_folds=True)
    _note(st)


@pytest.mark.parametrize("case", ["bf16_cosine", "f32_kappa"])
def test_every_donor_folds(case):
    """A threshold that every pair passes: each seed folds a long run of donors (hundreds), so
    the grouped donor list and the segment fold carry the whole decode trace."""
    if case == "bf16_cosine":
        w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=3, prefix=60, decode=5000, budget=384)
        p = parity.params_of(w, sim_threshold=-1.0)
    else:
        w = caches.scaled(W["cfg1"], decode=1500, budget=200, core=40)
        band = torch.rand(w.head_dim // 2, generator=torch.Generator().manual_seed(2)).to("cuda:0")
        p = parity.params_of(w, merge_geometry=1, band_weight=band, dist_threshold=1e30)
    c = caches.make(w, seed=41)
    st = parity.full_check(c, p, expect_folds=True)
    assert st["folded_donors"] > 0.8 * w.decode * w.n_kv_heads
    _note((case, st))


def test_more_seeds_than_one_cursor_pass():
    """More than 8192 seeds in a unit: the stable split of the donor list by seed takes the
    ordinals a range at a time (seventeen ranges here)."""
    w = caches.scaled(W["cfg1"], n_seqs=1, n_layers=1, n_kv_heads=1, prefix=40, decode=15000, budget=9400,
                      cluster_frac=0.6)
    c = caches.make(w, seed=43)
    p = parity.params_of(w, core=300, sim_threshold=0.1)
    pl = cask.plan(p, 40, 15040)
    assert pl["seeds"] > 8192 + 256
    st = parity.full_check(c, p, expect_folds=True)
    assert st["folded_donors"] > 300
    _note(st)


def test_every_donor_folds_into_more_seeds_than_one_range():
    """About 830 seeds and 14 000 folding donors in a unit: the grouping of the donor list takes
    the seed ordinals in two ranges of 512, every wave splitting its own run of a long list."""
    w = caches.scaled(W["cfg1"], n_seqs=1, n_layers=1, n_kv_heads=2, prefix=40, decode=15000, budget=1000,
                      cluster_frac=0.6)
    c = caches.make(w, seed=47)
    p = parity.params_of(w, core=100, sim_threshold=-1.0)
    pl = cask.plan(p, 40, 15040)
    assert 512 < pl["seeds"] <= 1024
    st = parity.full_check(c, p, expect_folds=True)
    assert st["folded_donors"] > 2 * 13000
    _note(st)


def test_group_diagnostics_with_row_stride_and_arbitrary_assignments():
    """cask_group_diagnostics takes any assignment and any K_out with a row stride: random
    slots, a third of the rows dropped, out-of-range slots skipped; fp32 and bf16, d 64 / 128."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(71)
    for name, kw in (("cfg1", dict(decode=700)), ("cfg1", dict(head_dim=128, q_per_kv=2, decode=300)),
                     ("cfg2", dict(n_layers=1, n_kv_heads=3, prefix=40, decode=1100, budget=256)),
                     ("cfg2", dict(head_dim=64, n_layers=1, n_kv_heads=2, q_per_kv=2, prefix=30, decode=500,
                                   window=32, budget=128))):
        w = caches.scaled(W[name], **kw)
        c = caches.make(w, seed=9)
        band = torch.rand(w.head_dim // 2, generator=torch.Generator().manual_seed(3))
        p = parity.params_of(w, band_weight=band.to(dev))
        rp = parity.ref_params(p)
        row_off, prefix_len, K, V, Q = parity.host_arrays(c)
        n_units, total, B = len(row_off) - 1, int(row_off[-1]), p.budget
        stride = B + 37
        assign = rng.integers(0, B, total).astype(np.int32)
        assign[rng.random(total) < 0.33] = -1
        scores = (rng.random(total) ** 4).astype(np.float32)
        K_out = np.ascontiguousarray(K[rng.integers(0, total, n_units * stride)].reshape(n_units, stride, -1))
        want_d, want_l = ref.group_diagnostics(rp, row_off, K, scores, assign, K_out)
        b = parity.to_device(c, p)
        ko = torch.from_numpy(K_out.view(np.int16) if K_out.dtype == np.uint16 else K_out).to(dev)
        if p.dtype == cask.BF16:
            ko = ko.view(torch.bfloat16)
        skipped = assign.copy()
        skipped[::17] = B + 5                             # beyond the budget: skipped, no fault
        for a_in, wd, wl in ((assign, want_d, want_l),):
            d, l = cask.binding.group_diagnostics(b, torch.from_numpy(scores).to(dev),
                                                  torch.from_numpy(a_in).to(dev), ko)
            torch.cuda.synchronize()
            np.testing.assert_allclose(d.cpu().numpy(), wd, rtol=1e-5)
            np.testing.assert_allclose(l.cpu().numpy(), wl, rtol=2e-6)
        keep = skipped < B
        masked = np.where(keep, skipped, -1)
        wd2, wl2 = ref.group_diagnostics(rp, row_off, K, np.where(keep, scores, 0).astype(np.float32), masked, K_out)
        d, l = cask.binding.group_diagnostics(b, torch.from_numpy(scores).to(dev),
                                              torch.from_numpy(skipped).to(dev), ko)
        torch.cuda.synchronize()
        np.testing.assert_allclose(d.cpu().numpy(), wd2, rtol=1e-5)
        np.testing.assert_allclose(l.cpu().numpy(), wl2, rtol=2e-6)     # a skipped row is not "lost" either
        _note((name, kw, float(want_d.max()), float(want_l.max())))


SHORT_CASES = {
    # name: (workload overrides, parameter overrides, expect_folds)
    "steady_state": (dict(n_layers=1, n_kv_heads=4, prefix=96, decode=416, budget=384), dict(sim_threshold=0.5), True),
    "ragged_lengths": (dict(n_seqs=5, n_layers=1, n_kv_heads=2, prefix=70, decode=260, decode_hi=930, budget=300),
                       dict(sim_threshold=0.4), True),
    "every_donor_folds": (dict(n_layers=1, n_kv_heads=3, prefix=40, decode=900, budget=256), dict(sim_threshold=-1.0), True),
    "seeds_in_several_blocks": (dict(n_layers=1, n_kv_heads=2, prefix=30, decode=990, budget=700),
                                dict(core=20, sim_threshold=0.3), True),
    "radius": (dict(n_layers=1, n_kv_heads=2, prefix=64, decode=800, budget=320), dict(sim_threshold=0.2, merge_radius=30), True),
    "d64": (dict(head_dim=64, n_layers=1, n_kv_heads=3, q_per_kv=2, prefix=50, decode=600, window=48, budget=256),
            dict(sim_threshold=0.3), True),
    "prefix_evicted_too": (dict(n_layers=1, n_kv_heads=2, prefix=500, decode=400, budget=256), dict(sim_threshold=0.5), False),
    "identity_and_short": (dict(n_seqs=4, n_layers=1, n_kv_heads=1, prefix=20, decode=140, decode_hi=420, budget=250),
                           dict(sim_threshold=0.5), False),
    "prefix_budget_exhausted": (dict(n_layers=1, n_kv_heads=2, prefix=600, decode=300, budget=200),
                                dict(prefix_budget=72, recent=128, sim_threshold=0.5), False),
}


@pytest.mark.parametrize("tail", ["one_launch", "general_kernels"])
@pytest.mark.parametrize("case", sorted(SHORT_CASES))
def test_short_units_through_both_tails(case, tail, monkeypatch):
    """Units of at most 1024 rows (bf16) finish the event in one launch; CASK_FUSED_TAIL=0 sends
    them through the general kernels.  Both must match the oracle."""
    monkeypatch.setenv("CASK_FUSED_TAIL", "1" if tail == "one_launch" else "0")
    wkw, pkw, folds = SHORT_CASES[case]
    w = caches.scaled(W["cfg2"], **wkw)
    c = caches.make(w, seed=51)
    assert int((c["row_off"][1:] - c["row_off"][:-1]).max()) <= 1024
    st = parity.full_check(c, parity.params_of(w, **pkw), expect_folds=folds)
    _note((case, tail, st))


@pytest.mark.parametrize("tail", ["one_launch", "general_kernels"])
@pytest.mark.parametrize("seed", list(range(12)))
def test_random_short_batches(seed, tail, monkeypatch):
    """Seeded random shapes and parameters for batches of short ragged units (lengths, prefix,
    budget, core size, recent tail, threshold, radius, head dimension, heads per group)."""
    monkeypatch.setenv("CASK_FUSED_TAIL", "1" if tail == "one_launch" else "0")
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([64, 128]))
    window = int(rng.choice([16, 32, 48, 64]))
    G = int(rng.choice([1, 2, 4]))
    prefix = int(rng.integers(0, 400))
    lo = int(rng.integers(window + 8, 500))
    hi = int(rng.integers(lo + 1, 1024 - prefix)) if 1024 - prefix > lo + 1 else lo + 1
    if prefix + hi > 1024:
        hi = 1024 - prefix
    lo = min(lo, hi - 1) if hi - 1 >= window else window
    recent = int(rng.integers(0, window + 1))
    budget = int(rng.integers(recent + window + 8, 900))
    core = int(rng.choice([-1, 0, 10, budget // 2]))
    w = caches.scaled(W["cfg2"], head_dim=d, n_seqs=int(rng.integers(1, 4)), n_layers=1,
                      n_kv_heads=int(rng.integers(1, 4)), q_per_kv=G, prefix=prefix, decode=lo, decode_hi=hi,
                      window=window, budget=budget, recent=recent, core=core,
                      cluster_frac=float(rng.choice([0.1, 0.4, 0.8])))
    c = caches.make(w, seed=200 + seed)
    assert int((c["row_off"][1:] - c["row_off"][:-1]).max()) <= 1024
    p = parity.params_of(w, sim_threshold=float(rng.choice([-1.0, 0.2, 0.6, 0.95])),
                         merge_radius=int(rng.choice([0, 0, 17, 200])),
                         prefix_budget=int(rng.choice([-1, -1, 0, 40])))
    st = parity.full_check(c, p)
    _note((seed, tail, dict(d=d, W=window, G=G, P=prefix, dec=(lo, hi), B=budget, core=core, R=recent), st))


@pytest.mark.parametrize("rows", ["chosen", "wide_rows"])
@pytest.mark.parametrize("seed", list(range(8)))
def test_random_longer_batches(seed, rows, monkeypatch):
    """Seeded random shapes and parameters for ragged units of up to a few thousand rows: both
    dtypes, both head dimensions, both merge geometries; the scoring sweeps in the form the
    library picks and forced into their wide form (it only exists for bf16, d = 128)."""
    monkeypatch.setenv("CASK_WIDE_ROWS", "1" if rows == "wide_rows" else "0")
    rng = np.random.default_rng(3000 + seed)
    f32 = bool(rng.integers(0, 2))
    base = W["cfg1"] if f32 else W["cfg2"]
    d = int(rng.choice([64, 128]))
    window = int(rng.choice([16, 32, 64]))
    G = int(rng.choice([1, 2, 7])) if not f32 else int(rng.choice([1, 2]))
    prefix = int(rng.integers(0, 3000))
    lo = int(rng.integers(1100, 2500))
    hi = int(rng.integers(lo + 1, 4500))
    recent = int(rng.integers(0, window + 1))
    budget = int(rng.integers(recent + window + 8, 1500))
    core = int(rng.choice([-1, 0, 25, budget // 2]))
    w = caches.scaled(base, head_dim=d, n_seqs=int(rng.integers(1, 3)), n_layers=1, n_kv_heads=int(rng.integers(1, 3)),
                      q_per_kv=G, prefix=prefix, decode=lo, decode_hi=hi, window=window, budget=budget, recent=recent,
                      core=core, fixed_clusters=None, cluster_lo=3, cluster_hi=12,
                      cluster_frac=float(rng.choice([0.1, 0.5])))
    c = caches.make(w, seed=300 + seed)
    kw = dict(merge_radius=int(rng.choice([0, 0, 64])), prefix_budget=int(rng.choice([-1, -1, 100])))
    if rng.integers(0, 3) == 0:
        band = torch.rand(d // 2, generator=torch.Generator().manual_seed(seed)).to("cuda:0")
        kw.update(merge_geometry=1, band_weight=band, dist_threshold=float(rng.choice([4.0, 12.0, 1e9])))
    else:
        kw.update(sim_threshold=float(rng.choice([-1.0, 0.3, 0.7])))
    st = parity.full_check(c, parity.params_of(w, **kw))
    _note((seed, dict(f32=f32, d=d, W=window, G=G, P=prefix, dec=(lo, hi), B=budget, core=core, R=recent,
                      **{k: v for k, v in kw.items() if k != "band_weight"}), st))


def _attend_check(p, rp, got, want, Qh, Kh, Vh, lens, cnt):
    """cask_attend against the oracle.  Tolerance per element: rtol * |want| + k * A with
    A = sum_t p_t |v_t| (the oracle again, over |V|: the softmax weights do not depend on V).
    bf16: rtol = 1e-2, the bar for bf16 results of fp32 accumulation (the one rounding of the
    output is 2^-9 of the element); k = 2e-4 covers what happens before that rounding: weights
    entering the value product as two bf16 terms (2^-17 each), fp32 sums of up to 2300 terms and
    fp32 logits, all relative to the magnitudes summed, not to a result that may cancel.
    fp32: rtol = 1e-5, k = 5e-6 (fp32 accumulation alone)."""
    rtol, k = (1e-5, 5e-6) if p.dtype == cask.F32 else (1e-2, 2e-4)
    Vabs = np.abs(Vh) if Vh.dtype == np.float32 else (Vh & np.uint16(0x7FFF))
    A = ref.attend(rp, Qh, Kh, Vabs, lens, count=cnt)
    g = got.float().cpu().numpy().astype(np.float64)
    err = np.abs(g - want)
    bound = rtol * np.abs(want) + k * A
    bad = err > bound
    assert not bad.any(), f"{int(bad.sum())} elements off; worst excess {float((err - bound).max()):.3e}"
    return float((err / np.maximum(bound, 1e-300)).max())


@pytest.mark.parametrize("case", ["bf16_d128_g7", "bf16_d128_g1", "bf16_d128_g4", "bf16_d128_g12",
                                  "bf16_d64_g2", "bf16_d64_g8", "f32_d128_g5", "f32_d64_g1",
                                  "bf16_d128_g7_vector", "bf16_d64_g6_vector"])
def test_attend_over_a_compressed_cache(case, monkeypatch):
    """cask_attend against the oracle: ragged lengths inside a row stride (none, one row, fewer
    rows than a tile, tile and workgroup boundaries, thousands), with and without counts, more
    query heads than one pass takes."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(91)
    f32 = case.startswith("f32")
    d = 128 if "d128" in case else 64
    G = int(case.split("_g")[1].split("_")[0])
    # bf16 caches take the MFMA kernel; "_vector" sends them through the kernel fp32 caches use
    monkeypatch.setenv("CASK_ATTEND_VECTOR", "1" if case.endswith("_vector") else "0")
    stride = 2300
    lens = np.array([1, 7, 16, 17, 300, 2300, 1111, 0, 32, 33, 256, 257, 511], dtype=np.int32)
    n = len(lens)
    dt = torch.float32 if f32 else torch.bfloat16
    Q = (1.5 * torch.randn(n, G, d, generator=torch.Generator().manual_seed(1))).to(dt).to(dev)
    Kc = torch.randn(n, stride, d, generator=torch.Generator().manual_seed(2)).to(dt).to(dev)
    Vc = torch.randn(n, stride, d, generator=torch.Generator().manual_seed(3)).to(dt).to(dev)
    count = rng.integers(1, 40, (n, stride + 5)).astype(np.int32)
    count[rng.random(count.shape) < 0.7] = 1
    p = cask.Params(dtype=cask.F32 if f32 else cask.BF16, head_dim=d, q_per_kv=G, window=1, budget=stride)
    rp = parity.ref_params(p)
    Qh, Kh, Vh = caches.host_bits(Q), caches.host_bits(Kc), caches.host_bits(Vc)
    for cnt in (None, count):
        want = ref.attend(rp, Qh, Kh, Vh, np.maximum(lens, 1), count=cnt)
        want[lens == 0] = 0.0                       # the library's convention for an empty unit
        got = cask.attend(p, Q, Kc, Vc, torch.from_numpy(lens).to(dev),
                          count=None if cnt is None else torch.from_numpy(cnt).to(dev))
        torch.cuda.synchronize()
        assert not got[torch.from_numpy(lens == 0).to(dev)].float().abs().any()
        live = lens > 0
        _note((case, cnt is not None, "worst error / bound",
               _attend_check(p, rp, got[torch.from_numpy(live).to(dev)], want[live], Qh[live], Kh[live], Vh[live],
                             lens[live], None if cnt is None else cnt[live])))
    again = cask.attend(p, Q, Kc, Vc, torch.from_numpy(lens).to(dev), count=torch.from_numpy(count).to(dev))
    torch.cuda.synchronize()
    assert torch.equal(got, again)                                       # same bits every run


def test_attend_rows_behind_the_counted_ones():
    """A count array narrower than the row stride: the rows behind it (tokens decoded since the
    last event) enter with count 1."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(5)
    n, G, d, stride, pitch = 6, 7, 128, 520, 384
    lens = np.array([520, 384, 385, 100, 450, 519], dtype=np.int32)
    Q = (1.5 * torch.randn(n, G, d, generator=torch.Generator().manual_seed(11))).to(torch.bfloat16).to(dev)
    Kc = torch.randn(n, stride, d, generator=torch.Generator().manual_seed(12)).to(torch.bfloat16).to(dev)
    Vc = torch.randn(n, stride, d, generator=torch.Generator().manual_seed(13)).to(torch.bfloat16).to(dev)
    count = rng.integers(1, 30, (n, pitch)).astype(np.int32)
    padded = np.ones((n, stride), dtype=np.int32)
    padded[:, :pitch] = count
    p = cask.Params(dtype=cask.BF16, head_dim=d, q_per_kv=G, window=1, budget=pitch)
    want = ref.attend(parity.ref_params(p), caches.host_bits(Q), caches.host_bits(Kc), caches.host_bits(Vc),
                      lens, count=padded)
    got = cask.attend(p, Q, Kc, Vc, torch.from_numpy(lens).to(dev), count=torch.from_numpy(count).to(dev))
    torch.cuda.synchronize()
    _attend_check(p, parity.ref_params(p), got, want, caches.host_bits(Q), caches.host_bits(Kc),
                  caches.host_bits(Vc), lens, padded)


def test_attend_on_the_output_of_an_event():
    """The event's own outputs as the cache: K_out, V_out with their row stride, out_len and
    out_count from cask_compress_step, then one decode step's attention with and without the
    count bias, against the oracle on the oracle's event."""
    dev = torch.device("cuda:0")
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=4, prefix=96, decode=416, budget=384)
    c = caches.make(w, seed=61)
    p = parity.params_of(w, sim_threshold=0.3)
    rp = parity.ref_params(p)
    row_off, prefix_len, K, V, Q = parity.host_arrays(c)
    n_units, S = len(row_off) - 1, 512
    want = ref.compress_step(rp, row_off, prefix_len, K, V, Q, out_stride_rows=S)
    b = parity.to_device(c, p)
    out = cask.Outputs(b)
    Ko = torch.zeros(n_units, S, w.head_dim, dtype=torch.bfloat16, device=dev)
    Vo = torch.zeros_like(Ko)
    oc = torch.zeros(n_units, p.budget, dtype=torch.int32, device=dev)
    cask.compress_step(b, Ko, Vo, out, out_count=oc, scores=torch.from_numpy(want["scores"]).to(dev))
    torch.cuda.synchronize()
    assert np.array_equal(oc.cpu().numpy(), want["out_count"]) and int(want["out_count"].max()) > 1
    q = (2.0 * torch.randn(n_units, w.q_per_kv, w.head_dim, generator=torch.Generator().manual_seed(4))).to(torch.bfloat16).to(dev)
    qh = caches.host_bits(q)
    # (a) over the oracle's event: the same cache bits on both sides
    Kw = torch.from_numpy(want["K_out"].view(np.int16)).view(torch.bfloat16).to(dev)
    Vw = torch.from_numpy(want["V_out"].view(np.int16)).view(torch.bfloat16).to(dev)
    len_w = torch.from_numpy(want["out_len"]).to(dev)
    for cnt_w in (want["out_count"], None):
        ref_o = ref.attend(rp, qh, want["K_out"], want["V_out"], want["out_len"], count=cnt_w)
        got = cask.attend(p, q, Kw, Vw, len_w, count=None if cnt_w is None else torch.from_numpy(cnt_w).to(dev))
        torch.cuda.synchronize()
        _attend_check(p, rp, got, ref_o, qh, want["K_out"], want["V_out"], want["out_len"], cnt_w)
    # (b) over the library's own event (its folds differ from the oracle's by their bf16
    # rounding, so the oracle attends over a host copy of what the library wrote)
    Kg, Vg = caches.host_bits(Ko), caches.host_bits(Vo)
    len_g = out.out_len.cpu().numpy()
    assert np.array_equal(len_g, want["out_len"])
    for cnt_g in (oc, None):
        cnt_h = None if cnt_g is None else cnt_g.cpu().numpy()
        ref_o = ref.attend(rp, qh, Kg, Vg, len_g, count=cnt_h)
        got = cask.attend(p, q, Ko, Vo, out.out_len, count=cnt_g)
        torch.cuda.synchronize()
        _attend_check(p, rp, got, ref_o, qh, Kg, Vg, len_g, cnt_h)


def test_consolidate_with_caller_roles_naming_many_seeds():
    """cask_consolidate takes any role array: here far more seeds than the plan would ever
    produce, so the seeds of a unit do not fit one LDS block."""
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=2, prefix=50, decode=1800, budget=384)
    c = caches.make(w, seed=17)
    p = parity.params_of(w, sim_threshold=0.2)
    rp = parity.ref_params(p)
    row_off, prefix_len, K, V, Q = parity.host_arrays(c)
    rng = np.random.default_rng(3)
    total = int(row_off[-1])
    role = np.full(total, ref.DONOR, dtype=np.uint8)
    for u in range(2):
        lo, hi = int(row_off[u]), int(row_off[u + 1])
        role[lo:lo + 50] = ref.PREFIX_KEEP
        role[hi - 128:hi] = ref.RECENT
        seeds = lo + 50 + rng.choice(hi - 128 - lo - 50, size=300, replace=False)
        role[seeds] = ref.SEED
    s = rng.random(total).astype(np.float32)
    want, best, second = ref.consolidate(rp, row_off, prefix_len, K, s, role, want_sims=True)
    b = parity.to_device(c, p)
    got = cask.consolidate(b, torch.from_numpy(s).to(b.device), torch.from_numpy(role).to(b.device))
    torch.cuda.synchronize()
    n = parity.check_assign_excused(got.cpu().numpy(), want, best, second, float(np.float32(0.2)), "caller roles")
    assert (want >= 0).sum() > 1000
    _note(("excused", n))


DEDUP_CASES = {
    # name: (workload overrides, parameter overrides)
    "bf16_d128": (dict(n_kv_heads=3, prefix=100, decode=2600, budget=384, cluster_frac=0.5),
                  dict(sim_threshold=0.8, seed_dedup=4)),
    "f32_d64": (dict(base="cfg1", head_dim=64, n_kv_heads=2, prefix=40, decode=1500, budget=200, core=-1,
                     fixed_clusters=None, cluster_lo=3, cluster_hi=12, cluster_frac=0.6),
                dict(sim_threshold=0.7, seed_dedup=3)),
    # several hundred seeds: many walk blocks, kept seeds staged through LDS in many chunks
    "many_seeds": (dict(n_kv_heads=2, prefix=64, decode=5000, budget=900, core=100, cluster_frac=0.6),
                   dict(sim_threshold=0.85, seed_dedup=2)),
    # the walk covers the whole scratch (h * M beyond it)
    "whole_scratch": (dict(n_kv_heads=2, prefix=30, decode=700, budget=300, cluster_frac=0.7),
                      dict(sim_threshold=0.8, seed_dedup=30)),
    # h = 1: the walk may only pass rows over, never replace them (fewer than M seeds)
    "h1_short_units": (dict(n_kv_heads=4, prefix=60, decode=450, budget=256, cluster_frac=0.8),
                       dict(sim_threshold=0.8, seed_dedup=1)),
    # bf16 d = 64 and ragged units
    "bf16_d64_ragged": (dict(head_dim=64, n_seqs=3, n_kv_heads=2, prefix=80, decode=900, decode_hi=2400,
                             budget=320, cluster_frac=0.5),
                        dict(sim_threshold=0.75, seed_dedup=5)),
}


@pytest.mark.parametrize("case", sorted(DEDUP_CASES) + ["bf16_d128_vector", "many_seeds_vector"])
def test_dedup_seeding(case, monkeypatch):
    """De-duplicated seeding through cask_partition and the whole event against the oracle's
    walk: roles bit-exact on injected scores, folds and outputs as for the default rule.
    bf16 caches take the MFMA kernel; "_vector" sends them through the one fp32 caches use."""
    monkeypatch.setenv("CASK_DEDUP_VECTOR", "1" if case.endswith("_vector") else "0")
    case = case[:-len("_vector")] if case.endswith("_vector") else case
    wkw, pkw = DEDUP_CASES[case]
    wkw = dict(wkw)
    base = W[wkw.pop("base", "cfg2")]
    w = caches.scaled(base, n_layers=1, **wkw)
    c = caches.make(w, seed=71)
    row_off, prefix_len, K, V, Q = parity.host_arrays(c)
    # take the first threshold near the stated one that no walk decision of this cache comes
    # close to (decided on the oracle alone): a decision on the threshold would flip a whole
    # seed set, which the near-tie rule for single tokens does not cover
    for dt in (0.0, 0.013, -0.017, 0.031, -0.029, 0.047):
        p = parity.params_of(w, **{**pkw, "sim_threshold": pkw["sim_threshold"] + dt})
        rp = parity.ref_params(p)
        scores = ref.score(rp, row_off, K, Q)
        role0, _ = ref.prefix_evict(rp, row_off, prefix_len, scores)
        gap = ref.partition_keys(rp, row_off, prefix_len, K, scores, role0)[2]
        if gap.min() >= 1e-3:
            break
    else:
        pytest.fail("no clear threshold for this cache")
    st = parity.full_check(c, p, expect_folds=True)
    lo, hi = st["dedup_seeds"]
    default = parity.ref_params(parity.params_of(w, **{**pkw, "seed_dedup": 0}))
    M = max(ref.plan(default, int(prefix_len[u]), int(row_off[u + 1] - row_off[u]))["seeds"]
            for u in range(len(row_off) - 1))
    assert hi <= M and (case != "h1_short_units" or lo < M)
    _note((case, st))


def test_dedup_seeding_validates_on_the_host():
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=1, prefix=50, decode=3000, budget=1500, core=100)
    c = caches.make(w, seed=3)
    p = parity.params_of(w, seed_dedup=2)                 # 2 * 1400 possible seeds: over the walk's capacity
    b = parity.to_device(c, p)
    s = torch.rand(b.total_rows, device=b.device)
    with pytest.raises(cask.CaskError):
        cask.partition(b, s)
    band = torch.ones(w.head_dim // 2, device=b.device)
    p2 = parity.params_of(caches.scaled(w, budget=384, core=-1), seed_dedup=2, merge_geometry=1,
                          band_weight=band, dist_threshold=1.0)
    with pytest.raises(cask.CaskError):
        cask.partition(parity.to_device(c, p2), s)


@pytest.mark.parametrize("radius", [5, 40, 400])
def test_merge_radius_bf16_mfma_and_fp32(radius):
    """Donors fold only into seeds at most `radius` cache rows away (Section 5.2)."""
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=2, prefix=60, decode=2400, budget=700)
    c = caches.make(w, seed=31)
    st = parity.full_check(c, parity.params_of(w, core=150, sim_threshold=0.2, merge_radius=radius),
                           expect_folds=radius >= 40)
    _note((radius, st))
    w32 = caches.scaled(W["cfg1"], decode=900, budget=300, core=60)
    c32 = caches.make(w32, seed=32)
    _note(parity.full_check(c32, parity.params_of(w32, sim_threshold=0.1, merge_radius=radius)))


@pytest.mark.parametrize("dtype_case", ["bf16_d128", "bf16_d64", "f32_d64", "f32_d128"])
def test_kappa_weighted_merge_distance(dtype_case):
    """Geometry 1 (Section 2.5): nearest seed in the band-weighted distance, folded when within
    dist_threshold; every entry point against the oracle, with and without a radius."""
    dev = torch.device("cuda:0")
    if dtype_case == "bf16_d128":
        w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=2, prefix=60, decode=1500, budget=500)
    elif dtype_case == "bf16_d64":
        w = caches.scaled(W["cfg2"], head_dim=64, n_layers=1, n_kv_heads=2, q_per_kv=2, prefix=60, decode=900,
                          window=48, budget=300)
    elif dtype_case == "f32_d64":
        w = caches.scaled(W["cfg1"], decode=700, budget=256, core=60)
    else:
        w = caches.scaled(W["cfg1"], head_dim=128, q_per_kv=2, decode=700, window=20, recent=16, budget=200,
                          core=-1, fixed_clusters=None, cluster_lo=4, cluster_hi=9)
    c = caches.make(w, seed=33)
    d = w.head_dim
    g = torch.Generator().manual_seed(7)
    band = (torch.rand(d // 2, generator=g) ** 2).to(dev)            # a few bands dominate
    for theta, radius in ((6.0, 0), (1e9, 0), (25.0, 64)):
        p = parity.params_of(w, core=(60 if w.core < 0 else w.core), merge_geometry=1, band_weight=band,
                             dist_threshold=theta, merge_radius=radius)
        st = parity.full_check(c, p, expect_folds=theta > 1e6)
        _note((dtype_case, theta, radius, st))


def test_stage_timing_api():
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=2, decode=1200)
    c = caches.make(w)
    p = parity.params_of(w)
    b = parity.to_device(c, p)
    out = cask.compress(b)
    torch.cuda.synchronize()
    ref_src = out.out_src.clone()
    cask.binding.timing_enable(3)
    for _ in range(4):          # the fourth call is beyond the armed count: not recorded
        cask.compress(b, out)
    ms, n = cask.binding.timing_read()
    assert n == 3 and set(ms) == set(cask.binding.STAGES)
    assert all(v >= 0 for v in ms.values()) and ms["score_rows"] > 0 and ms["emit"] > 0
    cask.binding.timing_enable(2, 2)   # only the two scoring sweeps
    cask.compress(b, out)
    cask.compress(b, out)
    ms2, n2 = cask.binding.timing_read()
    assert n2 == 2 and ms2["score_rows"] > 0 and ms2["score_cols"] > 0
    assert all(ms2[k] == 0 for k in cask.binding.STAGES[2:])
    cask.binding.timing_enable(0)
    torch.cuda.synchronize()
    assert torch.equal(out.out_src, ref_src)   # recording changes nothing


def test_ragged_batch_llama_shape():
    w = caches.scaled(W["cfg5"], n_seqs=5, n_layers=1, n_kv_heads=2, decode=300, decode_hi=3000)
    c = caches.make(w)
    _note(parity.full_check(c, parity.params_of(w)))


@pytest.mark.parametrize("Wn,G,N,path", [(16, 3, 6000, "two_launches"), (64, 7, 6000, "two_launches"),
                                         (128, 7, 3000, "two_launches"), (128, 7, 3000, "two_launches_narrow"),
                                         (128, 7, 3000, "two_launches_wide"), (16, 3, 6000, "two_launches_wide"),
                                         (128, 8, 3000, "two_launches"), (100, 3, 3000, "two_launches"),
                                         (128, 4, 5000, "one_launch_long"),
                                         (64, 2, 5000, "one_launch_long"), (32, 7, 900, "one_launch_short")])
def test_score_with_steep_logit_ramps(Wn, G, N, path):
    """Logits that climb (or fall) by hundreds of octaves along the cache.  Climbing, the sums
    of the row statistics leave the fp32 range against their first-logit reference and the
    waves recompute their share with a running maximum (full row blocks, a half block, both
    one-launch forms of the scoring); falling, every later term underflows next to the first."""
    d = 128
    rng = np.random.default_rng(4)
    q = rng.standard_normal(d).astype(np.float32)
    q /= np.linalg.norm(q)
    two = cask.binding.PATH_NO_FUSED_SWEEPS | cask.binding.PATH_NO_FUSED_SCORE
    flags = {"two_launches": two, "two_launches_narrow": two | cask.binding.PATH_NARROW_ROWS,
             "two_launches_wide": two | cask.binding.PATH_WIDE_ROWS,
             "one_launch_long": cask.binding.PATH_FORCE_FUSED_SWEEPS, "one_launch_short": 0}[path]
    for direction in (+1, -1):
        ramp = np.linspace(0.0, 1.0, N, dtype=np.float32)
        if direction < 0:
            ramp = ramp[::-1].copy()
        # logit_j = scale * |Q| * ramp_j * gain  ->  up to ~500 in base-2 units
        K = (ramp[:, None] * q[None, :] * 60.0 + 0.05 * rng.standard_normal((N, d))).astype(np.float32)
        Qm = (q[None, :] * 66.0 + 0.1 * rng.standard_normal((Wn * G, d))).astype(np.float32)
        c = dict(K=torch.from_numpy(K).to(torch.bfloat16), V=torch.from_numpy(K).to(torch.bfloat16),
                 Q=torch.from_numpy(Qm).to(torch.bfloat16).reshape(1, Wn, G, d),
                 row_off=torch.tensor([0, N], dtype=torch.int64), prefix_len=torch.tensor([0], dtype=torch.int32))
        p = cask.Params(dtype=cask.BF16, head_dim=d, q_per_kv=G, window=Wn, budget=Wn + 100, path_flags=flags)
        row_off, prefix_len, Kb, Vb, Qb = parity.host_arrays(c)
        want = ref.score(parity.ref_params(p), row_off, Kb, Qb)
        b = parity.to_device(c, p)
        # (short units score inside the event: the whole event is run and its scores taken)
        got = cask.compress(b).scores if path == "one_launch_short" else cask.score(b)
        torch.cuda.synchronize()
        assert np.isfinite(got.cpu().numpy()).all()
        err = parity.check_scores(got.cpu().numpy(), want, row_off)
        _note((path, Wn, G, direction, "max score", float(want.max()), "rel err", err))


# ------------------------------------------------------------------ selection under ties

@pytest.mark.parametrize("longest", [4000, 4097, 9000, 12000, 16384, 20000])
@pytest.mark.parametrize("quant", [0, 3, 50])
def test_selection_with_tied_scores(quant, longest):
    """quant == 0: all scores equal; else scores rounded to `quant` levels so that every
    rank boundary falls inside a run of equal values.  The batch's longest unit picks the
    selection kernel's instance (4, 6, 9, 12 or 16 keys per thread; beyond 16 384 rows the keys
    are read again in every pass)."""
    rng = np.random.default_rng(quant)
    lens = [1500, 2600, longest]
    pref = [300, 1200, 100]
    row_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    total = int(row_off[-1])
    s = np.full(total, 0.25, dtype=np.float32) if quant == 0 else \
        (np.floor(rng.random(total) * quant) / quant).astype(np.float32)
    p = cask.Params(dtype=cask.BF16, head_dim=128, q_per_kv=1, window=64, budget=400)
    rp = parity.ref_params(p)
    role_w, _ = ref.prefix_evict(rp, row_off, np.array(pref), s)
    role_w, st_w = ref.partition(rp, row_off, np.array(pref), s, role_w)
    dev = torch.device("cuda:0")
    K = torch.zeros(total, 128, dtype=torch.bfloat16, device=dev)
    b = cask.Batch(p, torch.from_numpy(row_off), torch.tensor(pref, dtype=torch.int32), K, K, None)
    sd = torch.from_numpy(s).to(dev)
    role, st = cask.prefix_evict(b, sd)
    role, st = cask.partition(b, sd, role)
    torch.cuda.synchronize()
    assert np.array_equal(role.cpu().numpy(), role_w)
    assert np.array_equal(st.cpu().numpy(), st_w)


@pytest.mark.parametrize("tail", ["one_launch", "general_kernels"])
@pytest.mark.parametrize("quant", [0, 3, 50])
def test_whole_event_on_short_units_with_tied_scores(quant, tail, monkeypatch):
    """The same ties through the whole event on units of at most 1024 rows, where the
    one-launch tail ranks rows by counting: keep-sets, roles' consequences (assignments) and
    values against the oracle on the same injected scores.  The keys are far apart (nothing
    folds), so the comparison is exact."""
    monkeypatch.setenv("CASK_FUSED_TAIL", "1" if tail == "one_launch" else "0")
    rng = np.random.default_rng(100 + quant)
    lens = [300, 700, 1024, 513]
    pref = [100, 500, 30, 0]
    row_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    total = int(row_off[-1])
    s = np.full(total, 0.25, dtype=np.float32) if quant == 0 else \
        (np.floor(rng.random(total) * quant) / quant).astype(np.float32)
    p = cask.Params(dtype=cask.BF16, head_dim=128, q_per_kv=1, window=64, budget=200, sim_threshold=0.9)
    rp = parity.ref_params(p)
    Kf = rng.standard_normal((total, 128)).astype(np.float32)
    Vf = rng.standard_normal((total, 128)).astype(np.float32)
    dev = torch.device("cuda:0")
    Kd = torch.from_numpy(Kf).to(dev).to(torch.bfloat16)
    Vd = torch.from_numpy(Vf).to(dev).to(torch.bfloat16)
    Qd = torch.zeros(len(lens), 64, 1, 128, dtype=torch.bfloat16, device=dev)
    K, V, Q = caches.host_bits(Kd), caches.host_bits(Vd), caches.host_bits(Qd)
    want = ref.compress(rp, row_off, np.array(pref, dtype=np.int32), K, V, Q, scores=s)
    b = cask.Batch(p, torch.from_numpy(row_off), torch.tensor(pref, dtype=torch.int32), Kd, Vd, Qd)
    out = cask.compress(b, scores=torch.from_numpy(s).to(dev))
    torch.cuda.synchronize()
    got = parity.gpu_outputs(out, p)
    assert np.array_equal(got["out_len"], want["out_len"])
    assert np.array_equal(got["out_src"], want["out_src"])
    assert np.array_equal(got["assign"], want["assign"])
    assert np.array_equal(got["status"], want["status"])
    for u in range(len(lens)):
        L = int(want["out_len"][u])
        assert np.array_equal(got["K_out"][u, :L], want["K_out"][u, :L])
        assert np.array_equal(got["V_out"][u, :L], want["V_out"][u, :L])
        assert np.array_equal(got["out_mass"][u, :L], want["out_mass"][u, :L])


def test_selection_handles_zero_and_tiny_scores():
    rng = np.random.default_rng(5)
    N, P = 3000, 500
    s = (rng.random(N) ** 8 * 1e-30).astype(np.float32)
    s[rng.integers(0, N, 400)] = 0.0
    s[rng.integers(0, N, 50)] = -0.0
    p = cask.Params(dtype=cask.BF16, head_dim=128, q_per_kv=1, window=32, budget=300)
    rp = parity.ref_params(p)
    row_off = np.array([0, N], dtype=np.int64)
    role_w, _ = ref.prefix_evict(rp, row_off, np.array([P]), s)
    role_w, _ = ref.partition(rp, row_off, np.array([P]), s, role_w)
    dev = torch.device("cuda:0")
    K = torch.zeros(N, 128, dtype=torch.bfloat16, device=dev)
    b = cask.Batch(p, torch.from_numpy(row_off), torch.tensor([P], dtype=torch.int32), K, K, None)
    sd = torch.from_numpy(s).to(dev)
    role, _ = cask.prefix_evict(b, sd)
    role, _ = cask.partition(b, sd, role)
    torch.cuda.synchronize()
    assert np.array_equal(role.cpu().numpy(), role_w)


# ------------------------------------------------------------------ folds

def test_zero_mass_group_and_exact_fold():
    """Scores injected: one group whose members all score zero (uniform weights) and one whose
    donors carry zero weight next to a seed with weight 1/4 (the fold is the seed, exactly)."""
    d, N, P = 128, 600, 0
    rng = np.random.default_rng(2)
    K = rng.integers(-4, 5, (N, d)).astype(np.float32)
    V = rng.integers(-4, 5, (N, d)).astype(np.float32)
    K[1], K[2] = 2 * K[0], 4 * K[0]            # parallel to row 0: cosine 1
    K[201], K[202] = K[200], K[200]
    V[201], V[202] = V[200], V[200]
    s = np.zeros(N, dtype=np.float32)
    core = 10 + rng.permutation(N - 64 - 10)[:30]
    core = core[~np.isin(core, [200, 201, 202])]
    s[core] = 0.5
    s[200] = 0.25     # its two duplicates score zero, like everything outside the core
    p = cask.Params(dtype=cask.BF16, head_dim=d, q_per_kv=1, window=64, budget=64 + len(core) + 2,
                    core=len(core), prefix_budget=0, sim_threshold=0.999)
    rp = parity.ref_params(p)
    tb = lambda x: torch.from_numpy(x).to(torch.bfloat16)
    c = dict(K=tb(K), V=tb(V), Q=torch.zeros(1, 64, 1, d, dtype=torch.bfloat16),
             row_off=torch.tensor([0, N], dtype=torch.int64), prefix_len=torch.tensor([P], dtype=torch.int32))
    row_off, prefix_len, Kb, Vb, Qb = parity.host_arrays(c)
    want = ref.compress(rp, row_off, prefix_len, Kb, Vb, Qb, scores=s)
    # seeds: row 200 (0.25) and row 0 (first of the zero-score tie)
    assert want["role"][0] == ref.SEED and want["role"][200] == ref.SEED
    assert want["assign"][1] == want["assign"][0] == want["assign"][2]
    assert want["assign"][201] == want["assign"][200] == want["assign"][202]
    b = parity.to_device(c, p)
    out = cask.compress(b, scores=torch.from_numpy(s).cuda())
    torch.cuda.synchronize()
    got = parity.gpu_outputs(out, p)
    assert np.array_equal(got["out_src"], want["out_src"])
    assert np.array_equal(got["assign"], want["assign"])
    assert np.array_equal(got["status"], want["status"])
    assert parity.check_values(p, got, want, Kb.reshape(N, d), Vb.reshape(N, d), row_off) == 2
    t200, t0 = want["assign"][200], want["assign"][0]
    np.testing.assert_array_equal(parity.rows_as_float(got["K_out"][0, t200], cask.BF16), K[200])
    np.testing.assert_array_equal(parity.rows_as_float(got["V_out"][0, t200], cask.BF16), V[200])
    assert got["out_mass"][0, t200] == 0.25 and got["out_mass"][0, t0] == 0.0
    np.testing.assert_allclose(parity.rows_as_float(got["K_out"][0, t0], cask.BF16), K[0] * 7 / 3, rtol=1e-2)


@pytest.mark.parametrize("n_fold", [1, 63, 64, 65, 300])
def test_donor_list_lengths_around_the_short_list_split(n_fold):
    """Exactly n_fold donors of the first unit fold (copies of a seed's key, scaled), 300 of the
    second: lists of at most 64 entries are grouped by seed by a single wave, longer ones by the
    histogram path; both sit in one launch.  Scores injected, so roles are exact."""
    d, N, Wn, n_core, M = 128, 3000, 64, 20, 16
    rng = np.random.default_rng(700 + n_fold)
    Ks, Vs, ss = [], [], []
    for unit_fold in (n_fold, 300):
        K = rng.integers(-4, 5, (N, d)).astype(np.float32)
        V = rng.integers(-4, 5, (N, d)).astype(np.float32)
        s = (1e-3 * (1.0 + rng.permutation(N))).astype(np.float32) / N   # distinct, small
        free = rng.permutation(N - Wn)
        core, seeds, donors = free[:n_core], free[n_core:n_core + M], free[n_core + M:n_core + M + unit_fold]
        s[core] = 0.5 + 1e-3 * np.arange(n_core, dtype=np.float32)
        s[seeds] = 0.25 + 1e-3 * np.arange(M, dtype=np.float32)
        for j, r in enumerate(donors):
            K[r] = K[seeds[j % M]] * (2.0 if j % 2 else 1.0)           # cosine 1 with that seed
        Ks.append(K); Vs.append(V); ss.append(s)
    p = cask.Params(dtype=cask.BF16, head_dim=d, q_per_kv=1, window=Wn, budget=Wn + n_core + M,
                    core=n_core, prefix_budget=0, sim_threshold=0.999)
    rp = parity.ref_params(p)
    tb = lambda x: torch.from_numpy(x).to(torch.bfloat16)
    Kc, Vc, sc = np.concatenate(Ks), np.concatenate(Vs), np.concatenate(ss)
    c = dict(K=tb(Kc), V=tb(Vc), Q=torch.zeros(2, Wn, 1, d, dtype=torch.bfloat16),
             row_off=torch.tensor([0, N, 2 * N], dtype=torch.int64), prefix_len=torch.tensor([0, 0], dtype=torch.int32))
    row_off, prefix_len, Kb, Vb, Qb = parity.host_arrays(c)
    want = ref.compress(rp, row_off, prefix_len, Kb, Vb, Qb, scores=sc)
    folded = [(want["assign"][u * N:(u + 1) * N] >= 0).sum() - want["out_len"][u] for u in range(2)]
    assert folded == [n_fold, 300], folded
    b = parity.to_device(c, p)
    out = cask.compress(b, scores=torch.from_numpy(sc).cuda())
    torch.cuda.synchronize()
    got = parity.gpu_outputs(out, p)
    assert np.array_equal(got["out_len"], want["out_len"])
    assert np.array_equal(got["out_src"], want["out_src"])
    assert np.array_equal(got["assign"], want["assign"])
    assert np.array_equal(got["status"], want["status"])
    assert parity.check_values(p, got, want, Kb.reshape(2 * N, d), Vb.reshape(2 * N, d), row_off) >= min(n_fold, M)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_group_sizes_around_the_single_wave_fold_limit(dtype):
    """One seed each with 1, 63, 64, 65, 200 and 1500 donors (copies of the seed's key, scaled)
    in a unit, and a second unit with one group of 700: a seed with up to 64 donors is folded
    by one wave, a longer group by the four waves of a workgroup whose sums meet in LDS.
    Scores injected, so roles are exact; V random, so every donor's weight shows."""
    d, N, Wn, n_core, M = 128, 3000, 64, 20, 16
    dt = cask.BF16 if dtype == "bf16" else cask.F32
    rng = np.random.default_rng(911)
    Ks, Vs, ss, expect = [], [], [], []
    for sizes in ([1, 63, 64, 65, 200, 1500], [700]):
        K = rng.integers(-4, 5, (N, d)).astype(np.float32)
        V = rng.integers(-4, 5, (N, d)).astype(np.float32)
        s = (1e-3 * (1.0 + rng.permutation(N))).astype(np.float32) / N   # distinct, small
        free = rng.permutation(N - Wn)
        core, seeds, rest = free[:n_core], free[n_core:n_core + M], free[n_core + M:]
        s[core] = 0.5 + 1e-3 * np.arange(n_core, dtype=np.float32)
        s[seeds] = 0.25 + 1e-3 * np.arange(M, dtype=np.float32)
        at = 0
        for j, n in enumerate(sizes):
            for i, r in enumerate(rest[at:at + n]):
                K[r] = K[seeds[j]] * (2.0 if i % 2 else 1.0)              # cosine 1 with that seed
            at += n
        Ks.append(K); Vs.append(V); ss.append(s); expect.append(sum(sizes))
    p = cask.Params(dtype=dt, head_dim=d, q_per_kv=1, window=Wn, budget=Wn + n_core + M,
                    core=n_core, prefix_budget=0, sim_threshold=0.999)
    rp = parity.ref_params(p)
    tt = (lambda x: torch.from_numpy(x).to(torch.bfloat16)) if dtype == "bf16" else torch.from_numpy
    Kc, Vc, sc = np.concatenate(Ks), np.concatenate(Vs), np.concatenate(ss)
    c = dict(K=tt(Kc), V=tt(Vc), Q=tt(np.zeros((2, Wn, 1, d), np.float32)),
             row_off=torch.tensor([0, N, 2 * N], dtype=torch.int64), prefix_len=torch.tensor([0, 0], dtype=torch.int32))
    row_off, prefix_len, Kb, Vb, Qb = parity.host_arrays(c)
    want = ref.compress(rp, row_off, prefix_len, Kb, Vb, Qb, scores=sc)
    folded = [int((want["assign"][u * N:(u + 1) * N] >= 0).sum() - want["out_len"][u]) for u in range(2)]
    assert folded == expect, folded
    b = parity.to_device(c, p)
    outs = [parity.gpu_outputs(cask.compress(b, scores=torch.from_numpy(sc).cuda()), p) for _ in range(2)]
    torch.cuda.synchronize()
    got = outs[0]
    for k in got:
        assert np.array_equal(got[k], outs[1][k]), k          # the same bits on a second run
    assert np.array_equal(got["out_len"], want["out_len"])
    assert np.array_equal(got["out_src"], want["out_src"])
    assert np.array_equal(got["assign"], want["assign"])
    assert np.array_equal(got["status"], want["status"])
    assert parity.check_values(p, got, want, Kb.reshape(2 * N, d), Vb.reshape(2 * N, d), row_off) == 7


@pytest.mark.parametrize("step", [1, 3, 256, 32768])
def test_selection_with_scores_a_few_ulps_apart(step):
    """All scores of a unit are `step` fp32 ulps apart (a shuffled arithmetic progression of bit
    patterns), so every radix digit but the lowest ones is shared by long runs and the rank
    boundaries fall in the middle of a bucket of the last pass, at its edge, or (large steps) are
    decided passes earlier, where the select stops.  Roles against the oracle, three units."""
    rng = np.random.default_rng(step)
    lens = [3000, 9000, 20000]
    pref = [500, 2000, 300]
    row_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    parts = []
    for n in lens:
        bits = (np.uint32(0x30000000) + np.uint32(step) * rng.permutation(n).astype(np.uint32)).astype(np.uint32)
        parts.append(bits.view(np.float32))
        assert np.isfinite(parts[-1]).all() and len(np.unique(parts[-1])) == n
    s = np.concatenate(parts)
    p = cask.Params(dtype=cask.BF16, head_dim=128, q_per_kv=1, window=64, budget=400)
    rp = parity.ref_params(p)
    role_w, _ = ref.prefix_evict(rp, row_off, np.array(pref), s)
    role_w, st_w = ref.partition(rp, row_off, np.array(pref), s, role_w)
    dev = torch.device("cuda:0")
    K = torch.zeros(int(row_off[-1]), 128, dtype=torch.bfloat16, device=dev)
    b = cask.Batch(p, torch.from_numpy(row_off), torch.tensor(pref, dtype=torch.int32), K, K, None)
    sd = torch.from_numpy(s).to(dev)
    role, st = cask.prefix_evict(b, sd)
    role, st = cask.partition(b, sd, role)
    torch.cuda.synchronize()
    assert np.array_equal(role.cpu().numpy(), role_w)
    assert np.array_equal(st.cpu().numpy(), st_w)


@pytest.mark.parametrize("quant", [0, 40, None])
@pytest.mark.parametrize("N,P", [(18432, 16384), (33024, 256), (34000, 17000), (20000, 3000), (17000, 600)])
def test_event_selection_on_units_beyond_one_chunk_of_keys(N, P, quant):
    """Whole events on injected scores with units longer than the selection's 16 384 keys per
    walk: where the prefix and the decode trace take fewer chunks on their own than their span,
    the prefix rank is found in a walk of its own before the decode ranks (the first three
    shapes), else all three ranks in one walk.  quant: all scores equal / 40 levels (every rank
    boundary inside a run of equal values) / all distinct.  A short second unit rides along."""
    d, Wn = 128, 64
    rng = np.random.default_rng(N + (quant or 7))
    lens = [N, 2500]
    pref = [P, 300]
    row_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    total = int(row_off[-1])
    if quant is None:
        sc = ((1.0 + rng.permutation(total)) / total).astype(np.float32)
    elif quant == 0:
        sc = np.full(total, 0.25, dtype=np.float32)
    else:
        sc = (np.floor(rng.random(total) * quant) / quant).astype(np.float32)
    K = rng.integers(-4, 5, (total, d)).astype(np.float32)
    V = rng.integers(-4, 5, (total, d)).astype(np.float32)
    # (no donor reaches a threshold above 1: the roles alone decide every output)
    p = cask.Params(dtype=cask.BF16, head_dim=d, q_per_kv=1, window=Wn, budget=2048, sim_threshold=2.0)
    tb = lambda x: torch.from_numpy(x).to(torch.bfloat16)
    c = dict(K=tb(K), V=tb(V), Q=torch.zeros(2, Wn, 1, d, dtype=torch.bfloat16),
             row_off=torch.from_numpy(row_off), prefix_len=torch.tensor(pref, dtype=torch.int32))
    ro, plen, Kb, Vb, Qb = parity.host_arrays(c)
    want = ref.compress(parity.ref_params(p), ro, plen, Kb, Vb, Qb, scores=sc)
    out = cask.compress(parity.to_device(c, p), scores=torch.from_numpy(sc).cuda())
    torch.cuda.synchronize()
    got = parity.gpu_outputs(out, p)
    assert np.array_equal(got["status"], want["status"])
    assert np.array_equal(got["out_len"], want["out_len"])
    assert np.array_equal(got["out_src"], want["out_src"])
    assert np.array_equal(got["assign"], want["assign"])


# ------------------------------------------------------------------ determinism, errors, edges

@pytest.mark.parametrize("decode", [2500, 700])
def test_two_runs_are_bitwise_identical(decode):
    """Long units (general kernels) and short ones (one-launch scoring and tail, with many
    folds): every output of the event has the same bits on every run."""
    w = caches.scaled(W["cfg2"], n_layers=1, decode=decode)
    c = caches.make(w, seed=21)
    p = parity.params_of(w, sim_threshold=0.2)
    b = parity.to_device(c, p)
    a = parity.gpu_outputs(cask.compress(b), p)
    torch.cuda.synchronize()
    for _ in range(3):
        o = parity.gpu_outputs(cask.compress(b), p)
        for k in a:
            assert np.array_equal(a[k], o[k]), k


@pytest.mark.parametrize("kind", ["ties", "zeros", "identity", "long"])
def test_mass_diagnostics_edge_cases(kind):
    """rho_core / rho_rep (Section 2.6) with many rows tied at the rank-B score, with all-zero
    scores, in the identity regime, and on a unit longer than one radix chunk."""
    if kind == "identity":
        w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=2, prefix=40, decode=200, budget=384)
    elif kind == "long":
        w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=2, prefix=300, decode=20000, budget=512)
    else:
        w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=2, prefix=100, decode=1500, budget=256)
    c = caches.make(w, seed=13)
    p = parity.params_of(w, sim_threshold=0.3)
    rp = parity.ref_params(p)
    row_off, prefix_len, K, V, Q = parity.host_arrays(c)
    rng = np.random.default_rng(5)
    total = int(row_off[-1])
    if kind == "ties":
        s = (rng.integers(0, 6, total) / 8.0).astype(np.float32)      # six distinct values
    elif kind == "zeros":
        s = np.zeros(total, dtype=np.float32)
    else:
        s = (rng.random(total) ** 4).astype(np.float32)
    want = ref.compress(rp, row_off, prefix_len, K, V, Q, scores=s)
    want_rho = ref.mass_diagnostics(rp, row_off, s, want["role"], want["out_mass"], want["out_len"])
    b = parity.to_device(c, p)
    s_dev = torch.from_numpy(s).to(b.device)
    role, _ = cask.prefix_evict(b, s_dev)
    role, _ = cask.partition(b, s_dev, role)
    out = cask.compress(b, scores=s_dev)
    rho = cask.mass_diagnostics(b, s_dev, role, out.out_mass, out.out_len)
    torch.cuda.synchronize()
    assert np.array_equal(role.cpu().numpy(), want["role"])
    assert np.array_equal(out.out_len.cpu().numpy(), want["out_len"])
    # masses of merged rows depend on the assignment; compare rho_rep only where it agrees
    same = np.array_equal(out.assign.cpu().numpy(), want["assign"])
    got = rho.cpu().numpy()
    np.testing.assert_allclose(got[:, 0], want_rho[:, 0], rtol=2e-6)
    if same:
        np.testing.assert_allclose(got[:, 1], want_rho[:, 1], rtol=2e-6)
    if kind in ("zeros", "identity"):
        assert (got == 1.0).all()
    _note((kind, want_rho.tolist(), "assign equal" if same else "assign differs at near-ties"))


def test_decode_loop_events_with_count_carry():
    """Three events of a decode loop: each compresses B + delta rows back to B, decoded tokens
    are appended behind the output (row stride B + delta), and every cache row carries the
    number of original tokens it stands for.  Each event is compared with the oracle on the
    same state (the oracle's own output feeds the next event), so differences cannot pile up."""
    B, delta, G, d = 256, 128, 7, 128
    S = B + delta
    n_units = 3
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=n_units, prefix=90, decode=S - 90, budget=B)
    p = parity.params_of(w, sim_threshold=0.6)
    rp = parity.ref_params(p)
    first = caches.make(w, seed=21)
    ro, pl, K, V, Q = parity.host_arrays(first)
    K = K.reshape(n_units, S, d).copy()
    V = V.reshape(n_units, S, d).copy()
    cnt = np.ones((n_units, S), dtype=np.int32)
    plen = pl.copy()
    dev = torch.device("cuda:0")
    tau = float(np.float32(p.sim_threshold))
    folded_total = 0
    for ev in range(3):
        row_off = (np.arange(n_units + 1, dtype=np.int64) * S)
        want = ref.compress_step(rp, row_off, plen, K.reshape(-1, d), V.reshape(-1, d), Q,
                                 in_count=cnt.reshape(-1), out_stride_rows=S)
        _, best, second = ref.consolidate(rp, row_off, plen, K.reshape(-1, d), want["scores"], want["role"],
                                          want_sims=True)
        # the library on the same state, the oracle's scores injected
        dt = torch.bfloat16
        Kd = torch.from_numpy(K.view(np.int16)).view(dt).reshape(-1, d).to(dev)
        Vd = torch.from_numpy(V.view(np.int16)).view(dt).reshape(-1, d).to(dev)
        Qd = torch.from_numpy(Q.view(np.int16)).view(dt).to(dev)
        b = cask.Batch(p, torch.from_numpy(row_off), torch.from_numpy(plen), Kd, Vd, Qd)
        out = cask.Outputs(b)
        Ko = torch.zeros(n_units, S, d, dtype=dt, device=dev)
        Vo = torch.zeros_like(Ko)
        oc = torch.zeros(n_units, B, dtype=torch.int32, device=dev)
        cd = torch.from_numpy(cnt.reshape(-1)).to(dev)
        cask.compress_step(b, Ko, Vo, out, in_count=cd, out_count=oc,
                           scores=torch.from_numpy(want["scores"]).to(dev))
        torch.cuda.synchronize()
        got = dict(K_out=caches.host_bits(Ko)[:, :B], V_out=caches.host_bits(Vo)[:, :B],
                   out_len=out.out_len.cpu().numpy(), out_src=out.out_src.cpu().numpy(),
                   out_mass=out.out_mass.cpu().numpy(), assign=out.assign.cpu().numpy(),
                   status=out.status.cpu().numpy())
        wv = dict(want)
        wv["K_out"], wv["V_out"] = want["K_out"][:, :B], want["V_out"][:, :B]
        assert np.array_equal(got["out_len"], want["out_len"]) and (got["out_len"] == B).all()
        assert np.array_equal(got["out_src"], want["out_src"])
        n_bad = 0
        for u in range(n_units):
            sl = slice(row_off[u], row_off[u + 1])
            n_bad += parity.check_assign_excused(got["assign"][sl], want["assign"][sl], best[sl], second[sl],
                                                 tau, f"event {ev} unit {u}")
        if n_bad == 0:
            assert np.array_equal(got["status"], want["status"])
            assert np.array_equal(oc.cpu().numpy(), want["out_count"])
        folded_total += parity.check_values(p, got, wv, K.reshape(-1, d), V.reshape(-1, d), row_off)
        assert not caches.host_bits(Ko)[:, B:].any()            # rows behind the output stay untouched
        # own scores once per event: within the score tolerance
        s_own = cask.score(b)
        torch.cuda.synchronize()
        parity.check_scores(s_own.cpu().numpy(), want["scores"], row_off)
        # next state: the oracle's output, then delta freshly decoded tokens with count 1
        nxt = caches.make(w, seed=100 + ev)
        _, _, Kn, Vn, Qn = parity.host_arrays(nxt)
        Kn, Vn = Kn.reshape(n_units, S, d), Vn.reshape(n_units, S, d)
        K = np.concatenate([want["K_out"][:, :B], Kn[:, S - delta:]], axis=1).copy()
        V = np.concatenate([want["V_out"][:, :B], Vn[:, S - delta:]], axis=1).copy()
        cnt = np.concatenate([want["out_count"], np.ones((n_units, delta), dtype=np.int32)], axis=1)
        Q = Qn
        plen = np.array([ref.plan(rp, int(plen[u]), S)["p_keep"] for u in range(n_units)], dtype=np.int32)
    assert folded_total > 0
    assert int(cnt.max()) > 1          # some representative stands for several tokens by now
    _note(("decode loop", "folded rows", folded_total, "largest count", int(cnt.max()), "prefix", plen.tolist()))


def test_step_zero_mass_groups_average_by_token_count():
    """All scores zero: every fold is the count-weighted mean of its members."""
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=2, prefix=40, decode=1300, budget=200)
    p = parity.params_of(w, sim_threshold=-1.0)        # every donor folds
    rp = parity.ref_params(p)
    c = caches.make(w, seed=23)
    row_off, plen, K, V, Q = parity.host_arrays(c)
    total = int(row_off[-1])
    rng = np.random.default_rng(8)
    cnt = rng.integers(1, 20, total).astype(np.int32)
    s = np.zeros(total, dtype=np.float32)
    want = ref.compress_step(rp, row_off, plen, K, V, Q, in_count=cnt, scores=s)
    b = parity.to_device(c, p)
    out = cask.Outputs(b)
    Ko = torch.zeros(b.n_units, p.budget, p.head_dim, dtype=torch.bfloat16, device=b.device)
    Vo = torch.zeros_like(Ko)
    oc = torch.zeros(b.n_units, p.budget, dtype=torch.int32, device=b.device)
    cask.compress_step(b, Ko, Vo, out, in_count=torch.from_numpy(cnt).to(b.device), out_count=oc,
                       scores=torch.from_numpy(s).to(b.device))
    torch.cuda.synchronize()
    got = dict(K_out=caches.host_bits(Ko), V_out=caches.host_bits(Vo), out_len=out.out_len.cpu().numpy(),
               out_src=out.out_src.cpu().numpy(), out_mass=out.out_mass.cpu().numpy(),
               assign=out.assign.cpu().numpy())
    assert np.array_equal(got["out_src"], want["out_src"])
    d = p.head_dim
    folded = parity.check_values(p, got, want, K.reshape(-1, d), V.reshape(-1, d), row_off)
    assert folded >= 10
    if np.array_equal(got["assign"], want["assign"]):
        assert np.array_equal(oc.cpu().numpy(), want["out_count"])
    _note(("zero-mass folds", folded))


def test_step_with_dedup_seeding_counts_and_row_stride():
    """A decode-loop step (token counts in, counts out, output row stride beyond the budget)
    with de-duplicated seeding, on injected scores: source rows, folded values and counts
    against the oracle's step."""
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=3, prefix=70, decode=1700, budget=320, cluster_frac=0.6)
    c = caches.make(w, seed=29)
    row_off, plen, K, V, Q = parity.host_arrays(c)
    total, S = int(row_off[-1]), 448
    rng = np.random.default_rng(12)
    cnt = rng.integers(1, 6, total).astype(np.int32)
    for dt in (0.0, 0.013, -0.017, 0.031, -0.029, 0.047):
        p = parity.params_of(w, sim_threshold=0.8 + dt, seed_dedup=4)
        rp = parity.ref_params(p)
        s = ref.score(rp, row_off, K, Q)
        role0, _ = ref.prefix_evict(rp, row_off, plen, s)
        if ref.partition_keys(rp, row_off, plen, K, s, role0)[2].min() >= 1e-3:
            break
    else:
        pytest.fail("no clear threshold for this cache")
    want = ref.compress_step(rp, row_off, plen, K, V, Q, in_count=cnt, scores=s, out_stride_rows=S)
    b = parity.to_device(c, p)
    out = cask.Outputs(b)
    Ko = torch.zeros(b.n_units, S, p.head_dim, dtype=torch.bfloat16, device=b.device)
    Vo = torch.zeros_like(Ko)
    oc = torch.zeros(b.n_units, p.budget, dtype=torch.int32, device=b.device)
    cask.compress_step(b, Ko, Vo, out, in_count=torch.from_numpy(cnt).to(b.device), out_count=oc,
                       scores=torch.from_numpy(s).to(b.device))
    torch.cuda.synchronize()
    got = dict(K_out=caches.host_bits(Ko), V_out=caches.host_bits(Vo), out_len=out.out_len.cpu().numpy(),
               out_src=out.out_src.cpu().numpy(), out_mass=out.out_mass.cpu().numpy(),
               assign=out.assign.cpu().numpy())
    assert np.array_equal(got["out_len"], want["out_len"]) and np.array_equal(got["out_src"], want["out_src"])
    d = p.head_dim
    folded = parity.check_values(p, got, want, K.reshape(-1, d), V.reshape(-1, d), row_off)
    assert folded >= 5
    if np.array_equal(got["assign"], want["assign"]):
        assert np.array_equal(oc.cpu().numpy(), want["out_count"])
        assert int(want["out_count"].max()) > int(cnt.max())      # counts of folded rows add up
    _note(("dedup step", "folded rows", folded, "largest count", int(want["out_count"].max())))


def test_compress_replays_from_a_hip_graph():
    """The whole event is plain kernel launches on the caller's stream (no allocation, no
    synchronisation, no memset): it can be captured once and replayed; every replay must equal
    the eager result, with eager work in between."""
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=3, decode=2100)
    c = caches.make(w, seed=9)
    p = parity.params_of(w, sim_threshold=0.5)
    b = parity.to_device(c, p)
    eager = cask.compress(b)
    torch.cuda.synchronize()
    want = {k: getattr(eager, k).clone() for k in ("K_out", "V_out", "out_src", "out_len", "out_mass", "assign", "status", "scores")}
    out = cask.Outputs(b)
    b.workspace()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        cask.compress(b, out)          # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        cask.compress(b, out)
    for rep in range(3):
        for t in (out.K_out, out.V_out, out.out_mass, out.scores):
            t.zero_()
        out.out_src.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        L = want["out_len"]
        assert torch.equal(out.out_len, L) and torch.equal(out.status, want["status"])
        assert torch.equal(out.assign, want["assign"]) and torch.equal(out.scores, want["scores"])
        for u in range(b.n_units):
            n = int(L[u])
            assert torch.equal(out.out_src[u, :n], want["out_src"][u, :n])
            assert torch.equal(out.K_out[u, :n], want["K_out"][u, :n])
            assert torch.equal(out.V_out[u, :n], want["V_out"][u, :n])
            assert torch.equal(out.out_mass[u, :n], want["out_mass"][u, :n])
        cask.score(b)                  # eager work between the replays
        torch.cuda.synchronize()
    _note("graph replays equal the eager event")


def test_step_with_dedup_and_attention_replay_from_a_hip_graph():
    """A decode-loop step with de-duplicated seeding (three selection launches) followed by the
    consumer's attention over its output, captured as one graph: every replay equals eager."""
    dev = torch.device("cuda:0")
    w = caches.scaled(W["cfg2"], n_layers=1, n_kv_heads=3, prefix=80, decode=1900, budget=384, cluster_frac=0.5)
    c = caches.make(w, seed=19)
    p = parity.params_of(w, sim_threshold=0.8, seed_dedup=4)
    b = parity.to_device(c, p)
    S = 512
    q = torch.randn(b.n_units, w.q_per_kv, w.head_dim, generator=torch.Generator().manual_seed(2)).to(torch.bfloat16).to(dev)

    def run(out, Ko, Vo, oc, att):
        cask.compress_step(b, Ko, Vo, out, out_count=oc)
        cask.attend(p, q, Ko, Vo, out.out_len, count=oc, out=att)

    def fresh():
        Ko = torch.zeros(b.n_units, S, w.head_dim, dtype=torch.bfloat16, device=dev)
        return (cask.Outputs(b), Ko, torch.zeros_like(Ko),
                torch.zeros(b.n_units, p.budget, dtype=torch.int32, device=dev), torch.empty_like(q))

    eager = fresh()
    run(*eager)
    torch.cuda.synchronize()
    assert int(eager[3].max()) > 1                      # something folded
    cap = fresh()
    b.workspace()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(*cap)                                       # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run(*cap)
    for rep in range(3):
        for t in (cap[1], cap[2], cap[4]):
            t.zero_()
        cap[3].zero_()
        cap[0].out_src.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(cap[0].out_len, eager[0].out_len) and torch.equal(cap[0].status, eager[0].status)
        assert torch.equal(cap[0].assign, eager[0].assign)
        for u in range(b.n_units):
            n = int(eager[0].out_len[u])
            assert torch.equal(cap[0].out_src[u, :n], eager[0].out_src[u, :n])
            assert torch.equal(cap[1][u, :n], eager[1][u, :n]) and torch.equal(cap[2][u, :n], eager[2][u, :n])
            assert torch.equal(cap[3][u, :n], eager[3][u, :n])
        assert torch.equal(cap[4], eager[4])
        cask.score(b)                                   # eager work between the replays
        torch.cuda.synchronize()


def test_argument_errors_and_empty_batch():
    dev = torch.device("cuda:0")
    p = cask.Params(dtype=cask.BF16, head_dim=128, q_per_kv=2, window=16, budget=64)
    K = torch.zeros(100, 128, dtype=torch.bfloat16, device=dev)
    Q = torch.zeros(1, 16, 2, 128, dtype=torch.bfloat16, device=dev)
    ok = cask.Batch(p, torch.tensor([0, 100]), torch.tensor([10], dtype=torch.int32), K, K, Q)
    cask.compress(ok)
    torch.cuda.synchronize()

    def expect(code, fn):
        with pytest.raises(cask.CaskError) as e:
            fn()
        assert e.value.code == code

    Kodd = torch.zeros(100 * 128 + 8, dtype=torch.bfloat16, device=dev)[1:1 + 100 * 128].view(100, 128)
    mis = cask.Batch(p, torch.tensor([0, 100]), torch.tensor([10], dtype=torch.int32), Kodd, K, Q)
    expect(cask.binding.EINVAL, lambda: cask.compress(mis))              # K not 16-byte aligned
    short = cask.Batch(p, torch.tensor([0, 10]), torch.tensor([0], dtype=torch.int32), K, K, Q)
    expect(cask.binding.EINVAL, lambda: cask.compress(short))            # N < W
    badp = cask.Batch(p, torch.tensor([0, 100]), torch.tensor([101], dtype=torch.int32), K, K, Q)
    expect(cask.binding.EINVAL, lambda: cask.score(badp))                 # P > N
    for bad in (dataclasses.replace(p, budget=16), dataclasses.replace(p, head_dim=96),
                dataclasses.replace(p, dtype=5), dataclasses.replace(p, window=0)):
        bb = cask.Batch(dataclasses.replace(p), torch.tensor([0, 100]), torch.tensor([10], dtype=torch.int32), K, K, Q)
        bb.params = bad
        bb._ws = torch.empty(1 << 20, dtype=torch.uint8, device=dev)
        expect(cask.binding.EINVAL, lambda: cask.compress(bb))
    small = cask.Batch(p, torch.tensor([0, 100]), torch.tensor([10], dtype=torch.int32), K, K, Q)
    small._ws = torch.empty(256, dtype=torch.uint8, device=dev)
    expect(cask.binding.ENOMEM, lambda: cask.compress(small))
    expect(cask.binding.ENOMEM, lambda: cask.score(small))
    empty = cask.Batch(p, torch.tensor([0]), torch.zeros(0, dtype=torch.int32), K, K, Q)
    out = cask.compress(empty)
    torch.cuda.synchronize()
    assert out.out_len.numel() == 0


def test_probe_loops_run_and_report_sane_figures():
    """The measurement aids: the copy probe copies (whole buffer, odd multiple of 16 bytes), the
    read probe and the issue probes run, and their figures are in a sane range for the part."""
    dev = torch.device("cuda:0")
    lib = cask.load()
    n = (1 << 20) * 16 + 48
    src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 256)
    dst = torch.zeros_like(src)
    st = torch.cuda.current_stream().cuda_stream
    assert lib.cask_probe_copy(src.data_ptr(), dst.data_ptr(), n, st) == 0
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    assert lib.cask_probe_copy(src.data_ptr(), dst.data_ptr(), n - 8, st) == cask.binding.EINVAL   # not a multiple of 16
    assert lib.cask_probe_copy(None, dst.data_ptr(), n, st) == cask.binding.EINVAL
    r = cask.binding.probe_read(1 << 28, blocks=512, reps=2)
    assert 500.0 < r["gbs"] < 8000.0, r
    for kind in (0, 1, 2, 3, 4):
        p = cask.binding.probe_issue(kind, waves_per_simd=2, blocks=256, iters=500)
        assert 0.8 < p["ghz"] < 2.6 and 25.0 < p["cycles_per_unit"] < 120.0, (kind, p)
        if kind != 2:
            assert 200.0 < p["tflops"] < 2500.0, (kind, p)
    assert lib.cask_probe_issue(7, 2, 256, 10, src.data_ptr(), dst.data_ptr(), dst.data_ptr(), st) == cask.binding.EINVAL


# ------------------------------------------------------------------ full benchmark sizes

def _full_size(name, sample_units, seed=caches.BASE_SEED, layers=None):
    """Whole workload on the GPU in the benchmark's launch configuration; the oracle runs on a
    sample of units (each regenerated bit-identically on the host is not needed: the sampled
    rows are copied back)."""
    w = W[name]
    dev = torch.device("cuda:0")
    c = caches.make(w, seed=seed, device=dev, layers=layers)
    p = parity.params_of(w)
    b = cask.Batch(p, c["row_off"], c["prefix_len"], c["K"], c["V"], c["Q"])
    out = cask.compress(b)
    torch.cuda.synchronize()
    got = parity.gpu_outputs(out, p)
    ro = b.row_off_host.numpy()
    n_units = b.n_units
    if callable(sample_units):
        sample_units = sample_units(ro)
    # properties that hold at any size
    sums = np.add.reduceat(got["scores"].astype(np.float64), ro[:-1])
    np.testing.assert_allclose(sums, 1.0, atol=2e-5)
    for u in range(n_units):
        N = int(ro[u + 1] - ro[u])
        pl = cask.plan(p, int(b.prefix_len_host[u]), N)
        L = int(got["out_len"][u])
        assert L == min(N, p.budget)
        src = got["out_src"][u, :L]
        assert (np.diff(src) > 0).all() and src[0] >= 0 and src[-1] == N - 1
        assert (got["status"][u] & ~cask.binding.ST_MERGE_INACTIVE) == (pl["status"] & ~cask.binding.ST_MERGE_INACTIVE)
        assert (src < int(b.prefix_len_host[u])).sum() == pl["p_keep"]
    # sampled units against the oracle, as a sub-batch with the same bits; a unit whose event
    # folded donors joins the sample, so that fold rows of this launch are compared as well
    folding = [u for u in range(n_units) if got["status"][u] == cask.binding.ST_ACTIVE]
    sample_units = list(sample_units)
    if folding and not set(folding) & set(sample_units):
        sample_units.append(folding[len(folding) // 2])
    folded_rows = 0
    for u in sample_units:
        sl = slice(int(ro[u]), int(ro[u + 1]))
        sub = dict(K=c["K"][sl].cpu(), V=c["V"][sl].cpu(), Q=c["Q"][u:u + 1].cpu(),
                   row_off=torch.tensor([0, sl.stop - sl.start], dtype=torch.int64),
                   prefix_len=b.prefix_len_host[u:u + 1].clone())
        rp = parity.ref_params(p)
        row_off, prefix_len, K, V, Q = parity.host_arrays(sub)
        want = ref.compress(rp, row_off, prefix_len, K, V, Q)
        parity.check_scores(got["scores"][sl], want["scores"], row_off)
        L = int(want["out_len"][0])
        flips = parity.check_keepset_near_ties(rp, int(prefix_len[0]), want["scores"], got["out_src"][u, :L],
                                               want["out_src"][0, :L], f"{name} unit {u}")
        # the rows this launch wrote for the unit: kept rows bit for bit, folds to the tolerance
        got_u = {k: got[k][u:u + 1] for k in ("K_out", "V_out", "out_len", "out_src", "out_mass", "status")}
        got_u["assign"], got_u["scores"] = got["assign"][sl], got["scores"][sl]
        d = p.head_dim
        n_f = parity.check_values(p, got_u, want, K.reshape(-1, d), V.reshape(-1, d), row_off, own_scores=True)
        folded_rows += n_f
        if flips == 0:
            bad = parity.check_assign_near_ties(rp, row_off, prefix_len, K, want, got_u["assign"], f"{name} unit {u}")
            if bad == 0:
                assert got["status"][u] == want["status"][0]
        _note(f"{name} unit {u}: full-size launch: {n_f} fold rows compared, {flips} near-tie flips; "
              f"as a batch of its own: {parity.full_check(sub, p)}")
    if folding:
        assert folded_rows > 0, "no fold row of the full-size launch was compared"
    return got


def test_cfg2_full_size_sampled_units():
    _full_size("cfg2", [0, 37, 111])


def test_cfg3_full_size_sampled_units():
    _full_size("cfg3", [5])


def test_cfg4_full_size_sampled_units():
    _full_size("cfg4", [1, 60])


def test_cfg5_ragged_many_units_sampled():
    """Eight of cfg5's 32 layers (4096 ragged units of 4.6k - 33k rows, G = 4): the many-units
    launch configuration (one key split, thousands of workgroups per sweep); the oracle runs
    on the shortest unit, on one of median length and on the longest, and on one whose event
    folded donors."""
    def pick(ro):
        lens = ro[1:] - ro[:-1]
        order = np.argsort(lens, kind="stable")
        return [int(order[0]), int(order[len(order) // 2]), int(order[-1])]
    _full_size("cfg5", pick, layers=range(8))


def test_cfg4v_full_size_exhausted():
    w = W["cfg4v"]
    dev = torch.device("cuda:0")
    c = caches.make(w, device=dev, layers=range(4))
    p = parity.params_of(w)
    b = cask.Batch(p, c["row_off"], c["prefix_len"], c["K"], c["V"], c["Q"])
    out = cask.compress(b)
    torch.cuda.synchronize()
    got = parity.gpu_outputs(out, p)
    assert (got["status"] == cask.binding.ST_PREFIX_BUDGET_EXHAUSTED).all()
    assert (got["out_len"] == 1024).all()
    ro = b.row_off_host.numpy()
    u = 3
    sl = slice(int(ro[u]), int(ro[u + 1]))
    sub = dict(K=c["K"][sl].cpu(), V=c["V"][sl].cpu(), Q=c["Q"][u:u + 1].cpu(),
               row_off=torch.tensor([0, sl.stop - sl.start], dtype=torch.int64),
               prefix_len=b.prefix_len_host[u:u + 1].clone())
    _note(parity.full_check(sub, p))
