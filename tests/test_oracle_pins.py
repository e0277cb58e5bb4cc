"""Pins for the CPU oracle: closed forms, library routines, brute force and invariants.

Each test anchors one rule of the oracle to something other than the oracle itself, so that
a dropped term, a wrong sign or index, or a transposed operand fails at least one of them.
"""
import itertools
import os

import numpy as np
import pytest
import torch
from scipy.special import softmax as scipy_softmax

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ helpers

def f32_params(ref, **kw):
    base = dict(dtype=ref.F32, head_dim=16, q_per_kv=1, window=4, recent=-1, budget=32, core=-1,
                prefix_budget=-1, sim_threshold=0.9, softmax_scale=0.0, causal=1)
    base.update(kw)
    return ref.Params(**base)


def rand_unit(rng, N, d, W, G, n_units=1):
    K = rng.standard_normal((n_units * N, d)).astype(np.float32)
    V = rng.standard_normal((n_units * N, d)).astype(np.float32)
    Q = rng.standard_normal((n_units, W, G, d)).astype(np.float32)
    row_off = np.arange(n_units + 1, dtype=np.int64) * N
    return K, V, Q, row_off


def to_bf16_bits(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16) \
        .view(torch.int16).numpy().view(np.uint16)


def from_bf16_bits(b):
    return torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()


# ------------------------------------------------------------------ bf16 rounding

def test_bf16_rounding_matches_library(oracle):
    rng = np.random.default_rng(1)
    xs = np.concatenate([
        rng.standard_normal(2000).astype(np.float32) * 10.0,
        rng.standard_normal(200).astype(np.float32) * 1e-39,   # bf16 subnormals
        np.array([0.0, -0.0, 1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -7,
                  3.3895e38, -3.3895e38, 65504.0, 2.0 ** -133, 2.0 ** -134, 1.5 * 2.0 ** -133],
                 dtype=np.float32)])
    want = to_bf16_bits(xs)   # torch rounds float -> bfloat16 to nearest even
    got = np.array([oracle.bf16_from_double(float(x)) for x in xs], dtype=np.uint16)
    np.testing.assert_array_equal(got, want)
    # ties that exist only in double: halfway between two bf16 neighbours plus/minus a hair
    lo, hi = 1.0, 1.0 + 2.0 ** -7
    mid = 0.5 * (lo + hi)
    assert oracle.bf16_from_double(mid) == to_bf16_bits([lo])[0]              # tie -> even
    assert oracle.bf16_from_double(mid + 2.0 ** -40) == to_bf16_bits([hi])[0]
    assert oracle.bf16_from_double(mid - 2.0 ** -40) == to_bf16_bits([lo])[0]
    # round trip
    for h in [0x3F80, 0x4049, 0xC2F7, 0x0001, 0x8001, 0x7F7F]:
        assert oracle.bf16_from_double(oracle.bf16_to_double(h)) == h


# ------------------------------------------------------------------ R1 score

def test_score_sums_to_one(oracle):
    rng = np.random.default_rng(2)
    for causal in (0, 1):
        for (N, d, W, G) in [(37, 16, 5, 3), (64, 64, 32, 1), (9, 8, 9, 2)]:
            K, _, Q, ro = rand_unit(rng, N, d, W, G, n_units=3)
            p = f32_params(oracle, head_dim=d, window=W, q_per_kv=G, causal=causal)
            s = oracle.score(p, ro, K, Q)
            np.testing.assert_allclose(s.reshape(3, N).sum(1), 1.0, rtol=0, atol=2e-6)
            assert (s >= 0).all()


def test_score_single_row_is_library_softmax(oracle):
    rng = np.random.default_rng(3)
    N, d = 50, 24
    K, _, Q, ro = rand_unit(rng, N, d, 1, 1)
    for scale in (0.0, 0.37):
        p = f32_params(oracle, head_dim=d, window=1, q_per_kv=1, softmax_scale=scale)
        s = oracle.score(p, ro, K, Q)
        c = scale if scale > 0 else 1.0 / np.sqrt(d)
        want = scipy_softmax(np.float32(c).astype(np.float64) * (K.astype(np.float64) @ Q[0, 0, 0].astype(np.float64)))
        np.testing.assert_allclose(s, want.astype(np.float32), rtol=2e-7, atol=0)


def test_score_rows_decompose_into_library_softmax(oracle):
    """Row (w, g) sits at slot N-W+w and sees keys up to its own slot; the score is the mean
    of the rows' probabilities.  Each row is recomputed with scipy on the truncated key set."""
    rng = np.random.default_rng(4)
    N, d, W, G = 23, 12, 6, 3
    K, _, Q, ro = rand_unit(rng, N, d, W, G, n_units=2)
    for causal in (1, 0):
        p = f32_params(oracle, head_dim=d, window=W, q_per_kv=G, causal=causal)
        s = oracle.score(p, ro, K, Q).reshape(2, N)
        for u in range(2):
            Ku = K[u * N:(u + 1) * N].astype(np.float64)
            acc = np.zeros(N)
            for w in range(W):
                last = N - W + w if causal else N - 1
                for g in range(G):
                    logits = (Ku[: last + 1] @ Q[u, w, g].astype(np.float64)) / np.sqrt(d)
                    acc[: last + 1] += scipy_softmax(logits)
            np.testing.assert_allclose(s[u], (acc / (W * G)).astype(np.float32), rtol=3e-7, atol=1e-12)


def test_score_identical_keys_closed_form(oracle):
    """All keys equal => every visible key gets 1/(t_w+1): s_j = (1/W) sum_w [j<=t_w]/(t_w+1)."""
    N, d, W, G = 20, 8, 5, 2
    rng = np.random.default_rng(5)
    K = np.tile(rng.standard_normal((1, d)).astype(np.float32), (N, 1))
    Q = rng.standard_normal((1, W, G, d)).astype(np.float32)
    p = f32_params(oracle, head_dim=d, window=W, q_per_kv=G)
    s = oracle.score(p, np.array([0, N]), K, Q)
    want = np.zeros(N)
    for w in range(W):
        t = N - W + w
        want[: t + 1] += 1.0 / (t + 1)
    want /= W
    np.testing.assert_allclose(s, want.astype(np.float32), rtol=3e-7)


def test_score_log_integer_logits_closed_form(oracle):
    """Logits ln(1), ln(2), ..., ln(N) => probabilities j / (N(N+1)/2)."""
    N, d = 12, 4
    scale = 0.5
    K = np.zeros((N, d), dtype=np.float32)
    K[:, 1] = np.log(np.arange(1, N + 1)) / scale / 2.0
    Q = np.zeros((1, 1, 1, d), dtype=np.float32)
    Q[0, 0, 0, 1] = 2.0
    Q[0, 0, 0, 0] = 5.0   # orthogonal to every key: must not matter
    p = f32_params(oracle, head_dim=d, window=1, q_per_kv=1, softmax_scale=scale)
    s = oracle.score(p, np.array([0, N]), K, Q)
    want = np.arange(1, N + 1) / (N * (N + 1) / 2)
    np.testing.assert_allclose(s, want, rtol=2e-6)


def test_score_bf16_inputs_are_read_exactly(oracle):
    rng = np.random.default_rng(6)
    N, d, W, G = 40, 16, 4, 2
    K, _, Q, ro = rand_unit(rng, N, d, W, G)
    Kb, Qb = to_bf16_bits(K), to_bf16_bits(Q)
    pb = f32_params(oracle, dtype=oracle.BF16, head_dim=d, window=W, q_per_kv=G)
    pf = f32_params(oracle, head_dim=d, window=W, q_per_kv=G)
    s_b = oracle.score(pb, ro, Kb, Qb)
    s_f = oracle.score(pf, ro, from_bf16_bits(Kb).astype(np.float32).reshape(N, d),
                       from_bf16_bits(Qb).astype(np.float32).reshape(1, W, G, d))
    np.testing.assert_array_equal(s_b, s_f)


# ------------------------------------------------------------------ R2 order, R5 prefix

def test_topk_maximises_score_sum_bruteforce(oracle):
    rng = np.random.default_rng(7)
    for trial in range(6):
        P = 10
        N = P + 8
        s = rng.random(N).astype(np.float32)
        if trial % 2:
            s[:P] = np.round(s[:P] * 4) / 4     # many ties
        for bp in (1, 3, 5):
            # budget chosen so that P_keep = bp: decode (8 tokens, recent 4) never fills the room
            p = f32_params(oracle, window=4, recent=4, budget=16, prefix_budget=bp)
            pl = oracle.plan(p, P, N)
            k = pl["p_keep"]
            role, _ = oracle.prefix_evict(p, np.array([0, N]), np.array([P]), s)
            keep = np.flatnonzero(role[:P] == oracle.PREFIX_KEEP)
            assert len(keep) == k
            best = max(float(np.sum(s[list(c)].astype(np.float64)))
                       for c in itertools.combinations(range(P), k))
            assert float(np.sum(s[keep].astype(np.float64))) == pytest.approx(best, rel=0, abs=1e-12)
            # among equal scores the lower index is preferred: the kept set is the
            # lexicographically smallest maximiser
            order = np.lexsort((np.arange(P), -s[:P].astype(np.float64)))
            np.testing.assert_array_equal(np.sort(order[:k]), keep)


def test_constant_scores_keep_lowest_indices(oracle):
    P, D = 40, 30
    N = P + D
    s = np.full(N, 0.125, dtype=np.float32)
    p = f32_params(oracle, window=4, recent=6, budget=30, prefix_budget=10, core=8)
    pl = oracle.plan(p, P, N)
    assert (pl["p_keep"], pl["slots"], pl["core"], pl["seeds"]) == (10, 14, 8, 6)
    role, _ = oracle.prefix_evict(p, np.array([0, N]), np.array([P]), s)
    role, _ = oracle.partition(p, np.array([0, N]), np.array([P]), s, role)
    assert (role[:10] == oracle.PREFIX_KEEP).all() and (role[10:P] == oracle.PREFIX_DROP).all()
    assert (role[P:P + 8] == oracle.CORE).all()
    assert (role[P + 8:P + 14] == oracle.SEED).all()
    assert (role[P + 14:N - 6] == oracle.DONOR).all()
    assert (role[N - 6:] == oracle.RECENT).all()


def test_prefix_and_partition_match_library_sort(oracle):
    rng = np.random.default_rng(8)
    P, D = 300, 500
    N = P + D
    s = (rng.random(2 * N) ** 4).astype(np.float32)
    s[rng.integers(0, 2 * N, 200)] = s[0]       # planted ties
    ro = np.array([0, N, 2 * N])
    p = f32_params(oracle, window=16, recent=20, budget=200)
    pl = oracle.plan(p, P, N)
    role, st = oracle.prefix_evict(p, ro, np.array([P, P]), s)
    role, st = oracle.partition(p, ro, np.array([P, P]), s, role)
    for u in range(2):
        su = s[u * N:(u + 1) * N].astype(np.float64)
        ru = role[u * N:(u + 1) * N]
        order = np.lexsort((np.arange(P), -su[:P]))
        want = np.full(P, oracle.PREFIX_DROP)
        want[order[: pl["p_keep"]]] = oracle.PREFIX_KEEP
        np.testing.assert_array_equal(ru[:P], want)
        hi = N - pl["r_eff"]
        order = P + np.lexsort((np.arange(hi - P), -su[P:hi]))
        want = np.full(N - P, oracle.DONOR)
        want[order[: pl["core"]] - P] = oracle.CORE
        want[order[pl["core"]: pl["core"] + pl["seeds"]] - P] = oracle.SEED
        want[hi - P:] = oracle.RECENT
        np.testing.assert_array_equal(ru[P:], want)


# ------------------------------------------------------------------ R4 plan

def test_plan_golden_table(oracle):
    rows = 0
    with open(os.path.join(GOLDEN, "plan_table.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            lhs, rhs = line.split("|")
            P, D, B, R, core, *pb = (int(x) for x in lhs.split())
            r_eff, p_keep, slots, c, m, status = (int(x) for x in rhs.split())
            p = f32_params(oracle, window=min(128, P + D), recent=R, budget=B, core=core,
                           prefix_budget=pb[0] if pb else -1)
            got = oracle.plan(p, P, P + D)
            assert got == dict(r_eff=r_eff, p_keep=p_keep, slots=slots, core=c, seeds=m,
                               status=status), (line, got)
            rows += 1
    assert rows >= 18


def test_plan_fills_budget_exactly(oracle):
    """|R| <= B (Section 2.3) holds with equality whenever N > B: kept prefix + decode slots
    actually usable + recent tail == min(N, B)."""
    rng = np.random.default_rng(9)
    for _ in range(3000):
        R = int(rng.integers(0, 40))
        B = int(rng.integers(R + 1, 300))
        P = int(rng.integers(0, 2000))
        D = int(rng.integers(0, 2000))
        N = P + D
        if N < 1:
            continue
        p = f32_params(oracle, window=1, recent=R, budget=B,
                       core=int(rng.integers(-1, 50)), prefix_budget=int(rng.integers(-1, 200)))
        pl = oracle.plan(p, P, N)
        dnr = D - pl["r_eff"]
        used = pl["p_keep"] + min(dnr, pl["slots"]) + pl["r_eff"]
        assert used == min(N, B)
        assert 0 <= pl["p_keep"] <= P and pl["core"] + pl["seeds"] == min(pl["slots"], max(dnr, 0)) \
            or pl["status"] & (oracle.ST_IDENTITY | oracle.ST_MERGE_INACTIVE)
        assert pl["core"] >= 0 and pl["seeds"] >= 0 and pl["core"] + pl["seeds"] <= max(pl["slots"], 0)
        if pl["status"] & oracle.ST_PREFIX_BUDGET_EXHAUSTED:
            assert pl["slots"] == 0 and dnr > 0 and pl["p_keep"] == B - pl["r_eff"]


def test_plan_properties_of_the_split_rule(oracle):
    """What the budget-split rule fixes, stated as properties and checked over random sizes with
    the prefix budget, core size and recent tail drawn as well (two-stage compression, Section
    2.2; |R| <= B, Section 2.3; the exhausted regime, Section 5.2):
      - a closed form of the kept prefix written here from the rule's text:
        min(P, B - r, max(B_p, B - r - Dnr));
      - r_eff + p_keep + slots == B whenever N > B;
      - exhausted  <=>  N > B, no slot, and decode tokens outside the recent tail waiting;
      - a larger budget never keeps fewer prefix tokens or offers fewer slots;
      - a longer decode trace never keeps more prefix tokens."""
    rng = np.random.default_rng(77)
    for _ in range(3000):
        R = int(rng.integers(0, 150))
        B = int(rng.integers(R + 1, 1200))
        P = int(rng.integers(0, 70000)) if rng.integers(0, 2) else int(rng.integers(0, 600))
        D = int(rng.integers(0, 5000))
        if P + D == 0:
            continue
        kw = dict(window=1, recent=R, core=int(rng.integers(-1, 300)), prefix_budget=int(rng.integers(-1, 900)))
        pl = oracle.plan(f32_params(oracle, budget=B, **kw), P, P + D)
        r = min(R, D)
        dnr = D - r
        assert pl["r_eff"] == r
        if P + D <= B:
            assert pl["status"] == oracle.ST_IDENTITY and pl["p_keep"] == P and pl["core"] == dnr
            continue
        bp = kw["prefix_budget"] if kw["prefix_budget"] >= 0 else max(B // 4, -(-P // 64))
        assert pl["p_keep"] == min(P, B - r, max(bp, B - r - dnr)), (kw, P, D, B, pl)
        assert pl["r_eff"] + pl["p_keep"] + pl["slots"] == B
        exhausted = pl["slots"] == 0 and dnr > 0
        assert bool(pl["status"] & oracle.ST_PREFIX_BUDGET_EXHAUSTED) == exhausted
        if exhausted:
            assert pl["core"] == 0 and pl["seeds"] == 0
        elif dnr <= pl["slots"]:
            assert pl["status"] == oracle.ST_MERGE_INACTIVE and pl["core"] == dnr and pl["seeds"] == 0
        else:
            want_core = min(kw["core"], pl["slots"]) if kw["core"] >= 0 else (4 * pl["slots"]) // 5
            assert (pl["core"], pl["seeds"]) == (want_core, pl["slots"] - want_core)
            assert pl["status"] == (oracle.ST_ACTIVE if pl["seeds"] > 0 else oracle.ST_MERGE_INACTIVE)
        # monotone in the budget (explicit prefix budget: the default one grows with B as well)
        big = oracle.plan(f32_params(oracle, budget=B + int(rng.integers(1, 200)), **kw), P, P + D)
        if not big["status"] & oracle.ST_IDENTITY:
            assert big["p_keep"] >= pl["p_keep"] and big["slots"] >= pl["slots"]
        longer = oracle.plan(f32_params(oracle, budget=B, **kw), P, P + D + int(rng.integers(1, 500)))
        assert longer["p_keep"] <= pl["p_keep"] or R > D   # (a tail still growing into R shrinks the room)


# ------------------------------------------------------------------ R6 consolidate

def make_case(rng, oracle, P=20, D=120, d=16, W=8, G=2, B=64, tau=0.9, clusters=6, **kw):
    N = P + D
    K, V, Q, ro = rand_unit(rng, N, d, W, G)
    # near-duplicate groups in the decode span
    pos = P + rng.permutation(D - W)[: clusters * 5].reshape(clusters, 5)
    for c in range(clusters):
        base_k, base_v = K[pos[c, 0]].copy(), V[pos[c, 0]].copy()
        for t in pos[c, 1:]:
            K[t] = base_k + 0.03 * rng.standard_normal(d).astype(np.float32)
            V[t] = base_v + 0.03 * rng.standard_normal(d).astype(np.float32)
    p = f32_params(oracle, head_dim=d, window=W, q_per_kv=G, budget=B, sim_threshold=tau, **kw)
    return p, K, V, Q, ro, np.array([P], dtype=np.int32), pos


def test_consolidate_matches_numpy_cosine_argmax(oracle):
    rng = np.random.default_rng(10)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle)
    N = K.shape[0]
    s = (rng.random(N) ** 3).astype(np.float32)
    role, _ = oracle.prefix_evict(p, ro, pl, s)
    role, _ = oracle.partition(p, ro, pl, s, role)
    assign, best, second = oracle.consolidate(p, ro, pl, K, s, role, want_sims=True)
    Kn = K.astype(np.float64)
    Kn = Kn / np.linalg.norm(Kn, axis=1, keepdims=True)
    seeds = np.flatnonzero(role == oracle.SEED)
    donors = np.flatnonzero(role == oracle.DONOR)
    assert len(seeds) > 0 and len(donors) > 0
    cos = Kn[donors] @ Kn[seeds].T
    arg = cos.argmax(1)          # numpy argmax returns the first (lowest index) maximum
    mx = cos.max(1)
    want = np.where(mx >= np.float32(0.9).astype(np.float64), seeds[arg], -1)
    np.testing.assert_array_equal(assign[donors], want)
    np.testing.assert_allclose(best[donors], mx, rtol=1e-12)
    kept = np.isin(role, [oracle.PREFIX_KEEP, oracle.CORE, oracle.SEED, oracle.RECENT])
    np.testing.assert_array_equal(assign[kept], np.flatnonzero(kept))
    assert (assign[role == oracle.PREFIX_DROP] == -1).all()
    assert (assign[donors] >= 0).sum() > 0


def test_tau_above_one_is_pure_topk_eviction(oracle):
    rng = np.random.default_rng(11)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, tau=1.5)
    out = oracle.compress(p, ro, pl, K, V, Q)
    N, P = K.shape[0], int(pl[0])
    plan = oracle.plan(p, P, N)
    s = out["scores"].astype(np.float64)
    hi = N - plan["r_eff"]
    keep_p = np.sort(np.lexsort((np.arange(P), -s[:P]))[: plan["p_keep"]])
    keep_d = np.sort(P + np.lexsort((np.arange(hi - P), -s[P:hi]))[: plan["slots"]])
    want_src = np.concatenate([keep_p, keep_d, np.arange(hi, N)])
    L = int(out["out_len"][0])
    np.testing.assert_array_equal(out["out_src"][0, :L], want_src)
    np.testing.assert_array_equal(out["K_out"][0, :L], K[want_src])      # bit-identical rows
    np.testing.assert_array_equal(out["V_out"][0, :L], V[want_src])
    assert out["status"][0] & oracle.ST_MERGE_INACTIVE


def test_tau_minus_one_conserves_decode_mass(oracle):
    rng = np.random.default_rng(12)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, tau=-1.0)
    out = oracle.compress(p, ro, pl, K, V, Q)
    N, P = K.shape[0], int(pl[0])
    plan = oracle.plan(p, P, N)
    s = out["scores"].astype(np.float64)
    role = out["role"]
    assert (out["assign"][role == oracle.DONOR] >= 0).all()        # every donor merges
    L = int(out["out_len"][0])
    src = out["out_src"][0, :L]
    dec = src >= P
    assert float(out["out_mass"][0, :L][dec].astype(np.float64).sum()) == \
        pytest.approx(float(s[P:].sum()), rel=1e-6)
    # kept prefix rows carry their own score
    np.testing.assert_array_equal(out["out_mass"][0, :L][~dec], out["scores"][src[~dec]])
    assert plan["status"] == 0 and out["status"][0] == 0


def test_planted_clusters_fold_onto_their_seed(oracle):
    """Injected scores make exactly one member of each planted cluster a seed: all its mates
    must land on it and unrelated tokens must be evicted."""
    rng = np.random.default_rng(13)
    clusters = 6
    p, K, V, Q, ro, pl, pos = make_case(rng, oracle, clusters=clusters, B=8 + 10 + 6 + 20,
                                        core=10, prefix_budget=20)
    N, P = K.shape[0], int(pl[0])
    plan = oracle.plan(p, P, N)
    assert (plan["core"], plan["seeds"]) == (10, 6)
    s = (0.001 * rng.random(N)).astype(np.float32)
    free = np.setdiff1d(np.arange(P, N - 8), pos.ravel())
    s[free[:10]] = 0.9 + 0.01 * np.arange(10, dtype=np.float32)      # the core
    s[pos[:, 0]] = 0.5 + 0.01 * np.arange(clusters, dtype=np.float32)  # one seed per cluster
    out = oracle.compress(p, ro, pl, K, V, Q, scores=s)
    role, assign = out["role"], out["assign"]
    np.testing.assert_array_equal(np.sort(np.flatnonzero(role == oracle.SEED)), np.sort(pos[:, 0]))
    for c in range(clusters):
        seed_slot = assign[pos[c, 0]]
        assert seed_slot >= 0
        assert (assign[pos[c, 1:]] == seed_slot).all()
    others = np.setdiff1d(np.flatnonzero(role == oracle.DONOR), pos.ravel())
    assert (assign[others] == -1).all()
    assert out["status"][0] == 0


# ------------------------------------------------------------------ R7 fold

def test_fold_golden_example(oracle):
    a, ks, vs, want = [], [], [], None
    with open(os.path.join(GOLDEN, "fold_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [np.array(x.split(), dtype=np.float64) for x in line.split("|")]
            if len(a) < 3:
                a.append(parts[0][0]); ks.append(parts[1]); vs.append(parts[2])
            else:
                want = parts
    d = 4
    for dtype in (oracle.F32, oracle.BF16):
        # cache: 1 prefix token, 3 group tokens (seed first), 2 fillers, 1 recent
        K = np.zeros((7, d), dtype=np.float32)
        V = np.zeros((7, d), dtype=np.float32)
        K[0] = [1, 0, 0, 0]
        K[1:4], V[1:4] = np.array(ks), np.array(vs)
        # make the three group keys parallel enough: tau = -1 merges everything anyway
        K[4] = [0, 0, 9, 1]; K[5] = [7, 7, 7, 7]; K[6] = [1, 1, 1, 1]
        s = np.array([0.5, a[0], a[1], a[2], 0.9, 0.8, 0.1], dtype=np.float32)
        # B = 1 recent + 1 prefix + 2 core + 1 seed = 5 ; donors = rows 1 and 3 (0.25 each)
        p = oracle.Params(dtype=dtype, head_dim=d, q_per_kv=1, window=1, recent=1, budget=5,
                          core=2, prefix_budget=1, sim_threshold=-1.0)
        Kx, Vx = (K, V) if dtype == oracle.F32 else (to_bf16_bits(K).reshape(7, d), to_bf16_bits(V).reshape(7, d))
        out = oracle.compress(p, np.array([0, 7]), np.array([1]), Kx, Vx, None, scores=s)
        assert out["out_len"][0] == 5
        np.testing.assert_array_equal(out["role"], [1, 4, 3, 4, 2, 2, 5])
        np.testing.assert_array_equal(out["out_src"][0, :5], [0, 2, 4, 5, 6])
        np.testing.assert_array_equal(out["assign"], [0, 1, 1, 1, 2, 3, 4])
        ko, vo = out["K_out"][0, 1], out["V_out"][0, 1]
        if dtype == oracle.BF16:
            ko, vo = from_bf16_bits(ko), from_bf16_bits(vo)
        np.testing.assert_array_equal(ko, want[1])
        np.testing.assert_array_equal(vo, want[2])
        assert out["out_mass"][0, 1] == want[0][0]


def check_representatives(oracle, p, K, V, out, rtol):
    """Every output row is either an input row, bit for bit, or the score-weighted mean of its
    members (recomputed here from the assignment alone)."""
    s = out["scores"].astype(np.float64)
    L = int(out["out_len"][0])
    n_folded = 0
    for t in range(L):
        members = np.flatnonzero(out["assign"] == t)
        src = out["out_src"][0, t]
        assert src in members
        if len(members) == 1:
            np.testing.assert_array_equal(out["K_out"][0, t], K[src])
            np.testing.assert_array_equal(out["V_out"][0, t], V[src])
            assert out["out_mass"][0, t] == out["scores"][src]
            continue
        n_folded += 1
        a = s[members]
        m = a.sum()
        kk = (a[:, None] * K[members].astype(np.float64)).sum(0) / m
        vv = (a[:, None] * V[members].astype(np.float64)).sum(0) / m
        np.testing.assert_allclose(out["K_out"][0, t], kk, rtol=0, atol=rtol * np.abs(kk).max())
        np.testing.assert_allclose(out["V_out"][0, t], vv, rtol=0, atol=rtol * np.abs(vv).max())
        assert out["out_mass"][0, t] == pytest.approx(m, rel=1e-6)
    return n_folded


def test_representative_is_score_weighted_mean(oracle):
    rng = np.random.default_rng(14)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, tau=0.5)
    out = oracle.compress(p, ro, pl, K, V, Q)
    assert check_representatives(oracle, p, K, V, out, 1e-6) > 0
    L = int(out["out_len"][0])
    assert L <= p.budget
    assert (np.diff(out["out_src"][0, :L]) > 0).all()


def test_first_order_mass_identity(oracle):
    """sum_i a_i <q, k_i> = m <q, k~> for any probe q (the linear part of the perturbation
    decomposition, Section 2.6)."""
    rng = np.random.default_rng(15)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, tau=0.0)
    out = oracle.compress(p, ro, pl, K, V, Q)
    s = out["scores"].astype(np.float64)
    L = int(out["out_len"][0])
    q = rng.standard_normal(K.shape[1])
    checked = 0
    for t in range(L):
        members = np.flatnonzero(out["assign"] == t)
        if len(members) < 2:
            continue
        lhs = float((s[members] * (K[members].astype(np.float64) @ q)).sum())
        rhs = float(out["out_mass"][0, t]) * float(out["K_out"][0, t].astype(np.float64) @ q)
        assert lhs == pytest.approx(rhs, rel=2e-5, abs=1e-7)
        checked += 1
    assert checked > 0


def test_scaling_scores_by_power_of_two_changes_nothing(oracle):
    rng = np.random.default_rng(16)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, tau=0.3)
    s = (rng.random(K.shape[0]) ** 2).astype(np.float32)
    a = oracle.compress(p, ro, pl, K, V, Q, scores=s)
    b = oracle.compress(p, ro, pl, K, V, Q, scores=s * np.float32(2.0 ** -7))
    for key in ("K_out", "V_out", "out_src", "out_len", "assign", "role"):
        np.testing.assert_array_equal(a[key], b[key])
    np.testing.assert_array_equal(a["out_mass"] * np.float32(2.0 ** -7), b["out_mass"])


def test_zero_mass_group_uses_uniform_weights(oracle):
    d = 4
    K = np.array([[1, 0, 0, 0], [2, 0, 0, 0], [4, 0, 0, 0], [0, 1, 0, 0], [0, 0, 1, 0]], dtype=np.float32)
    V = np.arange(20, dtype=np.float32).reshape(5, d)
    s = np.array([0, 0, 0, 0.5, 0.25], dtype=np.float32)
    # P = 0, recent 1, budget 3: slots 2 -> core 1 (row 3), seed 1 (row 0: zero score, lowest
    # index among the ties), donors rows 1, 2 (parallel to row 0 => cosine 1)
    p = oracle.Params(dtype=oracle.F32, head_dim=d, q_per_kv=1, window=1, recent=1, budget=3,
                      core=1, prefix_budget=0, sim_threshold=0.99)
    out = oracle.compress(p, np.array([0, 5]), np.array([0]), K, V, None, scores=s)
    np.testing.assert_array_equal(out["role"], [3, 4, 4, 2, 5])
    np.testing.assert_array_equal(out["assign"], [0, 0, 0, 1, 2])
    np.testing.assert_allclose(out["K_out"][0, 0], K[:3].mean(0))
    np.testing.assert_allclose(out["V_out"][0, 0], V[:3].mean(0))
    assert out["out_mass"][0, 0] == 0.0


# ------------------------------------------------------------------ R8 / R9 and regimes

def test_core_and_recent_pass_through_bit_identically(oracle):
    rng = np.random.default_rng(17)
    for dtype in (oracle.F32, oracle.BF16):
        p, K, V, Q, ro, pl, _ = make_case(rng, oracle, tau=0.2)
        if dtype == oracle.BF16:
            shp = K.shape
            K, V, Q = to_bf16_bits(K).reshape(shp), to_bf16_bits(V).reshape(shp), to_bf16_bits(Q).reshape(Q.shape)
            p.dtype = oracle.BF16
        out = oracle.compress(p, ro, pl, K, V, Q)
        role = out["role"]
        for r in np.flatnonzero(np.isin(role, [oracle.CORE, oracle.RECENT, oracle.PREFIX_KEEP])):
            t = out["assign"][r]
            assert t >= 0 and out["out_src"][0, t] == r
            np.testing.assert_array_equal(out["K_out"][0, t], K[r])
            np.testing.assert_array_equal(out["V_out"][0, t], V[r])
        assert out["out_len"][0] == p.budget


def test_budget_not_smaller_than_cache_is_identity(oracle):
    rng = np.random.default_rng(18)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, B=140)
    N = K.shape[0]
    assert N == 140
    out = oracle.compress(p, ro, pl, K, V, Q)
    assert out["out_len"][0] == N and out["status"][0] == oracle.ST_IDENTITY
    np.testing.assert_array_equal(out["K_out"][0, :N], K)
    np.testing.assert_array_equal(out["V_out"][0, :N], V)
    np.testing.assert_array_equal(out["out_src"][0, :N], np.arange(N))
    np.testing.assert_array_equal(out["assign"], np.arange(N))


def test_second_compress_at_same_budget_is_identity(oracle):
    rng = np.random.default_rng(19)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, tau=0.3)
    a = oracle.compress(p, ro, pl, K, V, Q)
    L = int(a["out_len"][0])
    P2 = int((a["out_src"][0, :L] < pl[0]).sum())
    K2, V2 = a["K_out"][0, :L].copy(), a["V_out"][0, :L].copy()
    b = oracle.compress(p, np.array([0, L]), np.array([P2]), K2, V2, Q)
    assert b["status"][0] == oracle.ST_IDENTITY and b["out_len"][0] == L
    np.testing.assert_array_equal(b["K_out"][0, :L], K2)


def test_exhausted_prefix_turns_consolidation_off(oracle):
    rng = np.random.default_rng(20)
    P, D, d, W, G, B = 400, 60, 16, 8, 1, 40
    N = P + D
    K, V, Q, ro = rand_unit(rng, N, d, W, G)
    K[P + 10] = K[P + 11]       # an exact duplicate pair that would merge if the path were open
    p = f32_params(oracle, head_dim=d, window=W, q_per_kv=G, budget=B, prefix_budget=100)
    plan = oracle.plan(p, P, N)
    assert plan["status"] == oracle.ST_PREFIX_BUDGET_EXHAUSTED and plan["p_keep"] == B - W
    out = oracle.compress(p, ro, np.array([P]), K, V, Q)
    role = out["role"]
    assert out["status"][0] == oracle.ST_PREFIX_BUDGET_EXHAUSTED
    assert not np.isin(role, [oracle.SEED, oracle.DONOR, oracle.CORE]).any()
    assert (role[P:N - W] == oracle.DECODE_EVICT).all() and (out["assign"][P:N - W] == -1).all()
    assert out["out_len"][0] == B
    src = out["out_src"][0]
    np.testing.assert_array_equal(out["K_out"][0], K[src])          # no row is new
    np.testing.assert_array_equal(out["V_out"][0], V[src])
    np.testing.assert_array_equal(src[B - W:], np.arange(N - W, N))
    s = out["scores"].astype(np.float64)
    np.testing.assert_array_equal(src[:B - W], np.sort(np.lexsort((np.arange(P), -s[:P]))[:B - W]))


def test_representative_set_mass_not_below_core_mass(oracle):
    """rho_core <= rho_rep (Section 2.6) when the method's own score stands in for the
    oracle-relevant mass: R contains C, and folding keeps the donors' mass."""
    rng = np.random.default_rng(21)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, tau=0.3)
    out = oracle.compress(p, ro, pl, K, V, Q)
    s = out["scores"].astype(np.float64)
    L = int(out["out_len"][0])
    top = np.sort(s)[::-1][:p.budget].sum()
    core_mass = s[np.isin(out["role"], [oracle.CORE, oracle.RECENT, oracle.PREFIX_KEEP])].sum()
    rep_mass = out["out_mass"][0, :L].astype(np.float64).sum()
    assert 0.0 <= core_mass / top <= rep_mass / top + 1e-9
    assert rep_mass <= s.sum() * (1 + 1e-6)


def test_invalid_arguments_are_rejected(oracle):
    rng = np.random.default_rng(22)
    K, V, Q, ro = rand_unit(rng, 10, 16, 4, 1)
    with pytest.raises(ValueError):    # budget must exceed the recent tail
        oracle.compress(f32_params(oracle, budget=4, recent=4), ro, np.array([2]), K, V, Q)
    with pytest.raises(ValueError):    # cache shorter than the window
        oracle.compress(f32_params(oracle, window=4), np.array([0, 3]), np.array([0]), K[:3], V[:3], Q)
    with pytest.raises(ValueError):    # prefix longer than the cache
        oracle.compress(f32_params(oracle), ro, np.array([11]), K, V, Q)


def test_multi_unit_ragged_batch_equals_unit_by_unit(oracle):
    rng = np.random.default_rng(23)
    d, W, G, B = 16, 6, 2, 40
    lens = [70, 41, 120, 39]
    Ps = [10, 0, 60, 5]
    K = rng.standard_normal((sum(lens), d)).astype(np.float32)
    V = rng.standard_normal((sum(lens), d)).astype(np.float32)
    Q = rng.standard_normal((4, W, G, d)).astype(np.float32)
    ro = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    p = f32_params(oracle, head_dim=d, window=W, q_per_kv=G, budget=B, sim_threshold=0.1)
    out = oracle.compress(p, ro, np.array(Ps), K, V, Q)
    for u in range(4):
        sl = slice(ro[u], ro[u + 1])
        one = oracle.compress(p, np.array([0, lens[u]]), np.array([Ps[u]]), K[sl], V[sl], Q[u:u + 1])
        L = one["out_len"][0]
        assert out["out_len"][u] == L
        np.testing.assert_array_equal(out["K_out"][u, :L], one["K_out"][0, :L])
        np.testing.assert_array_equal(out["assign"][sl], one["assign"])
        np.testing.assert_array_equal(out["scores"][sl], one["scores"])
        assert out["status"][u] == one["status"][0]


# ------------------------------------------------------------------ mass diagnostics (Section 2.6)

def test_mass_diagnostics_match_a_library_sort(oracle):
    """rho_core and rho_rep against numpy: TopK mass from numpy's own sort, the core and
    representative masses summed directly, over several regimes and budgets."""
    rng = np.random.default_rng(31)
    for tau, B, P, D in ((0.9, 64, 20, 120), (0.3, 48, 0, 200), (-1.0, 40, 60, 90), (2.0, 64, 300, 40)):
        p, K, V, Q, ro, pl, _ = make_case(rng, oracle, P=P, D=D, B=B, tau=tau)
        out = oracle.compress(p, ro, pl, K, V, Q)
        rho = oracle.mass_diagnostics(p, ro, out["scores"], out["role"], out["out_mass"], out["out_len"])
        s = out["scores"].astype(np.float64)
        top = np.sort(s, kind="stable")[::-1][:min(B, s.size)].sum()
        prot = np.isin(out["role"], [oracle.PREFIX_KEEP, oracle.CORE, oracle.RECENT])
        L = int(out["out_len"][0])
        want = np.array([s[prot].sum() / top, out["out_mass"][0, :L].astype(np.float64).sum() / top])
        np.testing.assert_allclose(rho[0], want, rtol=2e-7)
        assert 0.0 <= rho[0, 0] <= rho[0, 1] * (1 + 1e-6)          # C is part of R
        assert rho[0, 1] <= s.sum() / top * (1 + 1e-6)             # R holds no more than everything


def test_mass_diagnostics_closed_forms(oracle):
    rng = np.random.default_rng(32)
    # identity regime (N <= B): everything is protected and kept, both ratios are exactly 1
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, P=10, D=40, B=64)
    out = oracle.compress(p, ro, pl, K, V, Q)
    rho = oracle.mass_diagnostics(p, ro, out["scores"], out["role"], out["out_mass"], out["out_len"])
    np.testing.assert_array_equal(rho, np.ones((1, 2), dtype=np.float32))
    # constant scores and no merging: the ratios count rows -- |C| / B and out_len / B = 1
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, P=30, D=150, B=64, tau=2.0)
    N = K.shape[0]
    s = np.full(N, 0.25, dtype=np.float32)
    out = oracle.compress(p, ro, pl, K, V, Q, scores=s)
    rho = oracle.mass_diagnostics(p, ro, s, out["role"], out["out_mass"], out["out_len"])
    n_prot = int(np.isin(out["role"], [oracle.PREFIX_KEEP, oracle.CORE, oracle.RECENT]).sum())
    plan = oracle.plan(p, 30, N)
    assert n_prot == plan["p_keep"] + plan["core"] + plan["r_eff"]
    np.testing.assert_allclose(rho[0], [n_prot / 64.0, 1.0], rtol=1e-7)
    # scaling every score by a power of two changes nothing
    s2 = (rng.random(N) ** 2).astype(np.float32)
    a = oracle.compress(p, ro, pl, K, V, Q, scores=s2)
    b = oracle.compress(p, ro, pl, K, V, Q, scores=s2 * np.float32(64.0))
    ra = oracle.mass_diagnostics(p, ro, s2, a["role"], a["out_mass"], a["out_len"])
    rb = oracle.mass_diagnostics(p, ro, s2 * np.float32(64.0), b["role"], b["out_mass"], b["out_len"])
    np.testing.assert_array_equal(ra, rb)
    # all scores zero: nothing to lose
    z = np.zeros(N, dtype=np.float32)
    o = oracle.compress(p, ro, pl, K, V, Q, scores=z)
    np.testing.assert_array_equal(oracle.mass_diagnostics(p, ro, z, o["role"], o["out_mass"], o["out_len"]),
                                  np.ones((1, 2), dtype=np.float32))


def test_mass_diagnostics_pure_eviction_of_the_best_rows(oracle):
    """No prefix, no recent tail, tau above 1: the event is plain top-B eviction, so the kept set
    IS TopK and rho_rep = 1; the core is the best C of them: rho_core = mass(top C) / mass(top B)."""
    rng = np.random.default_rng(33)
    d, W, G, B, N = 16, 4, 1, 40, 300
    K, V, Q, ro = rand_unit(rng, N, d, W, G)
    p = f32_params(oracle, head_dim=d, window=W, q_per_kv=G, budget=B, recent=0, sim_threshold=2.0)
    s = rng.permutation(N).astype(np.float32) + 1.0      # distinct
    out = oracle.compress(p, ro, np.array([0]), K, V, Q, scores=s)
    rho = oracle.mass_diagnostics(p, ro, s, out["role"], out["out_mass"], out["out_len"])
    best = np.sort(s.astype(np.float64))[::-1]
    C = oracle.plan(p, 0, N)["core"]
    np.testing.assert_allclose(rho[0], [best[:C].sum() / best[:B].sum(), 1.0], rtol=2e-7)


# ------------------------------------------------------------------ decode-loop step (counts, stride)

def test_step_with_unit_counts_is_the_plain_event(oracle):
    rng = np.random.default_rng(41)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, tau=0.3)
    a = oracle.compress(p, ro, pl, K, V, Q)
    N = K.shape[0]
    b = oracle.compress_step(p, ro, pl, K, V, Q, in_count=np.ones(N, dtype=np.int32), out_stride_rows=p.budget + 17)
    L = int(a["out_len"][0])
    for k in ("out_len", "out_src", "out_mass", "assign", "role", "status", "scores"):
        np.testing.assert_array_equal(a[k], b[k])
    np.testing.assert_array_equal(a["K_out"][0, :L], b["K_out"][0, :L])
    np.testing.assert_array_equal(a["V_out"][0, :L], b["V_out"][0, :L])
    assert b["K_out"].shape[1] == p.budget + 17 and not b["K_out"][0, p.budget:].any()
    # counts of an output row = members of its group
    members = np.bincount(a["assign"][a["assign"] >= 0], minlength=L)
    np.testing.assert_array_equal(b["out_count"][0, :L], members[:L])


def test_step_conserves_token_counts_and_places_units_by_stride(oracle):
    rng = np.random.default_rng(42)
    d, W, G, B = 16, 6, 2, 40
    lens, Ps = [90, 120, 41], [10, 30, 0]
    K = rng.standard_normal((sum(lens), d)).astype(np.float32)
    K[20:60] = K[20] + 0.01 * rng.standard_normal((40, d)).astype(np.float32)     # mergeable rows
    K[100:180] = K[100] + 0.01 * rng.standard_normal((80, d)).astype(np.float32)
    V = rng.standard_normal((sum(lens), d)).astype(np.float32)
    Q = rng.standard_normal((3, W, G, d)).astype(np.float32)
    ro = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    cnt = rng.integers(1, 9, sum(lens)).astype(np.int32)
    p = f32_params(oracle, head_dim=d, window=W, q_per_kv=G, budget=B, sim_threshold=0.5)
    out = oracle.compress_step(p, ro, np.array(Ps), K, V, Q, in_count=cnt, out_stride_rows=B + W)
    assert (out["assign"] >= 0).sum() > sum(out["out_len"])          # something was folded
    for u in range(3):
        sl = slice(ro[u], ro[u + 1])
        L = int(out["out_len"][u])
        kept = out["assign"][sl] >= 0
        assert out["out_count"][u, :L].sum() == cnt[sl][kept].sum()
        want = np.bincount(out["assign"][sl][kept], weights=cnt[sl][kept], minlength=L)
        np.testing.assert_array_equal(out["out_count"][u, :L], want[:L].astype(np.int32))
        one = oracle.compress_step(p, np.array([0, lens[u]]), np.array([Ps[u]]), K[sl], V[sl], Q[u:u + 1],
                                   in_count=cnt[sl])
        np.testing.assert_array_equal(out["K_out"][u, :L], one["K_out"][0, :L])   # stride only moves rows
        assert not out["K_out"][u, L:].any()
    # counts ride along: they weigh a fold only where the scores carry no mass, so other counts
    # change out_count and nothing else
    other = oracle.compress_step(p, ro, np.array(Ps), K, V, Q, in_count=3 * cnt + 1, out_stride_rows=B + W)
    for key in ("K_out", "V_out", "out_src", "out_mass", "assign", "status", "scores"):
        np.testing.assert_array_equal(out[key], other[key])
    assert not np.array_equal(out["out_count"], other["out_count"])
    with pytest.raises(ValueError):
        oracle.compress_step(p, ro, np.array(Ps), K, V, Q, in_count=np.zeros(sum(lens), dtype=np.int32))
    with pytest.raises(ValueError):
        oracle.compress_step(p, ro, np.array(Ps), K, V, Q, out_stride_rows=B - 1)


def test_step_zero_mass_group_is_the_count_weighted_mean(oracle):
    """Same hand-built unit as the uniform-weights pin, now with counts 1, 3, 4 on the three
    parallel rows: k~ = (1 k0 + 3 k1 + 4 k2) / 8 exactly."""
    d = 4
    K = np.array([[1, 0, 0, 0], [2, 0, 0, 0], [4, 0, 0, 0], [0, 1, 0, 0], [0, 0, 1, 0]], dtype=np.float32)
    V = np.arange(20, dtype=np.float32).reshape(5, d)
    s = np.array([0, 0, 0, 0.5, 0.25], dtype=np.float32)
    cnt = np.array([1, 3, 4, 2, 5], dtype=np.int32)
    p = oracle.Params(dtype=oracle.F32, head_dim=d, q_per_kv=1, window=1, recent=1, budget=3,
                      core=1, prefix_budget=0, sim_threshold=0.99)
    out = oracle.compress_step(p, np.array([0, 5]), np.array([0]), K, V, None, in_count=cnt, scores=s)
    np.testing.assert_array_equal(out["assign"], [0, 0, 0, 1, 2])
    np.testing.assert_array_equal(out["K_out"][0, 0], (1 * K[0] + 3 * K[1] + 4 * K[2]) / 8)
    np.testing.assert_array_equal(out["V_out"][0, 0], (1 * V[0] + 3 * V[1] + 4 * V[2]) / 8)
    np.testing.assert_array_equal(out["out_count"][0], [8, 2, 5])
    assert out["out_mass"][0, 0] == 0.0


# ------------------------------------------------------------------ merge geometry (Sections 2.5, 5.2)

def _roles_for(oracle, p, ro, pl, s):
    role, _ = oracle.prefix_evict(p, ro, pl, s)
    role, _ = oracle.partition(p, ro, pl, s, role)
    return role


def test_merge_radius_limits_candidates_to_neighbours(oracle):
    rng = np.random.default_rng(51)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, P=10, D=300, B=120, tau=-1.0)
    N = K.shape[0]
    s = (rng.random(N) ** 3).astype(np.float32)
    role = _roles_for(oracle, p, ro, pl, s)
    base = oracle.consolidate(p, ro, pl, K, s, role)
    for radius in (0, N, 10 * N):                      # no limit in effect
        p.merge_radius = radius
        np.testing.assert_array_equal(oracle.consolidate(p, ro, pl, K, s, role), base)
    Kn = K.astype(np.float64)
    Kn /= np.linalg.norm(Kn, axis=1, keepdims=True)
    seeds = np.flatnonzero(role == oracle.SEED)
    donors = np.flatnonzero(role == oracle.DONOR)
    for radius in (3, 17, 60):
        p.merge_radius = radius
        got = oracle.consolidate(p, ro, pl, K, s, role)
        cos = Kn[donors] @ Kn[seeds].T
        near = np.abs(donors[:, None] - seeds[None, :]) <= radius
        cos = np.where(near, cos, -np.inf)
        want = np.where(near.any(1), seeds[cos.argmax(1)], -1)     # tau = -1: any neighbour will do
        np.testing.assert_array_equal(got[donors], want)
        assert (got[donors] >= 0).sum() < (base[donors] >= 0).sum() or radius == 60


def test_kappa_distance_matches_numpy_and_closed_forms(oracle):
    rng = np.random.default_rng(52)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, P=10, D=200, B=100)
    d = p.head_dim
    N = K.shape[0]
    s = (rng.random(N) ** 3).astype(np.float32)
    role = _roles_for(oracle, p, ro, pl, s)
    seeds = np.flatnonzero(role == oracle.SEED)
    donors = np.flatnonzero(role == oracle.DONOR)
    w = rng.random(d // 2).astype(np.float32)
    p.merge_geometry, p.band_weight = 1, w
    # brute force: sum over bands (f, f + d/2) of w_f * 2-norm of the band difference
    diff = K[donors, None, :].astype(np.float64) - K[None, seeds, :].astype(np.float64)
    band = np.sqrt(diff[..., : d // 2] ** 2 + diff[..., d // 2:] ** 2)
    dist = (band * w.astype(np.float64)).sum(-1)
    for theta in (0.0, float(np.median(dist.min(1))), 1e9):
        p.dist_threshold = theta
        got, best, second = oracle.consolidate(p, ro, pl, K, s, role, want_sims=True)
        want = np.where(dist.min(1) <= np.float64(np.float32(theta)), seeds[dist.argmin(1)], -1)
        np.testing.assert_array_equal(got[donors], want)
        np.testing.assert_allclose(-best[donors], dist.min(1), rtol=1e-12)
    assert (got[donors] >= 0).all()                      # theta huge: every donor has a seed
    # one live band, 3-4-5 triangles: the distance is exactly 5 w_f per step
    Kc = np.zeros((N, d), dtype=np.float32)
    f0 = 3
    w1 = np.zeros(d // 2, dtype=np.float32)
    w1[f0] = 0.5
    Kc[:, 0] = rng.standard_normal(N)                    # other bands differ but weigh nothing
    steps = rng.integers(0, 4, N)
    Kc[:, f0], Kc[:, f0 + d // 2] = 3.0 * steps, 4.0 * steps
    p.band_weight, p.dist_threshold = w1, 2.5            # one step = 2.5 is still allowed
    got, best, _ = oracle.consolidate(p, ro, pl, Kc, s, role, want_sims=True)
    gap = np.abs(steps[donors, None] - steps[None, seeds]).min(1)
    np.testing.assert_array_equal(-best[donors], 2.5 * gap)
    np.testing.assert_array_equal(got[donors] >= 0, gap <= 1)
    # invalid weights are refused
    p.band_weight = -w1
    with pytest.raises(ValueError):
        oracle.consolidate(p, ro, pl, Kc, s, role)
    p.band_weight = None
    with pytest.raises(ValueError):
        oracle.consolidate(p, ro, pl, Kc, s, role)


def test_kappa_geometry_end_to_end_folds_planted_duplicates(oracle):
    rng = np.random.default_rng(53)
    p, K, V, Q, ro, pl, pos = make_case(rng, oracle, tau=0.9)
    d = p.head_dim
    p.merge_geometry, p.band_weight = 1, np.ones(d // 2, dtype=np.float32)
    p.dist_threshold = 1.0         # planted members differ by ~0.03 per channel: sum of 8 bands << 1
    # near-duplicate keys get near-identical scores from the window and then share one role;
    # independent scores spread each planted cluster over core, seeds and donors
    s = (rng.random(K.shape[0]) ** 2).astype(np.float32)
    out = oracle.compress(p, ro, pl, K, V, Q, scores=s)
    a = out["assign"]
    merged = np.flatnonzero((out["role"] == oracle.DONOR) & (a >= 0))
    assert len(merged) > 0
    src = out["out_src"][0]
    for i in merged:                # a folded donor sits in the planted cluster of its seed
        seed = src[a[i]]
        ci = [c for c in range(pos.shape[0]) if i in pos[c]]
        assert ci and seed in pos[ci[0]]


# ------------------------------------------------------------------ dispersion and lost mass (Section 2.6, Appendix B)

def test_group_diagnostics_closed_forms(oracle):
    """Hand-built event: one group of two keys a 3-4-5 triangle apart inside one band, one kept
    row, one dropped row.  Equal scores put the representative at the midpoint, so each member
    is 2.5 w_f away; the dropped row's score is the lost mass."""
    d = 8
    K = np.zeros((5, d), dtype=np.float32)
    f = 1
    K[1, f], K[1, f + d // 2] = 3.0, 4.0                  # rows 0 and 1: one band apart by 5
    K[2, 0] = 7.0
    K[3, 2] = 1.0
    s = np.array([0.25, 0.25, 0.125, 0.0625, 0.5], dtype=np.float32)
    assign = np.array([0, 0, 1, -1, 2], dtype=np.int32)
    K_out = np.zeros((1, 4, d), dtype=np.float32)         # stride 4 > budget 3
    K_out[0, 0] = 0.5 * (K[0] + K[1])
    K_out[0, 1] = K[2]
    K_out[0, 2] = K[4]
    w = np.array([1.0, 0.5, 2.0, 1.0], dtype=np.float32)
    p = oracle.Params(dtype=oracle.F32, head_dim=d, q_per_kv=1, window=1, recent=1, budget=3,
                      band_weight=w)
    disp, lost = oracle.group_diagnostics(p, np.array([0, 5]), K, s, assign, K_out)
    assert disp[0] == np.float32(2 * 0.25 * 2.5 * 0.5) and lost[0] == np.float32(0.0625)
    p.band_weight = None                                  # unit weights
    disp, lost = oracle.group_diagnostics(p, np.array([0, 5]), K, s, assign, K_out)
    assert disp[0] == np.float32(2 * 0.25 * 2.5) and lost[0] == np.float32(0.0625)
    # unequal scores 3 : 1 -> the representative sits a quarter of the way: distances 1.25, 3.75
    K_out[0, 0] = 0.75 * K[0] + 0.25 * K[1]
    s2 = s.copy()
    s2[0], s2[1] = 0.75, 0.25
    disp, _ = oracle.group_diagnostics(p, np.array([0, 5]), K, s2, assign, K_out)
    assert disp[0] == np.float32(0.75 * 1.25 + 0.25 * 3.75)
    with pytest.raises(ValueError):
        oracle.group_diagnostics(p, np.array([0, 5]), K, s, np.array([0, 0, 1, -1, 3], dtype=np.int32), K_out)


def test_group_diagnostics_on_events_against_library_norms(oracle):
    """On whole events: numpy's own norm over the bands; mass bookkeeping (what the output
    carries plus what is lost is everything there was); no folds => no dispersion; identity =>
    nothing at all; both outputs scale with the scores, the dispersion with the weights."""
    rng = np.random.default_rng(61)
    for tau, dtype in ((0.5, "f32"), (-1.0, "f32"), (0.5, "bf16"), (2.0, "f32")):
        p, K, V, Q, ro, pl, _ = make_case(rng, oracle, P=30, D=300, d=16, B=90, tau=tau)
        if dtype == "bf16":
            p.dtype = oracle.BF16
            K, V, Q = to_bf16_bits(K), to_bf16_bits(V), to_bf16_bits(Q)
        out = oracle.compress(p, ro, pl, K, V, Q)
        w = rng.random(p.head_dim // 2).astype(np.float32)
        p.band_weight = w
        disp, lost = oracle.group_diagnostics(p, ro, K, out["scores"], out["assign"], out["K_out"])
        Kf = from_bf16_bits(K) if dtype == "bf16" else K
        Ko = from_bf16_bits(out["K_out"]) if dtype == "bf16" else out["K_out"]
        a, s = out["assign"], out["scores"].astype(np.float64)
        kept = a >= 0
        diff = (Kf[kept].astype(np.float64) - Ko[0, a[kept]].astype(np.float64)).reshape(-1, 2, p.head_dim // 2)
        norms = np.linalg.norm(diff, axis=1) @ w.astype(np.float64)
        assert disp[0] == pytest.approx(float((s[kept] * norms).sum()), rel=1e-6)
        L = int(out["out_len"][0])
        assert float(out["out_mass"][0, :L].astype(np.float64).sum()) + float(lost[0]) == \
            pytest.approx(float(s.sum()), rel=1e-6)
        folded = np.count_nonzero((out["role"] == oracle.DONOR) & kept)
        if tau > 1.0:
            assert folded == 0 and disp[0] == 0.0          # verbatim copies are exact zeros
        else:
            assert folded > 0 and disp[0] > 0.0
        d2, l2 = oracle.group_diagnostics(p, ro, K, 2 * out["scores"], a, out["K_out"])
        assert d2[0] == 2 * disp[0] and l2[0] == 2 * lost[0]
        p.band_weight = 4 * w
        d4, l4 = oracle.group_diagnostics(p, ro, K, out["scores"], a, out["K_out"])
        assert d4[0] == 4 * disp[0] and l4[0] == lost[0]
    # identity event: every row kept as it is
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, P=10, D=40, d=16, B=64)
    out = oracle.compress(p, ro, pl, K, V, Q)
    disp, lost = oracle.group_diagnostics(p, ro, K, out["scores"], out["assign"], out["K_out"])
    assert disp[0] == 0.0 and lost[0] == 0.0


def test_nonpositive_softmax_scale_is_the_default_scale(oracle):
    """One rule for the scale parameter everywhere: a value <= 0 stands for 1/sqrt(d), in the
    scorer and in the consumer-side attention alike."""
    rng = np.random.default_rng(5)
    d, W, G, N = 16, 4, 2, 50
    K, V, Q, ro = rand_unit(rng, N, d, W, G)
    explicit = float(np.float32(1.0 / np.sqrt(d)))   # exactly representable: d is a power of four
    base = dict(head_dim=d, window=W, q_per_kv=G, budget=30)
    s_def = oracle.score(f32_params(oracle, softmax_scale=0.0, **base), ro, K, Q)
    for sc in (-1.0, -0.0, explicit):
        np.testing.assert_array_equal(oracle.score(f32_params(oracle, softmax_scale=sc, **base), ro, K, Q), s_def)
    assert not np.array_equal(oracle.score(f32_params(oracle, softmax_scale=0.5, **base), ro, K, Q), s_def)
    q1 = rng.standard_normal((1, G, d)).astype(np.float32)
    Kc, Vc = K[None, :40], V[None, :40]
    lens = np.array([40], dtype=np.int32)
    pa = dict(head_dim=d, window=1, q_per_kv=G, budget=40)
    o_def = oracle.attend(f32_params(oracle, softmax_scale=0.0, **pa), q1, Kc, Vc, lens)
    for sc in (-1.0, explicit):
        np.testing.assert_array_equal(oracle.attend(f32_params(oracle, softmax_scale=sc, **pa), q1, Kc, Vc, lens), o_def)


# ------------------------------------------------------------------ consumer side: proportional attention

def test_attend_is_library_softmax_attention(oracle):
    """Without counts (or with all ones): scipy's softmax and a numpy matmul; fp32 and bf16
    inputs, a row stride, ragged lengths, a custom scale."""
    rng = np.random.default_rng(81)
    for dtype, scale in (("f32", 0.0), ("bf16", 0.0), ("f32", 0.21)):
        d, G, stride = 16, 3, 40
        lens = np.array([1, 17, 40], dtype=np.int32)
        Q = rng.standard_normal((3, G, d)).astype(np.float32)
        K = rng.standard_normal((3, stride, d)).astype(np.float32)
        V = rng.standard_normal((3, stride, d)).astype(np.float32)
        p = f32_params(oracle, head_dim=d, q_per_kv=G, window=1, budget=stride, softmax_scale=scale)
        if dtype == "bf16":
            p.dtype = oracle.BF16
            Qb, Kb, Vb = to_bf16_bits(Q), to_bf16_bits(K), to_bf16_bits(V)
            Q, K, V = from_bf16_bits(Qb), from_bf16_bits(Kb), from_bf16_bits(Vb)
            got = oracle.attend(p, Qb, Kb, Vb, lens)
            got1 = oracle.attend(p, Qb, Kb, Vb, lens, count=np.ones((3, stride), dtype=np.int32))
        else:
            got = oracle.attend(p, Q, K, V, lens)
            got1 = oracle.attend(p, Q, K, V, lens, count=np.ones((3, stride), dtype=np.int32))
        sc = float(np.float32(scale)) if scale else 1.0 / np.sqrt(d)     # the scale is an fp32 parameter
        for u in range(3):
            L = int(lens[u])
            w = scipy_softmax(sc * Q[u].astype(np.float64) @ K[u, :L].astype(np.float64).T, axis=-1)
            np.testing.assert_allclose(got[u], w @ V[u, :L].astype(np.float64), rtol=1e-12, atol=1e-14)
        np.testing.assert_array_equal(got, got1)
        np.testing.assert_allclose(got[0], np.broadcast_to(V[0, 0].astype(np.float64), (G, d)), rtol=1e-15)  # one row


def test_attend_with_counts_equals_attention_over_repeated_rows(oracle):
    """What fixes the ln(count) rule: a cache in which row t occurs n_t times gives the same
    output as the cache with every row once and count n_t.  Also: invalid counts are refused."""
    rng = np.random.default_rng(82)
    d, G, L = 8, 2, 9
    Q = rng.standard_normal((1, G, d)).astype(np.float32)
    K = rng.standard_normal((1, L, d)).astype(np.float32)
    V = rng.standard_normal((1, L, d)).astype(np.float32)
    n = rng.integers(1, 6, L).astype(np.int32)
    rep = np.repeat(np.arange(L), n)
    rng.shuffle(rep)                                                    # order of the rows does not matter
    p = f32_params(oracle, head_dim=d, q_per_kv=G, window=1, budget=64)
    long = oracle.attend(p, Q, K[:, rep], V[:, rep], np.array([len(rep)]))
    short = oracle.attend(p, Q, K, V, np.array([L]), count=n[None, :])
    np.testing.assert_allclose(short, long, rtol=1e-13, atol=1e-15)
    plain = oracle.attend(p, Q, K, V, np.array([L]))
    assert np.abs(plain - long).max() > 1e-3                            # the counts do matter
    with pytest.raises(ValueError):
        oracle.attend(p, Q, K, V, np.array([L]), count=np.zeros((1, L), dtype=np.int32))
    with pytest.raises(ValueError):
        oracle.attend(p, Q, K, V, np.array([L + 1]))


def test_attend_after_a_fold_of_exact_duplicates_is_lossless(oracle):
    """End to end with the event: when the folded donors are exact copies of their seed, the
    compressed cache with its counts attends exactly like the cache of kept and folded rows."""
    rng = np.random.default_rng(83)
    d, W, G, B = 16, 4, 2, 24
    N, P = 60, 0
    K = rng.standard_normal((N, d)).astype(np.float32)
    V = rng.standard_normal((N, d)).astype(np.float32)
    s = (rng.random(N).astype(np.float32) + 0.1)
    p = f32_params(oracle, head_dim=d, window=W, q_per_kv=G, budget=B, core=4, sim_threshold=0.999999)
    Qw = rng.standard_normal((1, W, G, d)).astype(np.float32)
    ro, pl = np.array([0, N]), np.array([P])
    # make every donor an exact copy of some seed (roles come from the scores alone)
    role = _roles_for(oracle, p, ro, pl, s)
    seeds, donors = np.flatnonzero(role == oracle.SEED), np.flatnonzero(role == oracle.DONOR)
    assert len(seeds) > 2 and len(donors) > 10
    src = rng.choice(seeds, size=len(donors))
    K[donors], V[donors] = K[src], V[src]
    out = oracle.compress_step(p, ro, pl, K, V, Qw, scores=s)
    L = int(out["out_len"][0])
    assert (out["assign"][donors] >= 0).all() and L == B
    q = rng.standard_normal((1, G, d)).astype(np.float32)
    comp = oracle.attend(p, q, out["K_out"], out["V_out"], out["out_len"], count=out["out_count"])
    alive = out["assign"] >= 0                                           # kept rows and folded donors
    full = oracle.attend(p, q, K[alive][None], V[alive][None], np.array([int(alive.sum())]))
    np.testing.assert_allclose(comp, full, rtol=1e-5, atol=1e-6)        # K_out, V_out are fp32-rounded means


# ------------------------------------------------------------------ de-duplicated seeding

def _dedup_roles(oracle, p, ro, pl, K, s):
    role, _ = oracle.prefix_evict(p, ro, pl, s)
    role, _, gap = oracle.partition_keys(p, ro, pl, K, s, role)
    return role, gap


def test_dedup_seeding_is_the_greedy_walk_by_its_defining_properties(oracle):
    """The walk is pinned by what characterises it, checked with numpy: seeds are pairwise
    below tau; a row passed over inside the walk resembles a seed ranked before it; the walk
    stops at M seeds or at its horizon; core, prefix and recent roles are those of the default
    rule."""
    for seed, tau, h in ((61, 0.9, 4), (62, 0.5, 2), (63, 0.97, 8), (64, 0.9, 1)):
        rng = np.random.default_rng(seed)
        p, K, V, Q, ro, pl, _ = make_case(rng, oracle, P=12, D=400, B=90, tau=tau, clusters=30)
        N, P = K.shape[0], int(pl[0])
        s = (rng.random(N) ** 3).astype(np.float32)
        base = _roles_for(oracle, p, ro, pl, s)
        p.seed_dedup = h
        role, gap = _dedup_roles(oracle, p, ro, pl, K, s)
        plan = oracle.plan(p, P, N)
        C, M, hi = plan["core"], plan["seeds"], N - plan["r_eff"]
        fixed = (base != oracle.SEED) & (base != oracle.DONOR)
        np.testing.assert_array_equal(role[fixed], base[fixed])
        scratch = np.flatnonzero(~fixed)
        assert set(np.unique(role[scratch])) <= {oracle.SEED, oracle.DONOR}
        order = scratch[np.lexsort((scratch, -s[scratch].astype(np.float64)))]   # score desc, index asc
        walk = order[: min(len(order), h * M)]
        seeds = [i for i in order if role[i] == oracle.SEED]
        assert 0 < len(seeds) <= M and set(seeds) <= set(walk)
        Kn = K.astype(np.float64)
        Kn /= np.linalg.norm(Kn, axis=1, keepdims=True)
        tau64 = float(np.float32(tau))
        cos_ss = Kn[seeds] @ Kn[seeds].T
        assert (cos_ss[np.triu_indices(len(seeds), 1)] < tau64).all()
        last = order.tolist().index(seeds[-1])
        stop = last if len(seeds) == M else len(walk) - 1          # rows examined: up to here
        rank_of = {i: t for t, i in enumerate(order)}
        passed_over = 0
        for t in range(stop + 1):
            i = order[t]
            if role[i] == oracle.SEED:
                continue
            earlier = [q for q in seeds if rank_of[q] < t]
            assert earlier and (Kn[earlier] @ Kn[i]).max() >= tau64, (seed, t)
            passed_over += 1
        assert passed_over > 0 or h == 1
        assert gap[0] > 1e-6          # no decision of these cases sits on the threshold


def test_dedup_seeding_reduces_to_the_default_rule_and_to_one_seed(oracle):
    rng = np.random.default_rng(65)
    p, K, V, Q, ro, pl, _ = make_case(rng, oracle, P=10, D=300, B=80, tau=2.0)
    N = K.shape[0]
    s = (rng.random(N) ** 2).astype(np.float32)
    base = _roles_for(oracle, p, ro, pl, s)
    for h in (1, 3):                      # nothing resembles anything at tau > 1: the M best rows
        p.seed_dedup = h
        np.testing.assert_array_equal(_dedup_roles(oracle, p, ro, pl, K, s)[0], base)
    # tau <= -1: every later row resembles the first seed, which stays alone; the event then
    # folds the whole scratch into it and conserves the decode mass outside the recent tail
    p.sim_threshold, p.seed_dedup = -1.0, 4
    role, _ = _dedup_roles(oracle, p, ro, pl, K, s)
    plan = oracle.plan(p, int(pl[0]), N)
    scratch = np.flatnonzero((base == oracle.SEED) | (base == oracle.DONOR))
    best = scratch[np.lexsort((scratch, -s[scratch].astype(np.float64)))][0]
    assert list(np.flatnonzero(role == oracle.SEED)) == [best]
    out = oracle.compress(p, ro, pl, K, V, Q, scores=s)
    assert out["out_len"][0] == plan["p_keep"] + plan["core"] + 1 + plan["r_eff"]
    slot = int(np.flatnonzero(out["out_src"][0] == best)[0])
    assert np.isclose(out["out_mass"][0, slot], s[scratch].astype(np.float64).sum(), rtol=1e-6)


def test_dedup_seeding_keeps_one_copy_of_every_repeated_key(oracle):
    """Each of 40 distinct keys appears 6 times in the scratch: the seeds are the best-scored
    copy of each of the M best keys, where the default rule spends several seeds on one key."""
    rng = np.random.default_rng(66)
    d, P, W, reps, kinds = 16, 0, 4, 6, 40
    D = reps * kinds + W
    base_k = rng.standard_normal((kinds, d)).astype(np.float32)
    kind = np.concatenate([rng.permutation(np.repeat(np.arange(kinds), reps)), np.full(W, -1)])
    K = np.where(kind[:, None] >= 0, base_k[np.maximum(kind, 0)], rng.standard_normal((D, d))).astype(np.float32)
    V = rng.standard_normal((D, d)).astype(np.float32)
    Q = rng.standard_normal((1, W, 1, d)).astype(np.float32)
    ro, pl = np.array([0, D], dtype=np.int64), np.array([P], dtype=np.int32)
    # copies of a key score alike (as near-duplicates do), every score distinct
    s = (10.0 * rng.permutation(kinds + 1)[kind] + rng.permutation(D) / D).astype(np.float32)
    p = f32_params(oracle, head_dim=d, window=W, q_per_kv=1, recent=W, budget=W + 12, core=0,
                   prefix_budget=0, sim_threshold=0.99, seed_dedup=reps * kinds)
    plan = oracle.plan(p, P, D)
    M = plan["seeds"]
    assert plan["core"] == 0 and M == 12
    role, _ = _dedup_roles(oracle, p, ro, pl, K, s)
    seeds = np.flatnonzero(role == oracle.SEED)
    best_of_kind = np.array([np.flatnonzero(kind == k)[np.argmax(s[kind == k])] for k in range(kinds)])
    want = np.sort(best_of_kind[np.argsort(-s[best_of_kind])[:M]])
    np.testing.assert_array_equal(seeds, want)
    p.seed_dedup = 0
    default_seeds = np.flatnonzero(_roles_for(oracle, p, ro, pl, s) == oracle.SEED)
    assert len(np.unique(kind[default_seeds])) < M
