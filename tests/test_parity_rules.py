"""CPU checks of the comparator itself (tests/parity.py): the near-tie rules that excuse a
difference between the HIP path and the oracle must accept what they are meant to accept and
refuse a planted mistake.  The mistakes are planted in copies of the oracle's own results."""
import numpy as np
import pytest

from oracle import ref
from tests import parity


def _event(seed=0, N=400, P=60, B=120, W=16):
    rng = np.random.default_rng(seed)
    rp = ref.Params(dtype=ref.F32, head_dim=16, q_per_kv=1, window=W, budget=B, sim_threshold=2.0)
    s = (rng.random(N) ** 4).astype(np.float32) + np.float32(1e-3)
    row_off = np.array([0, N], dtype=np.int64)
    pl = np.array([P], dtype=np.int32)
    role, _ = ref.prefix_evict(rp, row_off, pl, s)
    role, _ = ref.partition(rp, row_off, pl, s, role)
    kept = np.flatnonzero(np.isin(role, [ref.PREFIX_KEEP, ref.CORE, ref.SEED, ref.RECENT]))
    return rp, P, s, role, kept


def test_identical_keep_sets_pass():
    rp, P, s, role, kept = _event()
    assert parity.check_keepset_near_ties(rp, P, s, kept, kept) == 0


def test_a_swap_across_a_wide_gap_is_refused():
    rp, P, s, role, kept = _event(1)
    # drop the best decode row the oracle keeps and keep one it evicts instead
    donors = np.flatnonzero(role == ref.DONOR)
    core = np.flatnonzero(role == ref.CORE)
    wrong = np.sort(np.concatenate([np.setdiff1d(kept, core[np.argmax(s[core])]), donors[:1]]))
    with pytest.raises(AssertionError):
        parity.check_keepset_near_ties(rp, P, s, wrong, kept)
    # same in the prefix
    keep_p = np.flatnonzero(role == ref.PREFIX_KEEP)
    drop_p = np.flatnonzero(role == ref.PREFIX_DROP)
    wrong = np.sort(np.concatenate([np.setdiff1d(kept, keep_p[np.argmax(s[keep_p])]), drop_p[:1]]))
    with pytest.raises(AssertionError):
        parity.check_keepset_near_ties(rp, P, s, wrong, kept)


def test_a_swap_at_a_near_tied_cut_is_accepted_and_only_there():
    rp, P, s, role, kept = _event(2)
    pl = ref.plan(rp, P, len(s))
    lo, hi = P, len(s) - pl["r_eff"]
    idx = np.arange(lo, hi)
    order = idx[np.lexsort((idx, -s[lo:hi].astype(np.float64)))]
    k = pl["core"] + pl["seeds"]
    last_in, first_out = order[k - 1], order[k]
    s2 = s.copy()
    s2[first_out] = np.nextafter(s2[last_in], np.float32(0))       # a near-tie at the cut
    rp2, _, _, role2, kept2 = rp, P, s2, *_roles(rp, P, s2)
    assert last_in in kept2 and first_out not in kept2
    flipped = np.sort(np.concatenate([np.setdiff1d(kept2, [last_in]), [first_out]]))
    assert parity.check_keepset_near_ties(rp, P, s2, flipped, kept2) == 2
    # the same near-tie does not excuse a row far from the cut
    far = order[k + 40]
    wrong = np.sort(np.concatenate([np.setdiff1d(kept2, [last_in]), [far]]))
    with pytest.raises(AssertionError):
        parity.check_keepset_near_ties(rp, P, s2, wrong, kept2)
    # nor an unpaired difference (a decode row traded for a prefix row)
    drop_p = np.flatnonzero(role2 == ref.PREFIX_DROP)
    wrong = np.sort(np.concatenate([np.setdiff1d(kept2, [last_in]), drop_p[:1]]))
    with pytest.raises(AssertionError):
        parity.check_keepset_near_ties(rp, P, s2, wrong, kept2)
    # nor a missing recent row
    with pytest.raises(AssertionError):
        parity.check_keepset_near_ties(rp, P, s2, kept2[:-1], kept2)


def _roles(rp, P, s):
    row_off = np.array([0, len(s)], dtype=np.int64)
    pl = np.array([P], dtype=np.int32)
    role, _ = ref.prefix_evict(rp, row_off, pl, s)
    role, _ = ref.partition(rp, row_off, pl, s, role)
    kept = np.flatnonzero(np.isin(role, [ref.PREFIX_KEEP, ref.CORE, ref.SEED, ref.RECENT]))
    return role, kept


def test_assignment_excusal_needs_a_near_tie_of_cosines():
    got = np.array([3, 5, -1, 7])
    want = np.array([3, 6, -1, 7])
    best = np.array([0.95, 0.93, 0.2, 0.99])
    second = np.array([0.5, 0.92995, 0.1, 0.3])
    assert parity.check_assign_excused(got, want, best, second, 0.9, "t") == 1
    with pytest.raises(AssertionError):
        parity.check_assign_excused(got, want, best, np.array([0.5, 0.92, 0.1, 0.3]), 0.9, "t")
    # a donor at the threshold
    assert parity.check_assign_excused(np.array([-1]), np.array([4]), np.array([0.90003]), np.array([0.1]), 0.9) == 1
