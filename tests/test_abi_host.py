"""CPU-only checks of the C-ABI library: it loads, exports every symbol that include/cask.h
declares, and its host-side logic (budget split, workspace sizing, argument validation)
behaves as documented.  No compute call is made here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def cask():
    import paper_2604_10900_amd as cask
    if not os.path.exists(cask.binding.LIB_PATH):
        from paper_2604_10900_amd.build import build_lib
        build_lib()
    cask.load()
    return cask


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cask.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cask_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(cask):
    names = declared_functions()
    assert {"cask_score", "cask_partition", "cask_consolidate", "cask_prefix_evict",
            "cask_compress", "cask_plan", "cask_workspace_bytes"} <= set(names)
    lib = cask.load()
    for n in names:
        assert getattr(lib, n) is not None, n
    assert sorted(cask.binding.EXPORTS) == names


def test_binding_declares_every_signature(cask):
    """Every entry point the binding calls has its argument and result types declared (an
    undeclared size_t argument would be marshalled as a 32-bit int), and the parameter counts
    match the header's prototypes."""
    lib = cask.load()
    text = open(os.path.join(ROOT, "include", "cask.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    for n in declared_functions():
        fn = getattr(lib, n)
        assert fn.argtypes is not None, n
        proto = re.search(r"\b%s\s*\(([^)]*)\)" % n, text).group(1)
        n_params = 0 if proto.strip() in ("", "void") else proto.count(",") + 1
        assert len(fn.argtypes) == n_params, (n, len(fn.argtypes), n_params)
        for i, par in enumerate(proto.split(",")):
            if "size_t" in par:
                assert fn.argtypes[i] is C.c_size_t, (n, i)
    assert lib.cask_workspace_bytes.restype is C.c_size_t


def test_workspace_sizes_of_4_gib_and_more_pass_the_boundary(cask):
    """A batch of cfg5's size needs a workspace beyond 2^32 bytes: the size comes back whole, and
    an entry point given that size (with an invalid batch) does not mistake it for a small one."""
    p = cask.Params(q_per_kv=4, budget=384)
    rows = 16384 * 19000
    n = cask.workspace_bytes(p, 16384, rows, 33280)
    assert n > (1 << 32) and n > 20 * rows
    lib = cask.load()
    ro = np.array([0, 1000], dtype=np.int64)
    pl = np.array([0], dtype=np.int32)
    fake = C.c_void_p(256)
    b1 = cask.binding._Batch(1, fake, fake, ro.ctypes.data, pl.ctypes.data, fake, fake, fake)
    ok = p.c()
    # one byte short of the layout is refused (the size check sees the whole size_t; that the
    # argument is declared as one is asserted in test_binding_declares_every_signature)
    need = cask.workspace_bytes(p, 1, 1000, 1000)
    assert lib.cask_compress_step(C.byref(ok), C.byref(b1), None, fake, fake, 384, fake, fake, None, None,
                                  None, None, fake, fake, need - 257, None) == cask.binding.ENOMEM


def test_plan_matches_golden_table(cask):
    rows = 0
    with open(os.path.join(GOLDEN, "plan_table.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            lhs, rhs = line.split("|")
            P, D, B, R, core, *pb = (int(x) for x in lhs.split())
            r_eff, p_keep, slots, c, m, status = (int(x) for x in rhs.split())
            p = cask.Params(window=min(128, P + D), recent=R, budget=B, core=core,
                            prefix_budget=pb[0] if pb else -1)
            assert cask.plan(p, P, P + D) == dict(r_eff=r_eff, p_keep=p_keep, slots=slots, core=c,
                                                  seeds=m, status=status), line
            rows += 1
    assert rows >= 18


def test_plan_agrees_with_oracle_on_random_sizes(cask, oracle):
    rng = np.random.default_rng(0)
    for _ in range(4000):
        R = int(rng.integers(0, 200))
        B = int(rng.integers(R + 1, 3000))
        P = int(rng.integers(0, 70000))
        D = int(rng.integers(0, 40000))
        if P + D == 0:
            continue
        kw = dict(window=1, recent=R, budget=B, core=int(rng.integers(-1, 400)),
                  prefix_budget=int(rng.integers(-1, 1500)))
        got = cask.plan(cask.Params(**kw), P, P + D)
        want = oracle.plan(oracle.Params(**kw), P, P + D)
        assert got == want, (kw, P, D)
        # the kernels size LDS blocks and fold workgroups by this bound on the seeds of a unit
        bound = (B + 4) // 5 if kw["core"] < 0 else max(0, B - kw["core"])
        assert got["seeds"] <= min(B, bound), (kw, P, D, got)
        assert got["p_keep"] + min(D - got["r_eff"], got["slots"]) + got["r_eff"] == min(P + D, B)


def test_plan_rejects_bad_sizes(cask):
    with pytest.raises(cask.CaskError):
        cask.plan(cask.Params(budget=100, recent=100), 10, 1000)
    with pytest.raises(cask.CaskError):
        cask.plan(cask.Params(), 11, 10)
    with pytest.raises(cask.CaskError):
        cask.plan(cask.Params(head_dim=100), 1, 10)


def test_workspace_size_is_sane(cask):
    p = cask.Params(q_per_kv=7, budget=384)
    small = cask.workspace_bytes(p, 4, 4 * 8448, 8448)
    big = cask.workspace_bytes(p, 112, 112 * 8448, 8448)
    assert 0 < small < big
    assert big < 64 * 112 * 8448            # a few dozen bytes per cached row
    assert cask.workspace_bytes(cask.Params(dtype=7), 1, 10, 10) == 0


def test_split_choice_of_the_first_sweep_shows_in_the_workspace_size(cask):
    """The per-split row statistics are the only part of the layout that depends on the number
    of key splits, so the size tells which count the cost model took: on the headline shape 8
    splits in the wide form of the sweep, 4 in the narrow one; a small batch stays narrow."""
    from paper_2604_10900_amd import binding
    kw = dict(q_per_kv=7, budget=384)
    shape = (112, 112 * 8448, 8448)
    auto = cask.workspace_bytes(cask.Params(**kw), *shape)
    narrow = cask.workspace_bytes(cask.Params(path_flags=binding.PATH_NARROW_ROWS, **kw), *shape)
    by_splits = {sp: cask.workspace_bytes(cask.Params(score_splits=sp, **kw), *shape) for sp in (2, 4, 8)}
    assert by_splits[2] < by_splits[4] < by_splits[8]
    assert auto == by_splits[8]
    assert narrow == by_splits[4]
    # one more split costs units x padded window rows x 8 bytes (up to the 256-byte rounding)
    per_split = (by_splits[8] - by_splits[4]) / 4
    assert abs(per_split - 112 * 896 * 8) <= 256
    small = (8, 8 * 8448, 8448)
    assert cask.workspace_bytes(cask.Params(**kw), *small) == \
        cask.workspace_bytes(cask.Params(path_flags=binding.PATH_NARROW_ROWS, **kw), *small)


def test_workspace_size_grows_with_every_argument(cask):
    """A workspace sized for longer units, more units or more rows also serves a smaller batch:
    the entry points lay it out again from the batch they get and only compare sizes."""
    for kw in (dict(q_per_kv=7, budget=384), dict(q_per_kv=1, window=16, budget=2048), dict(head_dim=64, budget=100)):
        p = cask.Params(**kw)
        prev = 0
        for L in sorted({p.window, 64, 300, 512, 1000, 1024, 1025, 3000, 4608, 9000, 40000, 200000}):
            n = cask.workspace_bytes(p, 64, 64 * 200000, L)
            assert n >= prev > -1, (kw, L)
            prev = n
        assert cask.workspace_bytes(p, 65, 64 * 200000, 9000) >= cask.workspace_bytes(p, 64, 64 * 200000, 9000)
        assert cask.workspace_bytes(p, 64, 65 * 200000, 9000) >= cask.workspace_bytes(p, 64, 64 * 200000, 9000)


def test_host_validation_needs_no_gpu(cask):
    """Bad arguments are refused before any HIP call; an empty batch is a no-op."""
    lib = cask.load()
    b = cask.binding._Batch(0, None, None, None, None, None, None, None)
    ok = cask.Params().c()
    assert lib.cask_compress(C.byref(ok), C.byref(b), None, None, None, None, None, None, None,
                             None, None, 0, None) == cask.binding.OK
    bad = cask.Params(window=0).c()
    assert lib.cask_score(C.byref(bad), C.byref(b), None, None, 0, None) == cask.binding.EINVAL
    assert lib.cask_score(None, C.byref(b), None, None, 0, None) == cask.binding.EINVAL
    assert lib.cask_compress(C.byref(ok), None, None, None, None, None, None, None, None, None,
                             None, 0, None) == cask.binding.EINVAL
    # one unit shorter than the window: refused on the host mirrors alone
    ro = np.array([0, 10], dtype=np.int64)
    pl = np.array([0], dtype=np.int32)
    fake = C.c_void_p(256)   # never dereferenced: validation fails first
    b1 = cask.binding._Batch(1, fake, fake, ro.ctypes.data, pl.ctypes.data, fake, fake, fake)
    assert lib.cask_compress(C.byref(ok), C.byref(b1), fake, fake, fake, fake, None, None, None,
                             fake, fake, 1 << 30, None) == cask.binding.EINVAL
    assert cask.load().cask_strerror(cask.binding.ENOMEM).decode() == "workspace too small"


def test_host_validation_alignment_and_unit_size(cask):
    """Misaligned data pointers and units beyond the 32-bit byte-offset limit are refused on the
    host; nothing is dereferenced."""
    lib = cask.load()
    ok = cask.Params().c()
    ro = np.array([0, 1000], dtype=np.int64)
    pl = np.array([100], dtype=np.int32)
    fake = C.c_void_p(4096)
    odd = C.c_void_p(4096 + 2)
    good = cask.binding._Batch(1, fake, fake, ro.ctypes.data, pl.ctypes.data, fake, fake, fake)
    # a well-formed call with a workspace that is too small gets past validation: ENOMEM
    assert lib.cask_compress(C.byref(ok), C.byref(good), fake, fake, fake, fake, None, None, None,
                             fake, fake, 16, None) == cask.binding.ENOMEM
    for k in range(3):
        ptrs = [fake, fake, fake]
        ptrs[k] = odd
        b = cask.binding._Batch(1, fake, fake, ro.ctypes.data, pl.ctypes.data, *ptrs)
        assert lib.cask_compress(C.byref(ok), C.byref(b), fake, fake, fake, fake, None, None, None,
                                 fake, fake, 16, None) == cask.binding.EINVAL
    assert lib.cask_compress(C.byref(ok), C.byref(good), odd, fake, fake, fake, None, None, None,
                             fake, fake, 16, None) == cask.binding.EINVAL
    assert lib.cask_compress(C.byref(ok), C.byref(good), fake, fake, fake, fake, None, None, None,
                             fake, odd, 1 << 40, None) == cask.binding.EINVAL
    big = np.array([0, 1 << 23], dtype=np.int64)
    b = cask.binding._Batch(1, fake, fake, big.ctypes.data, pl.ctypes.data, fake, fake, fake)
    assert lib.cask_score(C.byref(ok), C.byref(b), fake, fake, 1 << 40, None) == cask.binding.EINVAL


def test_timing_calls_validate_without_gpu(cask):
    lib = cask.load()
    assert lib.cask_timing_enable_stages(4, 0) == cask.binding.EINVAL
    assert lib.cask_timing_enable_stages(5000, 2) == cask.binding.EINVAL
    assert lib.cask_timing_enable(0) == cask.binding.OK
    ms = (C.c_float * 7)()
    n = C.c_int(-1)
    assert lib.cask_timing_read(ms, C.byref(n)) == cask.binding.OK and n.value == 0
    assert lib.cask_timing_read(None, C.byref(n)) == cask.binding.EINVAL


def test_mass_diagnostics_validates_on_the_host(cask):
    lib = cask.load()
    ok = cask.Params().c()
    ro = np.array([0, 1000], dtype=np.int64)
    pl = np.array([100], dtype=np.int32)
    fake = C.c_void_p(4096)
    good = cask.binding._Batch(1, fake, fake, ro.ctypes.data, pl.ctypes.data, fake, fake, fake)
    assert lib.cask_mass_diagnostics(C.byref(ok), C.byref(good), fake, fake, fake, fake, None, None) == cask.binding.EINVAL
    assert lib.cask_mass_diagnostics(C.byref(ok), C.byref(good), None, fake, fake, fake, fake, None) == cask.binding.EINVAL
    empty = cask.binding._Batch(0, None, None, None, None, None, None, None)
    assert lib.cask_mass_diagnostics(C.byref(ok), C.byref(empty), None, None, None, None, None, None) == cask.binding.OK



def test_merge_geometry_fields_validate_on_the_host(cask):
    """Negative radius, unknown geometry, and the kappa geometry without weights or with a
    negative / NaN threshold are refused before any HIP call."""
    lib = cask.load()
    b = cask.binding._Batch(0, None, None, None, None, None, None, None)

    def rc(**kw):
        cp = cask.Params().c()
        for k, v in kw.items():
            setattr(cp, k, v)
        return lib.cask_consolidate(C.byref(cp), C.byref(b), None, None, None, None, 0, None)

    assert rc() == cask.binding.OK
    assert rc(merge_radius=17) == cask.binding.OK
    assert rc(merge_radius=-1) == cask.binding.EINVAL
    assert rc(merge_geometry=2) == cask.binding.EINVAL
    assert rc(merge_geometry=-1) == cask.binding.EINVAL
    assert rc(merge_geometry=1) == cask.binding.EINVAL                       # no band weights
    assert rc(merge_geometry=1, band_weight=256, dist_threshold=-1.0) == cask.binding.EINVAL
    assert rc(merge_geometry=1, band_weight=256, dist_threshold=float("nan")) == cask.binding.EINVAL
    assert rc(merge_geometry=1, band_weight=256, dist_threshold=3.0) == cask.binding.OK   # empty batch: no-op


def test_seed_dedup_validates_on_the_host(cask):
    """Negative multiples, the kappa geometry, and walks longer than the kernel's LDS list
    (multiple x largest possible seed count > 2048) are refused before any HIP call."""
    lib = cask.load()
    b = cask.binding._Batch(0, None, None, None, None, None, None, None)

    def rc(**kw):
        cp = cask.Params().c()
        for k, v in kw.items():
            setattr(cp, k, v)
        return lib.cask_partition(C.byref(cp), C.byref(b), None, None, None, None, 0, None)

    assert rc(seed_dedup=0) == cask.binding.OK
    assert rc(seed_dedup=4) == cask.binding.OK                 # budget 384: at most 77 seeds, 308 rows
    assert rc(seed_dedup=-1) == cask.binding.EINVAL
    assert rc(seed_dedup=2, merge_geometry=1, band_weight=256, dist_threshold=1.0) == cask.binding.EINVAL
    assert rc(seed_dedup=26) == cask.binding.OK                # 26 * 77 = 2002
    assert rc(seed_dedup=27) == cask.binding.EINVAL            # 27 * 77 = 2079
    assert rc(seed_dedup=8, core=100) == cask.binding.EINVAL   # up to 284 seeds: 2272 rows
    assert rc(seed_dedup=7, core=100) == cask.binding.OK


def test_group_diagnostics_validates_on_the_host(cask):
    lib = cask.load()
    ok = cask.Params().c()
    ro = np.array([0, 1000], dtype=np.int64)
    pl = np.array([0], dtype=np.int32)
    fake = C.c_void_p(256)
    good = cask.binding._Batch(1, fake, fake, ro.ctypes.data, pl.ctypes.data, fake, fake, fake)
    B = cask.Params().budget

    def rc(scores=fake, assign=fake, K_out=fake, stride=B, disp=fake, lost=fake):
        return lib.cask_group_diagnostics(C.byref(ok), C.byref(good), scores, assign, K_out,
                                          C.c_int32(stride), disp, lost, None)

    assert rc(scores=None) == cask.binding.EINVAL
    assert rc(assign=None) == cask.binding.EINVAL
    assert rc(K_out=None) == cask.binding.EINVAL
    assert rc(K_out=C.c_void_p(264)) == cask.binding.EINVAL          # not 16-byte aligned
    assert rc(stride=B - 1) == cask.binding.EINVAL
    assert rc(disp=None) == cask.binding.EINVAL
    assert rc(lost=None) == cask.binding.EINVAL
    empty = cask.binding._Batch(0, None, None, None, None, None, None, None)
    assert lib.cask_group_diagnostics(C.byref(ok), C.byref(empty), None, None, None, C.c_int32(B), None,
                                      None, None) == cask.binding.OK


def test_attend_validates_on_the_host(cask):
    lib = cask.load()
    ok = cask.Params().c()
    fake = C.c_void_p(256)

    def rc(n=3, Q=fake, K=fake, V=fake, stride=100, length=fake, count=None, pitch=0, out=fake, params=ok):
        return lib.cask_attend(C.byref(params) if params is not None else None, C.c_int32(n), Q, K, V,
                               C.c_int32(stride), length, count, C.c_int32(pitch), out, None)

    assert rc(n=0) == cask.binding.OK                       # empty batch: nothing is touched
    assert rc(n=-1) == cask.binding.EINVAL
    assert rc(Q=None) == cask.binding.EINVAL
    assert rc(K=None) == cask.binding.EINVAL
    assert rc(V=None) == cask.binding.EINVAL
    assert rc(out=None) == cask.binding.EINVAL
    assert rc(length=None) == cask.binding.EINVAL
    assert rc(stride=0) == cask.binding.EINVAL
    assert rc(K=C.c_void_p(264)) == cask.binding.EINVAL     # not 16-byte aligned
    assert rc(count=fake, pitch=0) == cask.binding.EINVAL
    assert rc(params=None) == cask.binding.EINVAL
    assert rc(params=cask.Params(head_dim=100).c()) == cask.binding.EINVAL


def test_bench_refuses_more_than_one_gpu():
    """One GPU is what this build measures: `bench.py --gpus 2` says so and exits before it
    touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
