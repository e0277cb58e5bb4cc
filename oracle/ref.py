"""ctypes front end of the CASK compression-event ORACLE (test infrastructure).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this module.
Arrays are numpy arrays on the host; bf16 data travels as uint16 bit patterns.
The arithmetic lives in cask_ref.c; nothing here computes anything of the method.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcask_ref.so")

F32, BF16 = 0, 1
ST_ACTIVE, ST_IDENTITY, ST_PREFIX_BUDGET_EXHAUSTED, ST_MERGE_INACTIVE = 0, 1, 2, 4
PREFIX_DROP, PREFIX_KEEP, CORE, SEED, DONOR, RECENT, DECODE_EVICT = range(7)


def build(force: bool = False) -> str:
    """Compile cask_ref.c with gcc into libcask_ref.so next to this file.  (CASK_REF_LIB in the
    environment names another build of the same source to load instead, e.g. one made with
    sanitizers by tests/test_sanitizers.py; nothing is compiled then.)"""
    global _LIB_PATH
    other = os.environ.get("CASK_REF_LIB")
    if other:
        _LIB_PATH = other
        return _LIB_PATH
    src = os.path.join(_HERE, "cask_ref.c")
    hdr = os.path.join(_HERE, "cask_ref.h")
    if (not force and os.path.exists(_LIB_PATH)
            and os.path.getmtime(_LIB_PATH) >= max(os.path.getmtime(src), os.path.getmtime(hdr))):
        return _LIB_PATH
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-ffp-contract=off", "-o", _LIB_PATH, src, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


class _Params(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("head_dim", C.c_int32), ("q_per_kv", C.c_int32),
                ("window", C.c_int32), ("recent", C.c_int32), ("budget", C.c_int32),
                ("core", C.c_int32), ("prefix_budget", C.c_int32),
                ("sim_threshold", C.c_float), ("softmax_scale", C.c_float),
                ("causal", C.c_int32), ("merge_radius", C.c_int32), ("merge_geometry", C.c_int32),
                ("dist_threshold", C.c_float), ("band_weight", C.c_void_p),
                ("seed_dedup", C.c_int32)]


class _Plan(C.Structure):
    _fields_ = [("r_eff", C.c_int32), ("p_keep", C.c_int32), ("slots", C.c_int32),
                ("core", C.c_int32), ("seeds", C.c_int32), ("status", C.c_int32)]


@dataclass
class Params:
    dtype: int = BF16
    head_dim: int = 128
    q_per_kv: int = 1
    window: int = 128
    recent: int = -1
    budget: int = 384
    core: int = -1
    prefix_budget: int = -1
    sim_threshold: float = 0.9
    softmax_scale: float = 0.0
    causal: int = 1
    merge_radius: int = 0          # > 0: donors fold only into seeds at most this many rows away
    merge_geometry: int = 0        # 0 cosine (sim_threshold), 1 kappa-weighted band distance
    dist_threshold: float = 0.0    # geometry 1: fold iff distance <= this
    band_weight: Optional[np.ndarray] = None   # geometry 1: float32 [head_dim / 2], >= 0
    seed_dedup: int = 0            # h > 0: seeds chosen greedily among the best h*M scratch rows

    def c(self) -> _Params:
        bw = None
        if self.band_weight is not None:
            self._bw = np.ascontiguousarray(self.band_weight, dtype=np.float32)   # keep it alive
            assert self._bw.size == self.head_dim // 2
            bw = self._bw.ctypes.data
        return _Params(self.dtype, self.head_dim, self.q_per_kv, self.window, self.recent,
                       self.budget, self.core, self.prefix_budget, self.sim_threshold,
                       self.softmax_scale, self.causal, self.merge_radius, self.merge_geometry,
                       self.dist_threshold, bw, self.seed_dedup)


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB_PATH)
        _lib.cask_ref_bf16_from_double.restype = C.c_uint16
        _lib.cask_ref_bf16_from_double.argtypes = [C.c_double]
        _lib.cask_ref_bf16_to_double.restype = C.c_double
        _lib.cask_ref_bf16_to_double.argtypes = [C.c_uint16]
    return _lib


def _ptr(a):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _np_elem(dtype: int):
    return np.uint16 if dtype == BF16 else np.float32


def _check_data(p: Params, *arrs):
    for a in arrs:
        if a is not None:
            assert a.dtype == _np_elem(p.dtype), (a.dtype, p.dtype)


def bf16_from_double(x: float) -> int:
    return int(lib().cask_ref_bf16_from_double(float(x)))


def bf16_to_double(h: int) -> float:
    return float(lib().cask_ref_bf16_to_double(int(h)))


def plan(p: Params, P: int, N: int) -> dict:
    out = _Plan()
    cp = p.c()
    lib().cask_ref_plan(C.byref(cp), C.c_int32(P), C.c_int32(N), C.byref(out))
    return {k: getattr(out, k) for k, _ in _Plan._fields_}


def _units(row_off, prefix_len=None):
    row_off = np.ascontiguousarray(row_off, dtype=np.int64)
    n_units = row_off.shape[0] - 1
    if prefix_len is not None:
        prefix_len = np.ascontiguousarray(prefix_len, dtype=np.int32)
        assert prefix_len.shape[0] == n_units
    return row_off, prefix_len, n_units


def score(p: Params, row_off, K, Q, n_threads: int = 0) -> np.ndarray:
    row_off, _, n_units = _units(row_off)
    _check_data(p, K, Q)
    total = int(row_off[-1])
    assert K.size == total * p.head_dim
    assert Q.size == n_units * p.window * p.q_per_kv * p.head_dim
    s = np.zeros(total, dtype=np.float32)
    cp = p.c()
    rc = lib().cask_ref_score(C.byref(cp), C.c_int32(n_units), _ptr(row_off), _ptr(K), _ptr(Q),
                              _ptr(s), C.c_int(n_threads))
    if rc:
        raise ValueError(f"cask_ref_score: {rc}")
    return s


def prefix_evict(p: Params, row_off, prefix_len, scores, role=None):
    row_off, prefix_len, n_units = _units(row_off, prefix_len)
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    if role is None:
        role = np.full(int(row_off[-1]), 255, dtype=np.uint8)
    status = np.zeros(n_units, dtype=np.int32)
    cp = p.c()
    rc = lib().cask_ref_prefix_evict(C.byref(cp), C.c_int32(n_units), _ptr(row_off),
                                     _ptr(prefix_len), _ptr(scores), _ptr(role), _ptr(status))
    if rc:
        raise ValueError(f"cask_ref_prefix_evict: {rc}")
    return role, status


def partition(p: Params, row_off, prefix_len, scores, role=None):
    row_off, prefix_len, n_units = _units(row_off, prefix_len)
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    if role is None:
        role = np.full(int(row_off[-1]), 255, dtype=np.uint8)
    status = np.zeros(n_units, dtype=np.int32)
    cp = p.c()
    rc = lib().cask_ref_partition(C.byref(cp), C.c_int32(n_units), _ptr(row_off),
                                  _ptr(prefix_len), _ptr(scores), _ptr(role), _ptr(status))
    if rc:
        raise ValueError(f"cask_ref_partition: {rc}")
    return role, status


def partition_keys(p: Params, row_off, prefix_len, K, scores, role=None):
    """partition, then de-duplicated seeding when p.seed_dedup > 0; returns role, status, min_gap."""
    row_off, prefix_len, n_units = _units(row_off, prefix_len)
    _check_data(p, K)
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    if role is None:
        role = np.full(int(row_off[-1]), 255, dtype=np.uint8)
    status = np.zeros(n_units, dtype=np.int32)
    gap = np.zeros(n_units, dtype=np.float64)
    cp = p.c()
    rc = lib().cask_ref_partition_keys(C.byref(cp), C.c_int32(n_units), _ptr(row_off), _ptr(prefix_len),
                                       _ptr(K), _ptr(scores), _ptr(role), _ptr(status), _ptr(gap))
    if rc:
        raise ValueError(f"cask_ref_partition_keys: {rc}")
    return role, status, gap


def consolidate(p: Params, row_off, prefix_len, K, scores, role, want_sims: bool = False):
    row_off, prefix_len, n_units = _units(row_off, prefix_len)
    _check_data(p, K)
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    role = np.ascontiguousarray(role, dtype=np.uint8)
    total = int(row_off[-1])
    assign = np.full(total, -2, dtype=np.int32)
    best = np.zeros(total, dtype=np.float64) if want_sims else None
    second = np.zeros(total, dtype=np.float64) if want_sims else None
    cp = p.c()
    rc = lib().cask_ref_consolidate(C.byref(cp), C.c_int32(n_units), _ptr(row_off),
                                    _ptr(prefix_len), _ptr(K), _ptr(scores), _ptr(role),
                                    _ptr(assign), _ptr(best), _ptr(second))
    if rc:
        raise ValueError(f"cask_ref_consolidate: {rc}")
    if want_sims:
        return assign, best, second
    return assign


def compress(p: Params, row_off, prefix_len, K, V, Q, scores=None, n_threads: int = 0) -> dict:
    """Whole event.  `scores` given => used as input (scoring skipped)."""
    row_off, prefix_len, n_units = _units(row_off, prefix_len)
    _check_data(p, K, V, Q)
    total = int(row_off[-1])
    d, B = p.head_dim, p.budget
    given = scores is not None
    if given:
        scores = np.ascontiguousarray(scores, dtype=np.float32).copy()
        assert scores.size == total
    else:
        scores = np.zeros(total, dtype=np.float32)
    K_out = np.zeros((n_units, B, d), dtype=_np_elem(p.dtype))
    V_out = np.zeros((n_units, B, d), dtype=_np_elem(p.dtype))
    out_len = np.zeros(n_units, dtype=np.int32)
    out_src = np.full((n_units, B), -1, dtype=np.int32)
    out_mass = np.zeros((n_units, B), dtype=np.float32)
    assign = np.full(total, -2, dtype=np.int32)
    role = np.full(total, 255, dtype=np.uint8)
    status = np.zeros(n_units, dtype=np.int32)
    cp = p.c()
    rc = lib().cask_ref_compress(C.byref(cp), C.c_int32(n_units), _ptr(row_off), _ptr(prefix_len),
                                 _ptr(K), _ptr(V), _ptr(Q), C.c_int(1 if given else 0),
                                 _ptr(scores), _ptr(K_out), _ptr(V_out), _ptr(out_len),
                                 _ptr(out_src), _ptr(out_mass), _ptr(assign), _ptr(role),
                                 _ptr(status), C.c_int(n_threads))
    if rc:
        raise ValueError(f"cask_ref_compress: {rc}")
    return dict(K_out=K_out, V_out=V_out, out_len=out_len, out_src=out_src, out_mass=out_mass,
                assign=assign, role=role, status=status, scores=scores)


def compress_step(p: Params, row_off, prefix_len, K, V, Q, in_count=None, out_stride_rows: int = 0,
                  scores=None, n_threads: int = 0) -> dict:
    """One event of a decode loop: compress() with per-row token counts carried in and out and
    an output row stride (rows [u * stride, u * stride + out_len[u]) of K_out / V_out)."""
    row_off, prefix_len, n_units = _units(row_off, prefix_len)
    _check_data(p, K, V, Q)
    total = int(row_off[-1])
    d, B = p.head_dim, p.budget
    stride = out_stride_rows if out_stride_rows > 0 else B
    given = scores is not None
    if given:
        scores = np.ascontiguousarray(scores, dtype=np.float32).copy()
        assert scores.size == total
    else:
        scores = np.zeros(total, dtype=np.float32)
    if in_count is not None:
        in_count = np.ascontiguousarray(in_count, dtype=np.int32)
        assert in_count.size == total
    K_out = np.zeros((n_units, stride, d), dtype=_np_elem(p.dtype))
    V_out = np.zeros((n_units, stride, d), dtype=_np_elem(p.dtype))
    out_len = np.zeros(n_units, dtype=np.int32)
    out_src = np.full((n_units, B), -1, dtype=np.int32)
    out_mass = np.zeros((n_units, B), dtype=np.float32)
    out_count = np.zeros((n_units, B), dtype=np.int32)
    assign = np.full(total, -2, dtype=np.int32)
    role = np.full(total, 255, dtype=np.uint8)
    status = np.zeros(n_units, dtype=np.int32)
    cp = p.c()
    rc = lib().cask_ref_compress_step(C.byref(cp), C.c_int32(n_units), _ptr(row_off), _ptr(prefix_len),
                                      _ptr(K), _ptr(V), _ptr(Q), C.c_int(1 if given else 0),
                                      _ptr(scores), _ptr(in_count) if in_count is not None else None,
                                      _ptr(K_out), _ptr(V_out), C.c_int32(stride), _ptr(out_len),
                                      _ptr(out_src), _ptr(out_mass), _ptr(out_count), _ptr(assign),
                                      _ptr(role), _ptr(status), C.c_int(n_threads))
    if rc:
        raise ValueError(f"cask_ref_compress_step: {rc}")
    return dict(K_out=K_out, V_out=V_out, out_len=out_len, out_src=out_src, out_mass=out_mass,
                out_count=out_count, assign=assign, role=role, status=status, scores=scores)


def mass_diagnostics(p: Params, row_off, scores, role, out_mass, out_len) -> np.ndarray:
    """(rho_core, rho_rep) per unit, Section 2.6; inputs as returned by compress()."""
    row_off = np.ascontiguousarray(row_off, dtype=np.int64)
    n_units = len(row_off) - 1
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    role = np.ascontiguousarray(role, dtype=np.uint8)
    out_mass = np.ascontiguousarray(out_mass, dtype=np.float32)
    out_len = np.ascontiguousarray(out_len, dtype=np.int32)
    assert out_mass.shape == (n_units, p.budget) and scores.size == int(row_off[-1]) == role.size
    rho = np.zeros((n_units, 2), dtype=np.float32)
    cp = p.c()
    rc = lib().cask_ref_mass_diagnostics(C.byref(cp), C.c_int32(n_units), _ptr(row_off), _ptr(scores),
                                         _ptr(role), _ptr(out_mass), _ptr(out_len), _ptr(rho))
    if rc:
        raise ValueError(f"cask_ref_mass_diagnostics: {rc}")
    return rho


def group_diagnostics(p: Params, row_off, K, scores, assign, K_out):
    """(dispersion, lost_mass) per unit: within-group kappa-dispersion and lost mass of a finished
    event (Section 2.6, Appendix B).  K_out [n_units, stride, d] with stride >= budget."""
    row_off = np.ascontiguousarray(row_off, dtype=np.int64)
    n_units = len(row_off) - 1
    K = np.ascontiguousarray(K)
    K_out = np.ascontiguousarray(K_out)
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    assign = np.ascontiguousarray(assign, dtype=np.int32)
    assert K.dtype == K_out.dtype and K_out.ndim == 3 and K_out.shape[0] == n_units
    assert K_out.shape[2] == p.head_dim and scores.size == assign.size == int(row_off[-1])
    disp = np.zeros(n_units, dtype=np.float32)
    lost = np.zeros(n_units, dtype=np.float32)
    cp = p.c()
    rc = lib().cask_ref_group_diagnostics(C.byref(cp), C.c_int32(n_units), _ptr(row_off), _ptr(K),
                                          _ptr(scores), _ptr(assign), _ptr(K_out),
                                          C.c_int32(K_out.shape[1]), _ptr(disp), _ptr(lost))
    if rc:
        raise ValueError(f"cask_ref_group_diagnostics: {rc}")
    return disp, lost


def attend(p: Params, Q, K_c, V_c, length, count=None) -> np.ndarray:
    """One decode step's attention over a compressed cache with the proportional (ln count)
    bias; Q [n_units, G, d], K_c / V_c [n_units, stride, d], length [n_units], count
    [n_units, pitch] or None.  Returns float64 [n_units, G, d]."""
    Q, K_c, V_c = (np.ascontiguousarray(x) for x in (Q, K_c, V_c))
    n_units = K_c.shape[0]
    assert Q.shape == (n_units, p.q_per_kv, p.head_dim) and K_c.shape == V_c.shape and K_c.shape[2] == p.head_dim
    assert Q.dtype == K_c.dtype == V_c.dtype == _np_elem(p.dtype)
    length = np.ascontiguousarray(length, dtype=np.int32)
    pitch = 0
    if count is not None:
        count = np.ascontiguousarray(count, dtype=np.int32)
        assert count.ndim == 2 and count.shape[0] == n_units
        pitch = count.shape[1]
    out = np.zeros((n_units, p.q_per_kv, p.head_dim), dtype=np.float64)
    cp = p.c()
    rc = lib().cask_ref_attend(C.byref(cp), C.c_int32(n_units), _ptr(Q), _ptr(K_c), _ptr(V_c),
                               C.c_int32(K_c.shape[1]), _ptr(length),
                               _ptr(count) if count is not None else None, C.c_int32(pitch), _ptr(out))
    if rc:
        raise ValueError(f"cask_ref_attend: {rc}")
    return out
