"""Thin ctypes binding of libcask.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (torch is used for device
memory and streams, nothing else), passes their raw pointers and the current HIP stream to
the C ABI declared in include/cask.h, and returns the output tensors.  No step of the
compression event is computed here, and there is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcask.so")

F32, BF16 = 0, 1
OK, EINVAL, ENOMEM, EDEVICE = 0, -1, -2, -3
ST_ACTIVE, ST_IDENTITY, ST_PREFIX_BUDGET_EXHAUSTED, ST_MERGE_INACTIVE = 0, 1, 2, 4
PATH_NO_FUSED_TAIL, PATH_NO_FUSED_SCORE, PATH_DEDUP_VECTOR, PATH_ATTEND_VECTOR, PATH_NO_FUSED_SWEEPS = 1, 2, 4, 8, 16
PATH_FORCE_FUSED_SWEEPS = 32
PATH_NARROW_ROWS = 64
PATH_WIDE_ROWS = 128
(ROLE_PREFIX_DROP, ROLE_PREFIX_KEEP, ROLE_CORE, ROLE_SEED, ROLE_DONOR, ROLE_RECENT,
 ROLE_DECODE_EVICT) = range(7)

EXPORTS = ["cask_plan", "cask_workspace_bytes", "cask_score", "cask_prefix_evict",
           "cask_partition", "cask_consolidate", "cask_compress", "cask_compress_static", "cask_compress_step",
           "cask_mass_diagnostics", "cask_group_diagnostics", "cask_attend", "cask_strerror",
           "cask_timing_enable", "cask_timing_enable_stages", "cask_timing_read",
           "cask_probe_issue", "cask_probe_copy", "cask_probe_read"]
STAGES = ["score_rows", "score_cols", "select", "index_roles", "similarity", "gather", "emit"]


class CaskError(RuntimeError):
    def __init__(self, fn: str, code: int):
        self.code = code
        super().__init__(f"{fn} failed: {code} ({_strerror(code)})")


class _Params(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("head_dim", C.c_int32), ("q_per_kv", C.c_int32),
                ("window", C.c_int32), ("recent", C.c_int32), ("budget", C.c_int32),
                ("core", C.c_int32), ("prefix_budget", C.c_int32),
                ("sim_threshold", C.c_float), ("softmax_scale", C.c_float),
                ("causal", C.c_int32), ("scores_given", C.c_int32), ("merge_radius", C.c_int32),
                ("merge_geometry", C.c_int32), ("dist_threshold", C.c_float), ("band_weight", C.c_void_p),
                ("seed_dedup", C.c_int32), ("path_flags", C.c_uint32), ("score_splits", C.c_int32),
                ("score_qsplit", C.c_int32)]


class _Batch(C.Structure):
    _fields_ = [("n_units", C.c_int32), ("row_off", C.c_void_p), ("prefix_len", C.c_void_p),
                ("row_off_host", C.c_void_p), ("prefix_len_host", C.c_void_p),
                ("K", C.c_void_p), ("V", C.c_void_p), ("Q", C.c_void_p)]


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
    band_weight: Optional[torch.Tensor] = None   # geometry 1: device float32 [head_dim / 2], >= 0
    seed_dedup: int = 0            # h > 0: seeds chosen greedily among the best h * M scratch rows
    path_flags: int = 0            # PATH_* bits: kernel choice for measurements and tests
    score_splits: int = 0          # forced key splits of the first scoring sweep (0: the library's choice)
    score_qsplit: int = 0          # forced sharing of a key tile in the second sweep (0: the library's choice)

    def c(self, scores_given: int = 0) -> _Params:
        bw = None
        if self.band_weight is not None:
            t = self.band_weight
            assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == self.head_dim // 2
            bw = t.data_ptr()
        return _Params(self.dtype, self.head_dim, self.q_per_kv, self.window, self.recent,
                       self.budget, self.core, self.prefix_budget, self.sim_threshold,
                       self.softmax_scale, self.causal, scores_given, self.merge_radius,
                       self.merge_geometry, self.dist_threshold, bw, self.seed_dedup,
                       self.path_flags | _env_path_flags(), self.score_splits or _env_int("CASK_SPLITS"),
                       self.score_qsplit or _env_int("CASK_QSPLIT"))


def _env_int(name: str) -> int:
    try:
        return int(os.environ.get(name, "0"))
    except ValueError:
        return 0


def _env_path_flags() -> int:
    """Measurement switches of the Python layer (the library itself reads no environment):
    CASK_FUSED_TAIL=0, CASK_FUSED_SCORE=0, CASK_FUSED_SWEEPS=0, CASK_DEDUP_VECTOR=1,
    CASK_ATTEND_VECTOR=1, CASK_NARROW_ROWS=1, CASK_WIDE_ROWS=1 set the matching PATH_* bit of every call made through this binding."""
    env = os.environ
    f = 0
    if env.get("CASK_FUSED_TAIL", "1")[:1] == "0":
        f |= PATH_NO_FUSED_TAIL
    if env.get("CASK_FUSED_SCORE", "1")[:1] == "0":
        f |= PATH_NO_FUSED_SCORE
    if env.get("CASK_FUSED_SWEEPS", "1")[:1] == "0":
        f |= PATH_NO_FUSED_SWEEPS
    if env.get("CASK_DEDUP_VECTOR", "0")[:1] == "1":
        f |= PATH_DEDUP_VECTOR
    if env.get("CASK_ATTEND_VECTOR", "0")[:1] == "1":
        f |= PATH_ATTEND_VECTOR
    if env.get("CASK_NARROW_ROWS", "0")[:1] == "1":
        f |= PATH_NARROW_ROWS
    if env.get("CASK_WIDE_ROWS", "0")[:1] == "1":
        f |= PATH_WIDE_ROWS
    return f


_lib = None


def load():
    """Load libcask.so (built in-tree by paper_2604_10900_amd.build.build_lib)."""
    global _lib, LIB_PATH
    if _lib is None:
        # CASK_LIB names another build of the same sources to load (the host-sanitizer test)
        LIB_PATH = os.environ.get("CASK_LIB") or LIB_PATH
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -c 'import __graft_entry__ as g; g.build()'`")
        lib = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        # (restype, argtypes) of every entry point include/cask.h declares: without them ctypes
        # would pass a Python int as a 32-bit C int, which truncates a size_t workspace size
        sigs = {
            "cask_plan": (C.c_int, [vp, i32, i32, vp]),
            "cask_workspace_bytes": (sz, [vp, i32, i64, i32]),
            "cask_score": (C.c_int, [vp, vp, vp, vp, sz, vp]),
            "cask_prefix_evict": (C.c_int, [vp, vp, vp, vp, vp, vp, sz, vp]),
            "cask_partition": (C.c_int, [vp, vp, vp, vp, vp, vp, sz, vp]),
            "cask_consolidate": (C.c_int, [vp, vp, vp, vp, vp, vp, sz, vp]),
            "cask_compress": (C.c_int, [vp] * 11 + [sz, vp]),
            "cask_compress_static": (C.c_int, [vp] * 11),
            "cask_compress_step": (C.c_int, [vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
            "cask_mass_diagnostics": (C.c_int, [vp] * 8),
            "cask_group_diagnostics": (C.c_int, [vp, vp, vp, vp, vp, i32, vp, vp, vp]),
            "cask_attend": (C.c_int, [vp, i32, vp, vp, vp, i32, vp, vp, i32, vp, vp]),
            "cask_strerror": (C.c_char_p, [C.c_int]),
            "cask_timing_enable": (C.c_int, [C.c_int]),
            "cask_timing_enable_stages": (C.c_int, [C.c_int, C.c_int]),
            "cask_timing_read": (C.c_int, [vp, vp]),
            "cask_probe_issue": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp]),
            "cask_probe_copy": (C.c_int, [vp, vp, sz, vp]),
            "cask_probe_read": (C.c_int, [vp, sz, vp, C.c_int, vp]),
        }
        assert set(sigs) == set(EXPORTS)
        for name, (res, args) in sigs.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _strerror(code: int) -> str:
    try:
        return load().cask_strerror(code).decode()
    except Exception:  # pragma: no cover
        return "?"


def timing_enable(max_calls: int, n_stages: int = len(STAGES)) -> None:
    """Record the first n_stages stages of the next max_calls compress calls (0 = off)."""
    rc = load().cask_timing_enable_stages(C.c_int(max_calls), C.c_int(n_stages))
    if rc:
        raise CaskError("cask_timing_enable_stages", rc)


def timing_read() -> tuple:
    """(mean milliseconds per stage as a dict, number of recorded compress calls)."""
    ms = (C.c_float * len(STAGES))()
    n = C.c_int(0)
    rc = load().cask_timing_read(ms, C.byref(n))
    if rc:
        raise CaskError("cask_timing_read", rc)
    k = max(n.value, 1)
    return {s: ms[i] / k for i, s in enumerate(STAGES)}, n.value


def plan(p: Params, P: int, N: int) -> dict:
    """Host-side budget split of one unit (cask_plan)."""
    out = _Plan()
    cp = p.c()
    rc = load().cask_plan(C.byref(cp), P, N, C.byref(out))
    if rc:
        raise CaskError("cask_plan", rc)
    return {k: getattr(out, k) for k, _ in _Plan._fields_}


def _dptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor expected"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Batch:
    """Device pointers of one batch plus the host mirrors of its offsets."""

    def __init__(self, p: Params, row_off, prefix_len, K, V=None, Q=None):
        self.params = p
        host_ro = row_off.cpu() if isinstance(row_off, torch.Tensor) else torch.as_tensor(np.asarray(row_off))
        host_pl = prefix_len.cpu() if isinstance(prefix_len, torch.Tensor) else torch.as_tensor(np.asarray(prefix_len))
        self.row_off_host = host_ro.to(torch.int64).contiguous()
        self.prefix_len_host = host_pl.to(torch.int32).contiguous()
        dev = K.device
        self.row_off = (row_off if isinstance(row_off, torch.Tensor) and row_off.is_cuda and row_off.dtype == torch.int64
                        else self.row_off_host.to(dev)).contiguous()
        self.prefix_len = (prefix_len if isinstance(prefix_len, torch.Tensor) and prefix_len.is_cuda and prefix_len.dtype == torch.int32
                           else self.prefix_len_host.to(dev)).contiguous()
        self.n_units = int(self.row_off_host.numel() - 1)
        self.total_rows = int(self.row_off_host[-1]) if self.n_units > 0 else 0
        lens = self.row_off_host[1:] - self.row_off_host[:-1]
        self.max_unit_len = int(lens.max()) if self.n_units > 0 else 0
        want = torch.float32 if p.dtype == F32 else torch.bfloat16
        for t in (K, V, Q):
            if t is not None:
                assert t.dtype == want, (t.dtype, want)
        self.K, self.V, self.Q = K, V, Q
        self.device = dev
        self._ws = None

    def c(self) -> _Batch:
        return _Batch(self.n_units, self.row_off.data_ptr(), self.prefix_len.data_ptr(),
                      self.row_off_host.data_ptr(), self.prefix_len_host.data_ptr(),
                      self.K.data_ptr(), self.V.data_ptr() if self.V is not None else None,
                      self.Q.data_ptr() if self.Q is not None else None)

    def workspace(self) -> torch.Tensor:
        if self._ws is None:
            n = workspace_bytes(self.params, self.n_units, self.total_rows, self.max_unit_len)
            self._ws = torch.empty(max(n, 256), dtype=torch.uint8, device=self.device)
        return self._ws


def workspace_bytes(p: Params, n_units: int, total_rows: int, max_unit_len: int) -> int:
    cp = p.c()
    return int(load().cask_workspace_bytes(C.byref(cp), n_units, total_rows, max_unit_len))


def score(b: Batch, scores: Optional[torch.Tensor] = None) -> torch.Tensor:
    if scores is None:
        scores = torch.empty(b.total_rows, dtype=torch.float32, device=b.device)
    cp, cb, ws = b.params.c(), b.c(), b.workspace()
    rc = load().cask_score(C.byref(cp), C.byref(cb), _dptr(scores), _dptr(ws), ws.numel(), _stream())
    if rc:
        raise CaskError("cask_score", rc)
    return scores


def prefix_evict(b: Batch, scores: torch.Tensor, role: Optional[torch.Tensor] = None):
    if role is None:
        role = torch.full((b.total_rows,), 255, dtype=torch.uint8, device=b.device)
    status = torch.zeros(b.n_units, dtype=torch.int32, device=b.device)
    cp, cb, ws = b.params.c(), b.c(), b.workspace()
    rc = load().cask_prefix_evict(C.byref(cp), C.byref(cb), _dptr(scores), _dptr(role),
                                  _dptr(status), _dptr(ws), ws.numel(), _stream())
    if rc:
        raise CaskError("cask_prefix_evict", rc)
    return role, status


def partition(b: Batch, scores: torch.Tensor, role: Optional[torch.Tensor] = None):
    if role is None:
        role = torch.full((b.total_rows,), 255, dtype=torch.uint8, device=b.device)
    status = torch.zeros(b.n_units, dtype=torch.int32, device=b.device)
    cp, cb, ws = b.params.c(), b.c(), b.workspace()
    rc = load().cask_partition(C.byref(cp), C.byref(cb), _dptr(scores), _dptr(role),
                               _dptr(status), _dptr(ws), ws.numel(), _stream())
    if rc:
        raise CaskError("cask_partition", rc)
    return role, status


def consolidate(b: Batch, scores: torch.Tensor, role: torch.Tensor) -> torch.Tensor:
    assign = torch.full((b.total_rows,), -2, dtype=torch.int32, device=b.device)
    cp, cb, ws = b.params.c(), b.c(), b.workspace()
    rc = load().cask_consolidate(C.byref(cp), C.byref(cb), _dptr(scores), _dptr(role),
                                 _dptr(assign), _dptr(ws), ws.numel(), _stream())
    if rc:
        raise CaskError("cask_consolidate", rc)
    return assign


def compress_step(b: Batch, K_out: torch.Tensor, V_out: torch.Tensor, out: "Outputs",
                  in_count: Optional[torch.Tensor] = None, out_count: Optional[torch.Tensor] = None,
                  scores: Optional[torch.Tensor] = None) -> "Outputs":
    """One event of a decode loop (cask_compress_step).  K_out, V_out: [n_units, stride, d] with
    stride >= budget; out supplies out_len, out_src, out_mass, assign, scores, status."""
    assert K_out.shape == V_out.shape and K_out.dim() == 3 and K_out.shape[0] == b.n_units
    given = scores is not None
    if given:
        out.scores = scores
    cp, cb, ws = b.params.c(1 if given else 0), b.c(), b.workspace()
    rc = load().cask_compress_step(C.byref(cp), C.byref(cb), _dptr(in_count), _dptr(K_out), _dptr(V_out),
                                   C.c_int32(K_out.shape[1]), _dptr(out.out_len), _dptr(out.out_src),
                                   _dptr(out.out_mass), _dptr(out_count), _dptr(out.assign),
                                   _dptr(out.scores), _dptr(out.status), _dptr(ws), ws.numel(), _stream())
    if rc:
        raise CaskError("cask_compress_step", rc)
    return out


def mass_diagnostics(b: Batch, scores: torch.Tensor, role: torch.Tensor, out_mass: torch.Tensor,
                     out_len: torch.Tensor) -> torch.Tensor:
    """[n_units, 2] float: (rho_core, rho_rep) of every unit (cask_mass_diagnostics)."""
    rho = torch.zeros(b.n_units, 2, dtype=torch.float32, device=b.device)
    cp, cb = b.params.c(), b.c()
    rc = load().cask_mass_diagnostics(C.byref(cp), C.byref(cb), _dptr(scores), _dptr(role),
                                      _dptr(out_mass), _dptr(out_len), _dptr(rho), _stream())
    if rc:
        raise CaskError("cask_mass_diagnostics", rc)
    return rho


def group_diagnostics(b: Batch, scores: torch.Tensor, assign: torch.Tensor, K_out: torch.Tensor):
    """(dispersion, lost_mass), each [n_units] float (cask_group_diagnostics).  K_out
    [n_units, stride, d] in the cache dtype, stride >= budget."""
    assert K_out.is_contiguous() and K_out.dim() == 3 and K_out.shape[0] == b.n_units
    disp = torch.zeros(b.n_units, dtype=torch.float32, device=b.device)
    lost = torch.zeros(b.n_units, dtype=torch.float32, device=b.device)
    cp, cb = b.params.c(), b.c()
    rc = load().cask_group_diagnostics(C.byref(cp), C.byref(cb), _dptr(scores), _dptr(assign),
                                       _dptr(K_out), C.c_int32(K_out.shape[1]), _dptr(disp),
                                       _dptr(lost), _stream())
    if rc:
        raise CaskError("cask_group_diagnostics", rc)
    return disp, lost


def attend(p: Params, Q: torch.Tensor, K_c: torch.Tensor, V_c: torch.Tensor, length: torch.Tensor,
           count: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One decode step's attention over a compressed cache (cask_attend): Q [n_units, G, d],
    K_c / V_c [n_units, stride, d], length [n_units] int32, count [n_units, pitch] int32 or None."""
    n_units = K_c.shape[0]
    assert Q.is_contiguous() and K_c.is_contiguous() and V_c.is_contiguous() and K_c.shape == V_c.shape
    assert Q.shape == (n_units, p.q_per_kv, p.head_dim) and K_c.shape[2] == p.head_dim
    assert length.dtype == torch.int32 and length.numel() == n_units
    if count is not None:
        assert count.dtype == torch.int32 and count.dim() == 2 and count.shape[0] == n_units and count.is_contiguous()
    if out is None:
        out = torch.empty_like(Q)
    cp = p.c()
    rc = load().cask_attend(C.byref(cp), C.c_int32(n_units), _dptr(Q), _dptr(K_c), _dptr(V_c),
                            C.c_int32(K_c.shape[1]), _dptr(length), _dptr(count) if count is not None else None,
                            C.c_int32(count.shape[1] if count is not None else 0), _dptr(out), _stream())
    if rc:
        raise CaskError("cask_attend", rc)
    return out


class Outputs:
    """Pre-allocated output tensors of cask_compress for one batch shape."""

    def __init__(self, b: Batch, want_mass: bool = True, want_assign: bool = True,
                 want_scores: bool = True):
        p, dev = b.params, b.device
        dt = torch.float32 if p.dtype == F32 else torch.bfloat16
        self.K_out = torch.zeros(b.n_units, p.budget, p.head_dim, dtype=dt, device=dev)
        self.V_out = torch.zeros(b.n_units, p.budget, p.head_dim, dtype=dt, device=dev)
        self.out_len = torch.zeros(b.n_units, dtype=torch.int32, device=dev)
        self.out_src = torch.full((b.n_units, p.budget), -1, dtype=torch.int32, device=dev)
        self.out_mass = torch.zeros(b.n_units, p.budget, dtype=torch.float32, device=dev) if want_mass else None
        self.assign = torch.full((b.total_rows,), -2, dtype=torch.int32, device=dev) if want_assign else None
        self.scores = torch.zeros(b.total_rows, dtype=torch.float32, device=dev) if want_scores else None
        self.status = torch.zeros(b.n_units, dtype=torch.int32, device=dev)


def compress(b: Batch, out: Optional[Outputs] = None, scores: Optional[torch.Tensor] = None) -> Outputs:
    """One compression event.  `scores` given => used as input and scoring is skipped."""
    if out is None:
        out = Outputs(b)
    given = scores is not None
    if given:
        out.scores = scores
    cp, cb, ws = b.params.c(1 if given else 0), b.c(), b.workspace()
    rc = load().cask_compress(C.byref(cp), C.byref(cb), _dptr(out.K_out), _dptr(out.V_out),
                              _dptr(out.out_len), _dptr(out.out_src), _dptr(out.out_mass),
                              _dptr(out.assign), _dptr(out.scores), _dptr(out.status), _dptr(ws),
                              ws.numel(), _stream())
    if rc:
        raise CaskError("cask_compress", rc)
    return out


STATIC_WORKSPACE_BYTES = 48 << 20


def compress_static(b: Batch, out: Outputs, scores: Optional[torch.Tensor] = None) -> Outputs:
    """cask_compress_static: the event with the library's own fixed workspace (no workspace
    argument, nothing allocated by the call; `out` is allocated by the caller beforehand)."""
    given = scores is not None
    if given:
        out.scores = scores
    cp, cb = b.params.c(1 if given else 0), b.c()
    rc = load().cask_compress_static(C.byref(cp), C.byref(cb), _dptr(out.K_out), _dptr(out.V_out),
                                     _dptr(out.out_len), _dptr(out.out_src), _dptr(out.out_mass),
                                     _dptr(out.assign), _dptr(out.scores), _dptr(out.status), _stream())
    if rc:
        raise CaskError("cask_compress_static", rc)
    return out


def probe_issue(kind: int, waves_per_simd: int = 2, blocks: int = 256, iters: int = 20000) -> dict:
    """cask_probe_issue timed with events: {ms, ghz (shader clock read in the kernel), cycles_per_unit
    (per SIMD), tflops (kinds 0, 1)}."""
    dev = torch.device("cuda", torch.cuda.current_device())
    g = torch.Generator().manual_seed(1)
    ops = (torch.rand(16384, generator=g) * 2 - 1).to(torch.bfloat16).to(dev)
    cyc = torch.zeros(2 * blocks, dtype=torch.int64, device=dev)
    sink = torch.empty(blocks * 256 * waves_per_simd, dtype=torch.float32, device=dev)
    lib = load()

    def run(n):
        rc = lib.cask_probe_issue(kind, waves_per_simd, blocks, n, _dptr(ops), _dptr(cyc), _dptr(sink), _stream())
        if rc:
            raise CaskError("cask_probe_issue", rc)
    run(iters)      # warm-up of the same length: the clock settles while it runs
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    run(iters)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    c = cyc.cpu().numpy().reshape(-1, 2).astype(np.float64)
    ghz = float(c[:, 0].sum() / c[:, 1].sum() * 0.1)
    units = iters * 8.0
    # cycles per unit and SIMD from the wall time and the clock: the waves of a SIMD do not finish
    # together (the oldest ready wave is served first), so one wave's own cycle count says little
    rounds = -(-blocks // 256)          # workgroups beyond one per compute unit queue up
    res = dict(ms=ms, ghz=ghz, cycles_per_unit=ms * 1e6 * ghz / (units * waves_per_simd * rounds))
    if kind != 2:
        res["tflops"] = blocks * 4 * waves_per_simd * units * 32768.0 / (ms * 1e-3) / 1e12
    return res


def probe_copy(n_bytes: int = 1 << 30, reps: int = 5) -> dict:
    """cask_probe_copy timed with events: GB/s counting the bytes read plus the bytes written."""
    dev = torch.device("cuda", torch.cuda.current_device())
    src = torch.empty(n_bytes, dtype=torch.uint8, device=dev).random_(0, 256)
    dst = torch.empty_like(src)
    lib = load()

    def run():
        rc = lib.cask_probe_copy(_dptr(src), _dptr(dst), n_bytes, _stream())
        if rc:
            raise CaskError("cask_probe_copy", rc)
    run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    ok = bool(torch.equal(src[:4096], dst[:4096]) and torch.equal(src[-4096:], dst[-4096:]))
    return dict(ms=ms, gbs=2.0 * n_bytes / (ms * 1e-3) / 1e9, bytes=n_bytes, verified=ok)


def probe_read(n_bytes: int = 1 << 30, blocks: int = 512, reps: int = 5) -> dict:
    """cask_probe_read timed with events: GB/s of a read-only stream."""
    dev = torch.device("cuda", torch.cuda.current_device())
    src = torch.empty(n_bytes, dtype=torch.uint8, device=dev).random_(0, 256)
    sink = torch.empty(blocks * 256, dtype=torch.int32, device=dev)
    lib = load()

    def run():
        rc = lib.cask_probe_read(_dptr(src), n_bytes, _dptr(sink), blocks, _stream())
        if rc:
            raise CaskError("cask_probe_read", rc)
    run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    return dict(ms=ms, gbs=n_bytes / (ms * 1e-3) / 1e9, bytes=n_bytes, blocks=blocks)
