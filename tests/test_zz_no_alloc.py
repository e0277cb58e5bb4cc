"""cask_compress_static (the entry point that allocates nothing: its workspace is a fixed array
in device memory owned by the library) against cask_compress, through the C ABI.  Both run the
same kernels, so every output must be identical bit for bit; two calls in a row, the second on
a smaller batch, show that what the first left in the array does no harm."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2604_10900_amd as cask  # noqa: E402
from synth import caches  # noqa: E402
from tests import parity  # noqa: E402

FIELDS = ("K_out", "V_out", "out_len", "out_src", "out_mass", "assign", "scores", "status")


def _same(a: cask.Outputs, b: cask.Outputs, label):
    for f in FIELDS:
        x, y = getattr(a, f), getattr(b, f)
        assert torch.equal(x.view(torch.uint8) if x.dtype == torch.bfloat16 else x,
                           y.view(torch.uint8) if y.dtype == torch.bfloat16 else y), (label, f)


def _raw_call(b: cask.Batch, out: cask.Outputs) -> int:
    """The C ABI itself, no binding function in between."""
    lib = cask.load()
    cp, cb = b.params.c(0), b.c()
    vp = lambda t: C.c_void_p(t.data_ptr())  # noqa: E731
    return lib.cask_compress_static(C.byref(cp), C.byref(cb), vp(out.K_out), vp(out.V_out), vp(out.out_len),
                                    vp(out.out_src), vp(out.out_mass), vp(out.assign), vp(out.scores),
                                    vp(out.status), C.c_void_p(torch.cuda.current_stream().cuda_stream))


def test_static_workspace_event_equals_the_workspace_argument_event():
    big = caches.scaled(caches.WORKLOADS["cfg2"], n_layers=2, n_kv_heads=3, prefix=200, decode=5000, budget=384)
    small = caches.scaled(caches.WORKLOADS["cfg2"], n_layers=1, n_kv_heads=2, prefix=64, decode=1400, budget=384)
    short = caches.scaled(caches.WORKLOADS["cfg2"], n_layers=1, n_kv_heads=4, prefix=96, decode=416, budget=384)
    for i, (w, tau) in enumerate(((big, 0.5), (small, -1.0), (short, 0.3), (big, 0.9))):
        c = caches.make(w, seed=40 + i)
        p = parity.params_of(w, sim_threshold=tau)
        b = parity.to_device(c, p)
        want = cask.compress(b)                       # workspace argument (allocated by the binding)
        got = cask.Outputs(b)
        assert _raw_call(b, got) == cask.binding.OK
        torch.cuda.synchronize()
        _same(got, want, (i, "first"))
        # again into fresh outputs: same bits (the array keeps the last call's contents)
        got2 = cask.Outputs(b)
        cask.compress_static(b, got2)
        torch.cuda.synchronize()
        _same(got2, want, (i, "second"))
        # injected scores take the same route
        got3 = cask.Outputs(b)
        cask.compress_static(b, got3, scores=want.scores.clone())
        want3 = cask.compress(b, scores=want.scores.clone())
        torch.cuda.synchronize()
        _same(got3, want3, (i, "given"))
        assert int((want.status == 0).sum()) > 0 or tau > 0.8


def test_static_workspace_refuses_what_does_not_fit():
    """A batch whose workspace exceeds the fixed array is refused on the host (nothing runs);
    the sizes come from the host mirrors, so the data pointers are never touched."""
    p = cask.Params(q_per_kv=7, budget=384)
    n_units, N = 112, 33024
    assert cask.workspace_bytes(p, n_units, n_units * N, N) > cask.binding.STATIC_WORKSPACE_BYTES
    ro = torch.arange(n_units + 1, dtype=torch.int64) * N
    K = torch.zeros(256, 128, dtype=torch.bfloat16, device="cuda:0")      # far too small: never read
    b = cask.Batch(p, ro, torch.zeros(n_units, dtype=torch.int32), K, K, K)
    b.total_rows = 16                                                      # keeps Outputs small
    out = cask.Outputs(b)
    with pytest.raises(cask.CaskError) as e:
        cask.compress_static(b, out)
    assert e.value.code == cask.binding.ENOMEM
    # and an ordinary call still works afterwards
    w = caches.scaled(caches.WORKLOADS["cfg2"], n_layers=1, n_kv_heads=1, prefix=10, decode=700, budget=300)
    c = caches.make(w, seed=3)
    pb = parity.params_of(w)
    bb = parity.to_device(c, pb)
    got = cask.Outputs(bb)
    cask.compress_static(bb, got)
    torch.cuda.synchronize()
    _same(got, cask.compress(bb), "after a refusal")
