"""Seeded synthetic KV caches shaped like 7B/8B reasoning-model workloads.

This module only draws inputs: Gaussian keys/values with a few outlier channels, rotary
position embedding applied to keys and queries, planted clusters of near-duplicate tokens in
the decode span, and window queries.  It holds none of the compression method's arithmetic
and is the only code shared by the CPU oracle's tests and the HIP library's tests/benchmark.

Units are ordered (sequence, layer, kv_head).  Every (sequence, layer) group draws from its
own generator seeded from (seed, workload id, sequence, layer), so any group can be
regenerated alone and the result does not depend on which other groups are generated.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

BASE_SEED = 0xCA5C


@dataclass(frozen=True)
class Workload:
    name: str
    wid: int                      # enters the seed
    n_seqs: int
    n_layers: int
    n_kv_heads: int
    q_per_kv: int                 # G
    head_dim: int                 # d
    dtype: str                    # "f32" | "bf16"
    prefix: int                   # P (same for every sequence)
    decode: int                   # D, or the lower bound when decode_hi is set
    decode_hi: Optional[int]      # ragged: D ~ U{decode..decode_hi} per sequence
    window: int                   # W
    budget: int                   # B
    core: int = -1                # C (<0: library default)
    recent: int = -1              # R (<0: W)
    rope_theta: Optional[float] = 1.0e6
    outlier_channels: int = 4
    outlier_scale: float = 8.0
    cluster_frac: float = 0.20    # share of decode tokens that are planted near-duplicates
    cluster_lo: int = 4
    cluster_hi: int = 16
    cluster_sigma: float = 0.05
    cluster_span: int = 256       # members sit within this many positions after the anchor
    fixed_clusters: Optional[int] = None   # cfg1: exactly this many clusters, fresh bases
    q_shared_bias: bool = True    # q = b + z with b shared by the unit's window rows

    @property
    def n_units(self) -> int:
        return self.n_seqs * self.n_layers * self.n_kv_heads

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


WORKLOADS: Dict[str, Workload] = {
    # 1 layer, 1 KV head, fp32, 64 prefix + 1024 decode, 32 clusters of 8, budget 256 / core 128
    "cfg1": Workload("cfg1", 1, 1, 1, 1, 1, 64, "f32", 64, 1024, None, 32, 256, core=128,
                     recent=32, rope_theta=None, outlier_channels=0, cluster_lo=8, cluster_hi=8,
                     fixed_clusters=32, q_shared_bias=False),
    # Qwen2.5-7B shape: 28 layers x 4 KV heads, G = 7, d = 128, bf16
    "cfg2": Workload("cfg2", 2, 1, 28, 4, 7, 128, "bf16", 256, 8192, None, 128, 384),
    "cfg3": Workload("cfg3", 3, 1, 28, 4, 7, 128, "bf16", 256, 32768, None, 128, 512),
    "cfg4": Workload("cfg4", 4, 1, 28, 4, 7, 128, "bf16", 16384, 2048, None, 128, 2048),
    "cfg4v": Workload("cfg4v", 5, 1, 28, 4, 7, 128, "bf16", 65536, 2048, None, 128, 1024),
    # Llama-3-8B shape: 32 layers x 8 KV heads, G = 4, 64 ragged sequences
    "cfg5": Workload("cfg5", 6, 64, 32, 8, 4, 128, "bf16", 512, 4096, 32768, 128, 384),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller shapes for tests)."""
    return dataclasses.replace(w, **kw)


def decode_lengths(w: Workload, seed: int = BASE_SEED) -> List[int]:
    if w.decode_hi is None:
        return [w.decode] * w.n_seqs
    g = torch.Generator(device="cpu")
    g.manual_seed((seed * 1000003 + w.wid * 7919 + 17) & 0x7FFFFFFFFFFF)
    return torch.randint(w.decode, w.decode_hi + 1, (w.n_seqs,), generator=g).tolist()


def _group_seed(seed: int, wid: int, seq: int, layer: int) -> int:
    x = (seed & 0xFFFFFFFF) * 0x9E3779B1 + wid * 0x85EBCA77 + seq * 0xC2B2AE3D + layer * 0x27D4EB2F + 1
    return x & 0x7FFFFFFFFFFFFFFF


def _rope(x: torch.Tensor, pos: torch.Tensor, theta: float) -> torch.Tensor:
    """Rotary embedding, half-split pairing (c, c + d/2); x: [..., T, d] float32, pos: [T]."""
    d = x.shape[-1]
    half = d // 2
    f = torch.arange(half, device=x.device, dtype=torch.float64)
    omega = theta ** (-2.0 * f / d)
    ang = pos.to(torch.float64)[:, None] * omega[None, :]
    cos, sin = torch.cos(ang).to(torch.float32), torch.sin(ang).to(torch.float32)
    a, b = x[..., :half], x[..., half:]
    return torch.cat([a * cos - b * sin, b * cos + a * sin], dim=-1)


def _plant(w: Workload, K: torch.Tensor, V: torch.Tensor, P: int, N: int, g: torch.Generator):
    """Overwrite some decode rows of K, V ([H, N, d] float32, already in cache space) with
    near-duplicates of an anchor.  Later clusters win where two claim one position."""
    H, _, d = K.shape
    dev = K.device
    D = N - P
    if D < 2 or w.cluster_frac <= 0:
        return
    if w.fixed_clusters is not None:
        # fresh bases, members at distinct uniformly drawn decode positions
        nc, size = w.fixed_clusters, w.cluster_hi
        if nc * size > D:
            nc = max(D // size, 0)
        if nc == 0:
            return
        perm = torch.rand(H, D, generator=g, device=dev).argsort(dim=1)[:, : nc * size] + P
        base_k = torch.randn(H, nc, 1, d, generator=g, device=dev)
        base_v = torch.randn(H, nc, 1, d, generator=g, device=dev)
        nk = base_k + w.cluster_sigma * torch.randn(H, nc, size, d, generator=g, device=dev)
        nv = base_v + w.cluster_sigma * torch.randn(H, nc, size, d, generator=g, device=dev)
        idx = perm.reshape(H, nc * size, 1).expand(-1, -1, d)
        K.scatter_(1, idx, nk.reshape(H, nc * size, d))
        V.scatter_(1, idx, nv.reshape(H, nc * size, d))
        return
    span = min(w.cluster_span, D - 1)
    hi = min(w.cluster_hi, span)
    lo = min(w.cluster_lo, hi)
    mean_size = 0.5 * (lo + hi)
    nc = int(round(w.cluster_frac * D / mean_size))
    if nc == 0:
        return
    sizes = torch.randint(lo, hi + 1, (H, nc), generator=g, device=dev)
    anchors = torch.randint(P, N - span, (H, nc), generator=g, device=dev)
    offs = torch.rand(H, nc, span, generator=g, device=dev).argsort(dim=2)[:, :, :hi] + 1
    # the anchor is one of the cluster's tokens: size-1 further members
    member = torch.arange(hi, device=dev)[None, None, :] < (sizes[:, :, None] - 1)
    pos = anchors[:, :, None] + offs                       # [H, nc, hi]
    flat_id = torch.arange(nc * hi, device=dev).reshape(1, nc, hi).expand(H, -1, -1)
    # deterministic winner per position: the largest member id
    win = torch.full((H, N), -1, dtype=torch.long, device=dev)
    cand = torch.where(member, flat_id, torch.full_like(flat_id, -1))
    win.scatter_reduce_(1, pos.reshape(H, -1), cand.reshape(H, -1), reduce="amax")
    keep = member & (win.gather(1, pos.reshape(H, -1)).reshape(H, nc, hi) == flat_id)
    hh, cc, mm = keep.nonzero(as_tuple=True)
    src = anchors[hh, cc]
    dst = pos[hh, cc, mm]
    nk = K[hh, src] + w.cluster_sigma * torch.randn(hh.shape[0], d, generator=g, device=dev)
    nv = V[hh, src] + w.cluster_sigma * torch.randn(hh.shape[0], d, generator=g, device=dev)
    K[hh, dst] = nk
    V[hh, dst] = nv


def _make_group(w: Workload, seed: int, seq: int, layer: int, D: int, device):
    """K, V: [H, N, d]; Q: [H, W, G, d] in the workload's dtype for one (sequence, layer)."""
    H, d, G, W = w.n_kv_heads, w.head_dim, w.q_per_kv, w.window
    P = w.prefix
    N = P + D
    g = torch.Generator(device=device)
    g.manual_seed(_group_seed(seed, w.wid, seq, layer))
    K = torch.randn(H, N, d, generator=g, device=device)
    V = torch.randn(H, N, d, generator=g, device=device)
    if w.outlier_channels > 0:
        ch = torch.rand(H, d, generator=g, device=device).argsort(dim=1)[:, : w.outlier_channels]
        gain = torch.ones(H, d, device=device)
        gain.scatter_(1, ch, w.outlier_scale)
        K = K * gain[:, None, :]
    if w.rope_theta is not None:
        K = _rope(K, torch.arange(N, device=device), w.rope_theta)
    _plant(w, K, V, P, N, g)
    Q = torch.randn(H, W, G, d, generator=g, device=device)
    if w.q_shared_bias:
        Q = Q + torch.randn(H, 1, 1, d, generator=g, device=device)
    if w.rope_theta is not None:
        qpos = torch.arange(N - W, N, device=device)
        Q = _rope(Q.permute(0, 2, 1, 3), qpos, w.rope_theta).permute(0, 2, 1, 3)
    dt = w.torch_dtype
    return K.to(dt), V.to(dt), Q.contiguous().to(dt)


def make(w: Workload, seed: int = BASE_SEED, device="cpu", seqs: Optional[Sequence[int]] = None,
         layers: Optional[Sequence[int]] = None) -> dict:
    """Generate the cache of a workload (or of a subset of its sequences / layers).

    Returns K, V: [total_rows, d]; Q: [n_units, W, G, d]; row_off: int64 [n_units + 1];
    prefix_len: int32 [n_units]; units: list of (seq, layer, head)."""
    device = torch.device(device)
    seqs = list(range(w.n_seqs)) if seqs is None else list(seqs)
    layers = list(range(w.n_layers)) if layers is None else list(layers)
    dlen = decode_lengths(w, seed)
    H, d = w.n_kv_heads, w.head_dim
    lens: List[int] = []
    units = []
    for s in seqs:
        for l in layers:
            for h in range(H):
                lens.append(w.prefix + dlen[s])
                units.append((s, l, h))
    row_off = np.zeros(len(lens) + 1, dtype=np.int64)
    row_off[1:] = np.cumsum(np.asarray(lens, dtype=np.int64))
    total = int(row_off[-1])
    K = torch.empty(total, d, dtype=w.torch_dtype, device=device)
    V = torch.empty(total, d, dtype=w.torch_dtype, device=device)
    Q = torch.empty(len(lens), w.window, w.q_per_kv, d, dtype=w.torch_dtype, device=device)
    u = 0
    for s in seqs:
        N = w.prefix + dlen[s]
        for l in layers:
            k, v, q = _make_group(w, seed, s, l, dlen[s], device)
            r0 = int(row_off[u])
            K[r0: r0 + H * N] = k.reshape(H * N, d)
            V[r0: r0 + H * N] = v.reshape(H * N, d)
            Q[u: u + H] = q
            u += H
    return dict(K=K, V=V, Q=Q, row_off=torch.from_numpy(row_off).to(device),
                prefix_len=torch.full((len(lens),), w.prefix, dtype=torch.int32, device=device),
                units=units, workload=w)


def host_bits(t: torch.Tensor) -> np.ndarray:
    """Host numpy view of a tensor for the oracle: bf16 as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
