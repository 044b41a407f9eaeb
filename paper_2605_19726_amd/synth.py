"""Seeded synthetic Q, K, V generators for the five benchmark workloads.

This module holds no arithmetic of the attention method itself: it only draws
random tensors with the shapes and coarse value structure of the workloads the
paper evaluates on (diffusion-LM prefill, multimodal LM, video DiT; Sec. 4.1-4.2),
whose data and weights are not available.  Both the HIP path and the CPU checker
are fed from here, so that they see the same rounded values.

Tensors are returned as [1, heads, L, d] in the workload dtype.  Values are drawn
in fp32 on `device` with one torch.Generator per tensor and then rounded to the
workload dtype; the rounded values are the inputs.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Tuple

import torch

BASE_SEED = 1972600


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # seed offset
    kind: str                  # "salient" | "lowrank" | "multimodal" | "video"
    heads_q: int
    heads_kv: int
    L: int
    d: int
    block: int
    dtype: str                 # "f32" | "bf16"
    sparsities: Tuple[float, ...]
    salient_frac: float = 0.0  # fraction of key blocks made salient
    salient_count: int = 0     # absolute count (overrides the fraction when > 0)
    image_side: int = 0        # multimodal: image tokens form image_side^2 grid
    video_thw: Tuple[int, int, int] = (0, 0, 0)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def n_blocks(self) -> int:
        return (self.L + self.block - 1) // self.block

    def scaled(self, name, **kw) -> "Workload":
        return dataclasses.replace(self, name=name, **kw)


# The five configurations of the benchmark, in order.
CONFIGS = (
    Workload("cfg0_tiny_f32", 0, "salient", 1, 1, 1024, 64, 64, "f32", (0.5,), salient_count=3),
    Workload("cfg1_dlm_32k", 1, "lowrank", 32, 32, 32768, 128, 64, "bf16", (0.5,), salient_frac=0.05),
    Workload("cfg2_multimodal_64k", 2, "multimodal", 32, 8, 65536, 128, 128, "bf16", (0.5,),
             image_side=128),
    Workload("cfg3_video_75k", 3, "video", 40, 40, 75600, 128, 128, "bf16", (0.5, 0.75),
             video_thw=(21, 60, 60)),
    Workload("cfg4_dlm_128k", 4, "lowrank", 32, 32, 131072, 128, 128, "bf16",
             (0.0, 0.5, 0.75, 0.9), salient_frac=0.02),
)


def _gen(seed: int, which: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 10 + which)
    return g


def _randn(shape, g, device):
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def _unit(d, g, device):
    u = _randn((d,), g, device)
    return u / u.norm()


def _n_salient(w: Workload) -> int:
    if w.salient_count > 0:
        return w.salient_count
    return int(round(w.salient_frac * (w.L // w.block)))


def _add_salient(q, k, w: Workload, g_aux, device):
    """Shift a few key blocks (original order) and all queries along a shared unit
    direction u, so that block selection is not flat."""
    n_sal = _n_salient(w)
    if n_sal == 0:
        return
    u = _unit(w.d, g_aux, device)
    nb = w.L // w.block
    blocks = torch.randperm(nb, generator=g_aux, device=device)[:n_sal]
    for b in blocks.tolist():
        k[b * w.block:(b + 1) * w.block] += 2.0 * u
    q += 1.0 * u


def _head_salient(w, gq, gk, ga, device):
    q = _randn((w.L, w.d), gq, device)
    k = _randn((w.L, w.d), gk, device)
    _add_salient(q, k, w, ga, device)
    return q, k


def _head_lowrank(w, gq, gk, ga, device):
    rank = 8
    W = _randn((rank, w.d), ga, device) * math.sqrt(1.0 / rank)
    scale = w.d ** 0.25
    q = (_randn((w.L, w.d), gq, device) + 1.5 * (_randn((w.L, rank), gq, device) @ W)) / scale
    k = (_randn((w.L, w.d), gk, device) + 1.5 * (_randn((w.L, rank), gk, device) @ W)) / scale
    _add_salient(q, k, w, ga, device)
    return q, k


def _image_field(w, g, device):
    """Bilinear interpolation of an 8x8 lattice of random d-vectors over an
    image_side x image_side token grid, plus N(0, 0.3) noise."""
    s = w.image_side
    lat = _randn((8, 8, w.d), g, device)
    coord = torch.arange(s, device=device, dtype=torch.float32) * (7.0 / (s - 1))
    i0 = coord.floor().clamp(max=6).long()
    f = coord - i0.float()
    rows0, rows1 = lat[i0], lat[i0 + 1]                      # [s, 8, d]
    rows = rows0 * (1 - f)[:, None, None] + rows1 * f[:, None, None]
    c0, c1 = rows[:, i0], rows[:, i0 + 1]                    # [s, s, d]
    field = c0 * (1 - f)[None, :, None] + c1 * f[None, :, None]
    return field.reshape(s * s, w.d) + 0.3 * _randn((s * s, w.d), g, device)


def _head_multimodal(w, gq, gk, ga, device):
    n_img = w.image_side * w.image_side
    out = []
    for g in (gq, gk):
        img = _image_field(w, g, device)
        txt = _randn((w.L - n_img, w.d), g, device)
        out.append(torch.cat([img, txt], dim=0))
    return out[0], out[1]


def _video_field(w, g, device):
    """Sum of 16 low-frequency cosines over (t, h, w) with random d-vector
    amplitudes (unit total variance), plus N(0, 0.5) noise; t-major token order."""
    T, H, Wd = w.video_thw
    tt = torch.arange(T, device=device, dtype=torch.float32) / T
    hh = torch.arange(H, device=device, dtype=torch.float32) / H
    ww = torch.arange(Wd, device=device, dtype=torch.float32) / Wd
    p = torch.stack(torch.meshgrid(tt, hh, ww, indexing="ij"), dim=-1).reshape(-1, 3)
    n_modes = 16
    freqs = []
    while len(freqs) < n_modes:
        f = torch.randint(0, 4, (3,), generator=g, device=device)
        if int(f.sum()) > 0:
            freqs.append(f)
    F = torch.stack(freqs).float()                                         # [16, 3]
    amp = _randn((n_modes, w.d), g, device) * math.sqrt(1.0 / 8.0)
    phase = torch.rand((n_modes,), generator=g, device=device) * (2 * math.pi)
    basis = torch.cos(2 * math.pi * (p @ F.T) + phase)                     # [L, 16]
    return basis @ amp + 0.5 * _randn((p.shape[0], w.d), g, device)


def _head_video(w, gq, gk, ga, device):
    return _video_field(w, gq, device), _video_field(w, gk, device)


_HEAD_FN = {"salient": _head_salient, "lowrank": _head_lowrank,
            "multimodal": _head_multimodal, "video": _head_video}


def segments_of(w: Workload):
    """Token index at which each natural segment of the workload starts (the image and the text
    of the multimodal sequence, the frames of the video), or None when there is only one."""
    if w.kind == "multimodal" and 0 < w.image_side * w.image_side < w.L:
        return [0, w.image_side * w.image_side]
    if w.kind == "video" and w.video_thw[0] > 1:
        frame = w.video_thw[1] * w.video_thw[2]
        return [t * frame for t in range(w.video_thw[0])]
    return None


def make_qkv(w: Workload, device="cpu"):
    """Return (Q [1,Hq,L,d], K [1,Hkv,L,d], V [1,Hkv,L,d]) for workload `w`.

    Query head h is paired with KV head h // (Hq/Hkv); the shared structure of a
    head (low-rank mixing matrix, salient direction) is drawn per KV head and
    reused by the query heads of its group.
    """
    if w.kind == "video":
        assert w.L == w.video_thw[0] * w.video_thw[1] * w.video_thw[2]
    seed = BASE_SEED + w.index
    gq, gk, gv, ga = (_gen(seed, i, device) for i in range(4))
    dt = w.torch_dtype
    Q = torch.empty((1, w.heads_q, w.L, w.d), dtype=dt, device=device)
    K = torch.empty((1, w.heads_kv, w.L, w.d), dtype=dt, device=device)
    V = torch.empty((1, w.heads_kv, w.L, w.d), dtype=dt, device=device)
    group = w.heads_q // w.heads_kv
    fn = _HEAD_FN[w.kind]
    for hk in range(w.heads_kv):
        aux_state = ga.get_state()
        for j in range(group):
            # same auxiliary draws (mixing matrix, salient blocks) for the whole group
            ga.set_state(aux_state)
            q, k = fn(w, gq, gk, ga, device)
            Q[0, hk * group + j] = q.to(dt)
            if j == 0:
                K[0, hk] = k.to(dt)
        V[0, hk] = _randn((w.L, w.d), gv, device).to(dt)
    return Q, K, V
