"""Seeded synthetic inputs for the tests and the benchmark.

This module only draws numbers and names workloads; it holds none of the
method's arithmetic (no masks, no softmax, no recall) and is the only code the
CPU oracle's callers and the GPU path's callers share.

Workloads stand in for the activations of the video DiTs the paper evaluates
(Sec. 4.1: HunyuanVideo, OpenSoraPlan-1.2, CogVideoX-5B); only their shapes
are used.  Values are i.i.d. N(0,1)/sqrt(D) rounded to bf16, or the "planted"
heads below whose attention is concentrated on one of the three structures of
Sec. 3.2 so that the ARM has something to recognise.
"""
from dataclasses import dataclass, field
from typing import Tuple

import torch

SPATIAL, TEMPORAL, TEXTURAL, DENSE = 0, 1, 2, 3


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    nH: int
    D: int
    T: int
    H: int
    W: int
    text_len: int
    block: int
    seed: int
    planted: Tuple[int, ...] = field(default=())  # planted class per head (round robin) or ()

    @property
    def HW(self):
        return self.H * self.W

    @property
    def Nv(self):
        return self.T * self.H * self.W

    @property
    def N(self):
        return self.Nv + self.text_len

    def dense_flops(self):
        """4*N^2*D multiply-adds-as-two flops for QK^T and PV, all heads."""
        return 4.0 * self.N * self.N * self.D * self.nH * self.B


WORKLOADS = {
    # tiny oracle case
    "tiny": Workload("tiny", 1, 2, 64, 4, 8, 8, 0, 64, 1001),
    # CogVideoX-5B-shaped layer, 226 text tokens
    "cogvideox": Workload("cogvideox", 1, 48, 64, 13, 30, 45, 226, 256, 1002),
    # Open-Sora-Plan-1.2 720p-shaped layer
    "osp720p": Workload("osp720p", 1, 24, 96, 24, 45, 80, 0, 384, 1003),
    # HunyuanVideo 720p-shaped layer, 256 text tokens (headline)
    "hunyuan720p": Workload("hunyuan720p", 1, 24, 128, 33, 45, 80, 256, 384, 1004),
    # planted-structure ARM validation
    "planted": Workload("planted", 2, 16, 128, 16, 32, 32, 0, 128, 1005,
                        planted=(SPATIAL, TEMPORAL, TEXTURAL)),
    # the headline shape with planted heads, so that the ARM picks all three patterns there
    "hunyuan720p_planted": Workload("hunyuan720p_planted", 1, 24, 128, 33, 45, 80, 256, 384, 1009,
                                    planted=(SPATIAL, TEMPORAL, TEXTURAL)),
    # small ragged shapes for parity sweeps: frames not block aligned, ragged tail, text
    "ragged64": Workload("ragged64", 1, 3, 64, 5, 6, 11, 19, 64, 1006),
    "ragged96": Workload("ragged96", 1, 3, 96, 6, 9, 10, 37, 128, 1007),
    "ragged128": Workload("ragged128", 2, 3, 128, 7, 10, 13, 50, 128, 1008),
}


def _gen(seed, tensor_id, b, h):
    g = torch.Generator(device="cpu")
    g.manual_seed((seed * 1000003 + tensor_id * 7919 + b * 104729 + h * 1299709) % (2**63 - 1))
    return g


def planted_class(w: Workload, b: int, h: int) -> int:
    """Which structure head (b, h) of a planted workload is built around."""
    return w.planted[(b * w.nH + h) % len(w.planted)]


def head_qkv(w: Workload, b: int, h: int, scale: float = 1.0):
    """Q, K, V of one head as bf16 tensors [N, D] on the CPU.

    i.i.d. workloads: N(0,1)/sqrt(D) (times ``scale`` on Q, to make the softmax peaky).
    Planted workloads: q_n = k_n = g * R[:, code(n)] + N(0, 0.1^2), V ~ N(0,1), where R
    is a seeded random orthogonal matrix and code(n) is the frame (Spatial), the in-frame
    group of consecutive positions (Temporal; groups of 16, or as many as it takes for the
    number of groups to fit D) or the in-frame index mod 64 (Textural).
    """
    N, D = w.N, w.D
    if not w.planted:
        q = torch.randn(N, D, generator=_gen(w.seed, 0, b, h)) * (scale / D ** 0.5)
        k = torch.randn(N, D, generator=_gen(w.seed, 1, b, h)) / D ** 0.5
        v = torch.randn(N, D, generator=_gen(w.seed, 2, b, h)) / D ** 0.5
        return q.bfloat16(), k.bfloat16(), v.bfloat16()
    cls = planted_class(w, b, h)
    n = torch.arange(N)
    f, p = n // w.HW, n % w.HW
    if cls == SPATIAL:
        code = f
    elif cls == TEMPORAL:
        code = p // max(16, -(-w.HW // D))
    else:
        code = p % 64
    assert int(code.max()) < D
    R, _ = torch.linalg.qr(torch.randn(D, D, generator=_gen(w.seed, 3, b, h)))
    gain = (10.0 * D ** 0.5) ** 0.5
    base = gain * R[:, code].T  # [N, D]
    q = base + 0.1 * torch.randn(N, D, generator=_gen(w.seed, 0, b, h))
    k = base + 0.1 * torch.randn(N, D, generator=_gen(w.seed, 1, b, h))
    v = torch.randn(N, D, generator=_gen(w.seed, 2, b, h))
    return q.bfloat16(), k.bfloat16(), v.bfloat16()


def full_qkv(w: Workload, device="cpu", scale: float = 1.0):
    """Q, K, V as bf16 tensors [B, nH, N, D] on ``device``, head by head from head_qkv."""
    out = [torch.empty(w.B, w.nH, w.N, w.D, dtype=torch.bfloat16, device=device) for _ in range(3)]
    for b in range(w.B):
        for h in range(w.nH):
            for t, x in zip(out, head_qkv(w, b, h, scale)):
                t[b, h].copy_(x)
    return out


def round_robin_classes(w: Workload):
    """Spatial/Temporal/Textural by head index, as an int32 tensor [B, nH]."""
    return (torch.arange(w.B * w.nH, dtype=torch.int32) % 3).reshape(w.B, w.nH)


def thirds_classes(w: Workload):
    """First third of the heads Spatial, second Temporal, last Textural."""
    per = (w.nH + 2) // 3
    c = torch.clamp(torch.arange(w.nH, dtype=torch.int32) // per, max=2)
    return c.repeat(w.B, 1).contiguous()


def sample_rows(w: Workload, per_head: int, seed: int = 0):
    """Query rows worth checking one by one at sizes the oracle cannot sweep: first and
    last rows, frame boundaries, block tails, text rows, plus seeded random rows."""
    N, HW, blk = w.N, w.HW, w.block
    must = {0, 1, N - 1, N - 2, HW - 1, HW, w.Nv - 1, (N // blk) * blk - 1, min(N - 1, (N // blk) * blk),
            (w.T // 2) * HW, (w.T // 2) * HW + HW // 2, w.Nv - HW}
    if w.text_len:
        must |= {w.Nv, w.Nv + w.text_len // 2}
    must = sorted(r for r in must if 0 <= r < N)
    g = torch.Generator().manual_seed(w.seed * 31 + seed)
    extra = torch.randint(0, N, (max(0, per_head - len(must)),), generator=g).tolist()
    return sorted(set(must + extra))
