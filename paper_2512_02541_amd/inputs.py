"""Seeded synthetic inputs shaped like the paper's VGGT workloads.

This module holds no arithmetic of the method: it only draws Q/K/V tensors and
names the workload geometries.  Both the GPU library's tests/benchmark and the
CPU oracle's tests take their inputs from here, so both sides see identical bits
(tensors generated on one device are copied, never regenerated, when the other
side needs them).

Random numbers come from a counter-based generator: element ``i`` of stream
``(seed, tensor_id)`` is ``BoxMuller(hash(i, key1), hash(i, key2))`` with a
32-bit integer avalanche hash, evaluated with torch integer ops on whichever
device is asked for, then rounded to bf16 (round-to-nearest-even).

Workloads (AVGGT paper: VGGT token geometry of Sec. 4.1 -- 5 special tokens per
frame -- at the frame counts of its 100/300/800-frame regimes and its 333-frame
7-Scenes setting; the sigma -> stride table of Sec. 4.3):

* ``tiny``  : 2 frames x (16x16 + 5), i.i.d. N(0,1), strides (2,2).
* ``f100``  : 100 frames x (37x37 + 5), structured, strides (1,2).
* ``f300``  : 300 frames, structured, strides (2,2).
* ``f333``  : 333 frames, structured, strides (2,2).
* ``f800``  : 800 frames, structured, strides (3,3).

"Structured" means: a per-slot, per-head pattern ``A_K, A_V ~ N(0,1)`` shared by
every frame, plus per-frame noise of standard deviation 0.5; Q shares K's
pattern (``Q = A_K + 0.5 eps``) so that a query matches the same grid position in
other views -- the cross-view structure the paper reports for the middle global
layers (Sec. 3.1).
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

_M32 = 0xFFFFFFFF


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    N: int
    n_h: int
    n_w: int
    n_special: int
    H: int
    D: int
    s_h: int
    s_w: int
    keep_first_frame: int
    seed: int
    structured: bool

    @property
    def L(self) -> int:
        return self.n_special + self.n_h * self.n_w

    @property
    def NQ(self) -> int:
        return self.N * self.L


WORKLOADS = {
    "tiny": Workload("tiny", 1, 2, 16, 16, 5, 16, 64, 2, 2, 1, 1001, False),
    "f100": Workload("f100", 1, 100, 37, 37, 5, 16, 64, 1, 2, 1, 1100, True),
    "f300": Workload("f300", 1, 300, 37, 37, 5, 16, 64, 2, 2, 1, 1300, True),
    "f333": Workload("f333", 1, 333, 37, 37, 5, 16, 64, 2, 2, 1, 1333, True),
    "f800": Workload("f800", 1, 800, 37, 37, 5, 16, 64, 3, 3, 1, 1800, True),
}


def _avalanche(x: torch.Tensor) -> torch.Tensor:
    """32-bit integer finaliser on int64 lanes holding values in [0, 2^32)."""
    x = x ^ (x >> 16)
    x = (x * 0x7FEB352D) & _M32
    x = x ^ (x >> 15)
    x = (x * 0x846CA68B) & _M32
    x = x ^ (x >> 16)
    return x


def _stream_key(seed: int, tensor_id: int, lane: int) -> int:
    k = (seed * 0x9E3779B1 + tensor_id * 0x85EBCA77 + lane * 0xC2B2AE3D + 0x27D4EB2F) & _M32
    # one scalar avalanche round so nearby seeds give unrelated keys
    k ^= k >> 16
    k = (k * 0x7FEB352D) & _M32
    k ^= k >> 15
    k = (k * 0x846CA68B) & _M32
    k ^= k >> 16
    return k


def normal_stream(seed: int, tensor_id: int, start: int, count: int, device) -> torch.Tensor:
    """``count`` standard normals (float32) for counters ``start .. start+count-1``."""
    ctr = torch.arange(start, start + count, dtype=torch.int64, device=device)
    lo = ctr & _M32
    hi = _avalanche((ctr >> 32) & _M32)
    k1 = _stream_key(seed, tensor_id, 1)
    k2 = _stream_key(seed, tensor_id, 2)
    h1 = _avalanche(_avalanche(lo ^ k1) ^ hi)
    h2 = _avalanche(_avalanche(lo ^ k2) ^ hi)
    u1 = (h1.to(torch.float32) + 1.0) * (1.0 / 4294967296.0)
    u1 = torch.clamp(u1, min=2.0 ** -32, max=1.0)
    u2 = h2.to(torch.float32) * (1.0 / 4294967296.0)
    r = torch.sqrt(-2.0 * torch.log(u1))
    return r * torch.cos(6.283185307179586 * u2)


def normal_tensor(shape, seed: int, tensor_id: int, device, chunk: int = 1 << 25) -> torch.Tensor:
    """float32 tensor of i.i.d. N(0,1), generated in bounded chunks."""
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, dtype=torch.float32, device=device)
    for start in range(0, n, chunk):
        c = min(chunk, n - start)
        out[start:start + c] = normal_stream(seed, tensor_id, start, c, device)
    return out.view(*shape)


def iid_qkv(B: int, NQ: int, H: int, D: int, seed: int, device="cpu"):
    """Q, K, V ~ N(0,1) i.i.d., bf16, layout [B, NQ, H, D]."""
    return tuple(
        normal_tensor((B, NQ, H, D), seed, tid, device).to(torch.bfloat16) for tid in (0, 1, 2)
    )


def structured_qkv(B: int, N: int, L: int, H: int, D: int, seed: int, device="cpu",
                   noise: float = 0.5, frames_per_chunk: int = 16):
    """Shared per-slot pattern plus per-frame noise; bf16, layout [B, N*L, H, D]."""
    a_k = normal_tensor((1, 1, L, H, D), seed, 10, device)
    a_v = normal_tensor((1, 1, L, H, D), seed, 11, device)
    per_frame = L * H * D
    outs = []
    for tid, pat in ((0, a_k), (1, a_k), (2, a_v)):
        t = torch.empty((B, N, L, H, D), dtype=torch.bfloat16, device=device)
        for b in range(B):
            for f0 in range(0, N, frames_per_chunk):
                f1 = min(N, f0 + frames_per_chunk)
                start = (b * N + f0) * per_frame
                eps = normal_stream(seed, tid, start, (f1 - f0) * per_frame, device)
                t[b, f0:f1] = (pat[0] + noise * eps.view(f1 - f0, L, H, D)).to(torch.bfloat16)
        outs.append(t.view(B, N * L, H, D))
    return tuple(outs)


def make_qkv(w: Workload, device="cpu"):
    if w.structured:
        return structured_qkv(w.B, w.N, w.L, w.H, w.D, w.seed, device)
    return iid_qkv(w.B, w.NQ, w.H, w.D, w.seed, device)


def bf16_bits(t: torch.Tensor):
    """bf16 tensor -> numpy uint16 bit patterns on the host (a copy of the same bits)."""
    import numpy as np

    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def block_weights(C: int, seed: int, device="cpu"):
    """Random-init parameters of one attention block: LayerNorm scale/shift near (1, 0),
    projection matrices N(0, 1/C) as bf16 [C_out, C_in], small float32 biases."""
    s = 1.0 / (C ** 0.5)
    out = {
        "ln_gamma": 1.0 + 0.1 * normal_tensor((C,), seed, 20, device),
        "ln_beta": 0.1 * normal_tensor((C,), seed, 21, device),
        "ln_eps": 1e-6,
    }
    for i, name in enumerate(("q", "k", "v", "o")):
        out["w_" + name] = (s * normal_tensor((C, C), seed, 30 + i, device)).to(torch.bfloat16)
        out["b_" + name] = 0.02 * normal_tensor((C,), seed, 40 + i, device)
    return out


def block_input(B: int, NQ: int, C: int, seed: int, device="cpu"):
    """Block input activations ~ N(0,1), bf16 [B, NQ, C]."""
    return normal_tensor((B, NQ, C), seed, 50, device).to(torch.bfloat16)
