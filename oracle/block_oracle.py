"""CPU oracle for one global-attention block (TEST INFRASTRUCTURE ONLY).

    y = x + W_o Attn(Q, K, V) + b_o,     [Q|K|V] = W_{q,k,v} LayerNorm(x) + b_{q,k,v}

(AVGGT paper, Sec. 4.2: a global block is converted to frame attention, or subsampled as in
Sec. 4.3, with all its other components unchanged.)  Everything is float64 numpy, except that
the tensors the block DEFINES as bf16 -- the LayerNorm output, Q, K, V, the attention output
and y -- are rounded to bf16 (round to nearest even) where they are stored, exactly as the
library's interface states.  Attention itself is `sga_oracle`.  Weights are given as float64
arrays holding bf16-representable values; w_*: [C_out, C_in].

Pins (tests/test_oracle_pins.py::test_block_oracle_pieces_and_composition): the bf16 rounding
helper against torch's conversion incl. ties; LayerNorm and the linear map against
torch.nn.functional in float64; the block with identity projections against x + Attn(LN x);
the block with distinct random projections and biases against the formula written out with
torch float64 ops and torch's scaled_dot_product_attention.
"""
from __future__ import annotations

import numpy as np

from . import sga_oracle as orc

SGA, FRAME, DENSE = 0, 1, 2


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float64 -> bf16 bit patterns, round to nearest even (via float32)."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def layernorm(x: np.ndarray, gamma, beta, eps: float) -> np.ndarray:
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gamma + beta


def linear(x: np.ndarray, w: np.ndarray, b) -> np.ndarray:
    y = x @ w.T
    return y if b is None else y + b


def block(shape: orc.Shape, mode: int, x_bits: np.ndarray, wts: dict) -> np.ndarray:
    """x_bits: uint16 [B, NQ, C].  Returns y as float64 (already rounded to bf16 values)."""
    B, NQ, H, D = shape.B, shape.NQ, shape.H, shape.D
    C = H * D
    x = from_bf16_bits(x_bits).reshape(B, NQ, C)
    xn = from_bf16_bits(to_bf16_bits(layernorm(x, wts["ln_gamma"], wts["ln_beta"], wts["ln_eps"])))
    q = to_bf16_bits(linear(xn, wts["w_q"], wts.get("b_q"))).reshape(B, NQ, H, D)
    k = to_bf16_bits(linear(xn, wts["w_k"], wts.get("b_k"))).reshape(B, NQ, H, D)
    v = to_bf16_bits(linear(xn, wts["w_v"], wts.get("b_v"))).reshape(B, NQ, H, D)
    rows = np.arange(NQ, dtype=np.int64)
    if mode == SGA:
        o = orc.sga(shape, q, k, v, rows=rows)["O"]
    elif mode == FRAME:
        o, _ = orc.frame_rows(shape, q, k, v, rows)
    else:
        o, _ = orc.dense_rows(shape, q, k, v, rows)
    o = from_bf16_bits(to_bf16_bits(o)).reshape(B, NQ, C)
    y = x + linear(o, wts["w_o"], wts.get("b_o"))
    return from_bf16_bits(to_bf16_bits(y))
