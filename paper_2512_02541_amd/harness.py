"""Buffer plumbing around the C ABI for tests, the smoke check and the benchmark.

Allocates the device buffers the library's calls need (PyTorch owns the memory),
and decodes the fragment-order compacted tensors for comparison.  No arithmetic
of the method happens here.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding as agg


# ---- guard regions ------------------------------------------------------------------------
# With guards switched on (the GPU tests do), every buffer that a library call writes is
# allocated with GUARD_BYTES of a fixed pattern behind it; check_all_guards() synchronises and
# asserts that every pattern is intact: a bounds check on the kernels that cannot fault.
GUARD_BYTES = 4096
GUARD_VALUE = 0xA5
guards_enabled = False
_guards = []   # (name, raw uint8 tensor, payload bytes)


def _buf(shape, dtype, device, name):
    """torch.empty(shape, dtype) -- with a guard region behind it when guards are on."""
    if not guards_enabled:
        return torch.empty(shape, dtype=dtype, device=device)
    shape = (shape,) if isinstance(shape, int) else tuple(shape)
    numel = 1
    for n in shape:
        numel *= int(n)
    nbytes = numel * torch.empty((), dtype=dtype).element_size()
    raw = torch.empty(nbytes + GUARD_BYTES, dtype=torch.uint8, device=device)
    raw[nbytes:].fill_(GUARD_VALUE)
    _guards.append((name, raw, nbytes))
    return raw[:nbytes].view(dtype).view(shape)


def check_all_guards():
    """Synchronises, asserts that no guard region was written, and forgets the buffers."""
    if _guards:
        torch.cuda.synchronize()
    bad = [name for name, raw, n in _guards if not bool((raw[n:] == GUARD_VALUE).all())]
    count = len(_guards)
    _guards.clear()
    assert not bad, "written past the end of: %s" % ", ".join(bad)
    return count


def shape_of(w, flags=agg.AGG_DIAG | agg.AGG_MEAN, s_h=None, s_w=None, keep_first_frame=None,
             mean_logit_bias=0.0, scale=None) -> agg.agg_shape:
    """agg_shape for a ``inputs.Workload`` (strides / first-frame rule overridable)."""
    return agg.make_shape(
        w.B, w.N, w.n_h, w.n_w, w.n_special, w.H, w.D,
        w.s_h if s_h is None else s_h, w.s_w if s_w is None else s_w,
        w.keep_first_frame if keep_first_frame is None else keep_first_frame,
        flags, scale, mean_logit_bias)


@dataclass
class SgaBuffers:
    shape: agg.agg_shape
    M: int
    M_pad: int
    n_dropped: int
    Kc: torch.Tensor
    Vc: torch.Tensor
    idx: torch.Tensor
    kmean: torch.Tensor
    vmean: torch.Tensor
    workspace: torch.Tensor
    O: torch.Tensor
    lse: torch.Tensor


def alloc(shape: agg.agg_shape, device="cuda", with_lse=True, poison=False) -> SgaBuffers:
    M, nd = agg.agg_kv_count(shape)
    nbytes, m_pad = agg.agg_kv_compact_bytes(shape)
    B, H, D, NQ = shape.B, shape.H, shape.D, shape.NQ
    Kc = _buf(nbytes // 2, torch.bfloat16, device, "Kc")
    Vc = _buf(nbytes // 2, torch.bfloat16, device, "Vc")
    idx = _buf(M, torch.int32, device, "idx")
    kmean = _buf((B, H, D), torch.float32, device, "kmean")
    vmean = _buf((B, H, D), torch.float32, device, "vmean")
    ws = _buf(agg.agg_workspace_bytes(shape), torch.uint8, device, "subsample workspace")
    O = _buf((B, NQ, H, D), torch.bfloat16, device, "O")
    lse = _buf((B, H, NQ), torch.float32, device, "lse") if with_lse else None
    if poison:  # make stale or unwritten memory visible to the comparison
        for t in (Kc, Vc, kmean, vmean, O):
            t.fill_(float("nan"))
        idx.fill_(-7)
        ws.fill_(0xFF)
        if lse is not None:
            lse.fill_(float("nan"))
    return SgaBuffers(shape, M, m_pad, nd, Kc, Vc, idx, kmean, vmean, ws, O, lse)


def subsample(buf: SgaBuffers, K, V, stream=None):
    agg.agg_kv_subsample(buf.shape, K, V, buf.Kc, buf.Vc, buf.idx, buf.kmean, buf.vmean,
                         buf.workspace, buf.workspace.numel(), stream)


def attend(buf: SgaBuffers, Q, K, V, stream=None):
    agg.agg_global_attn_fwd(buf.shape, Q, K, V, buf.Kc, buf.Vc, buf.kmean, buf.vmean, buf.O,
                            buf.lse, stream)


def attend_idx(buf: SgaBuffers, Q, K, V, stream=None):
    """The same attention reading the kept rows of K/V in place through buf.idx."""
    agg.agg_global_attn_fwd_idx(buf.shape, Q, K, V, buf.idx, buf.kmean, buf.vmean, buf.O, buf.lse,
                                stream)


def sga_forward(shape, Q, K, V, poison=False) -> SgaBuffers:
    """One pass of the whole path: gather + mean terms, then attention."""
    buf = alloc(shape, Q.device, poison=poison)
    subsample(buf, K, V)
    attend(buf, Q, K, V)
    return buf


def dense_forward(shape, Q, K, V, with_lse=True):
    B, H, D, NQ = shape.B, shape.H, shape.D, shape.NQ
    O = _buf((B, NQ, H, D), torch.bfloat16, Q.device, "dense O")
    lse = _buf((B, H, NQ), torch.float32, Q.device, "dense lse") if with_lse else None
    agg.agg_dense_global_attn_fwd(shape, Q, K, V, O, lse)
    return O, lse


def frame_forward(shape, Q, K, V, with_lse=True):
    """Per-frame attention (Global-to-Frame conversion); lse comes back as [B*N, H, L]."""
    B, N, H, D, NQ = shape.B, shape.N, shape.H, shape.D, shape.NQ
    O = _buf((B, NQ, H, D), torch.bfloat16, Q.device, "frame O")
    lse = _buf((B * N, H, shape.L), torch.float32, Q.device, "frame lse") if with_lse else None
    agg.agg_frame_attn_fwd(shape, Q, K, V, O, lse)
    return O, lse


def block_forward(shape, mode, wts, x):
    """One global-attention block (LayerNorm, projections, attention of `mode`, output
    projection, residual); wts is the dict of device tensors from inputs.block_weights."""
    cw = agg.make_block_weights(wts["ln_gamma"], wts["ln_beta"], wts["ln_eps"], wts["w_q"],
                                wts["w_k"], wts["w_v"], wts["w_o"], wts.get("b_q"), wts.get("b_k"),
                                wts.get("b_v"), wts.get("b_o"))
    nws = agg.agg_block_workspace_bytes(shape, mode)
    ws = _buf(nws, torch.uint8, x.device, "block workspace")
    y = _buf(tuple(x.shape), x.dtype, x.device, "block y")
    agg.agg_global_block_fwd(shape, mode, cw, x, y, ws, nws)
    return y, ws


def decode_compact(flat: torch.Tensor, B: int, H: int, M: int, M_pad: int, which: str) -> torch.Tensor:
    """Fragment-order Kc ('k') or Vc ('v') -> plain [B, H, M_pad, 64] (layout of agg.h)."""
    nt = M_pad // 64
    x = flat.view(B, H, nt, 4096)
    if which == "k":
        # [kb(2)][ks(4)][g(2)][key(32)][e(8)] ; row = kb*32+key ; channel = ks*16 + g*8 + e
        x = x.view(B, H, nt, 2, 4, 2, 32, 8).permute(0, 1, 2, 3, 6, 4, 5, 7)
        return x.reshape(B, H, M_pad, 64)
    # [t(4)][g(2)][d(64)][e_hi(2)][e_lo(4)] ; row = 16t + 8e_hi + 4g + e_lo
    x = x.view(B, H, nt, 4, 2, 64, 2, 4).permute(0, 1, 2, 3, 6, 4, 7, 5)
    return x.reshape(B, H, M_pad, 64)


@dataclass
class ListBuffers:
    shape: agg.agg_shape
    M: int
    M_pad: int
    Kc: torch.Tensor
    Vc: torch.Tensor
    kmean: torch.Tensor
    vmean: torch.Tensor
    kept_bits: torch.Tensor
    n_dropped: torch.Tensor
    workspace: torch.Tensor
    O: torch.Tensor
    lse: torch.Tensor


def list_forward(shape, kv_list, Q, K, V, poison=False) -> ListBuffers:
    """The path over a caller's kept list: kv_list is a device int32 [B, M_list] tensor."""
    B, H, D, NQ = shape.B, shape.H, shape.D, shape.NQ
    M = kv_list.shape[1]
    nbytes, m_pad = agg.agg_list_compact_bytes(shape, M)
    dev = Q.device
    Kc = _buf(nbytes // 2, torch.bfloat16, dev, "list Kc")
    Vc = _buf(nbytes // 2, torch.bfloat16, dev, "list Vc")
    kmean = _buf((B, H, D), torch.float32, dev, "list kmean")
    vmean = _buf((B, H, D), torch.float32, dev, "list vmean")
    bits = _buf((B, (NQ + 31) // 32), torch.int32, dev, "kept_bits")
    nd = _buf((B,), torch.int32, dev, "n_dropped")
    ws = _buf(agg.agg_list_workspace_bytes(shape), torch.uint8, dev, "list workspace")
    O = _buf((B, NQ, H, D), torch.bfloat16, dev, "list O")
    lse = _buf((B, H, NQ), torch.float32, dev, "list lse")
    if poison:
        for t in (Kc, Vc, kmean, vmean, O, lse):
            t.fill_(float("nan"))
        bits.fill_(-1)
        nd.fill_(-7)
        ws.fill_(0xFF)
    agg.agg_kv_subsample_list(shape, kv_list, M, K, V, Kc, Vc, kmean, vmean, bits, nd, ws, ws.numel())
    agg.agg_global_attn_fwd_list(shape, M, Q, K, V, Kc, Vc, kmean, vmean, bits, nd, O, lse)
    return ListBuffers(shape, M, m_pad, Kc, Vc, kmean, vmean, bits, nd, ws, O, lse)


def select(shape, rule, seed, K):
    """Device int32 [B, M] list chosen by `rule` (agg_select_kv_indices)."""
    M, _ = agg.agg_kv_count(shape)
    out = _buf((shape.B, M), torch.int32, K.device, "selected list")
    out.fill_(-1)
    agg.agg_select_kv_indices(shape, rule, seed, K, out)
    return out


def pool_forward(shape, Q, K, V):
    """Cell-mean variant: pooled compacted set, then attention without extras (flags 0)."""
    plain = agg.make_shape(shape.B, shape.N, shape.n_h, shape.n_w, shape.n_special, shape.H,
                           shape.D, shape.s_h, shape.s_w, shape.keep_first_frame, 0, shape.scale, 0.0)
    buf = alloc(plain, Q.device, poison=True)
    buf.kmean.zero_()
    buf.vmean.zero_()
    agg.agg_kv_pool(plain, K, V, buf.Kc, buf.Vc)
    attend(buf, Q, K, V)
    return buf
