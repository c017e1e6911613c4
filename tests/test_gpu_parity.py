"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Index lists and the compacted copies must be bit-exact;
outputs must agree within max-abs 2e-2 and mean-abs 2e-3 on unit-scale values
(bf16 operands, float32 accumulation, probabilities rounded to bf16 for the
second product); mean terms within 1e-6 + 1e-5*|mean|; log-sum-exp within 1e-2 plus
what ONE bf16 rounding of the scaled query (the kernel's MFMA operand is
q*scale*log2(e) in bf16) can move a logit, see lse_tolerance()."""
import math

import numpy as np
import pytest
import torch

from oracle import sga_oracle as orc
from paper_2512_02541_amd import binding as agg
from paper_2512_02541_amd import harness, inputs

pytestmark = pytest.mark.gpu

MAX_ABS = 2e-2
MEAN_ABS = 2e-3
LSE_ABS = 1e-2


def lse_tolerance(q, k, scale, rows):
    """Bound on |lse error| per (batch, head, row): 1e-2 for bf16 probabilities and float32
    sums, plus the input perturbation the kernel makes on purpose: its MFMA operand is
    q*scale*log2(e) rounded to bf16 (relative error <= 2^-9 per channel), which moves a logit
    by at most 2^-9 * scale * sum_d |q_d k_d| <= 2^-9 * scale * |q_i| * |k_j| (Cauchy-Schwarz),
    and lse moves by at most the largest logit error of its row.  Every key a row can see --
    kept, pooled (a mean of keys), its own, or the mean key -- has a norm of at most the
    largest key norm of its batch element and head."""
    r = torch.as_tensor(np.asarray(rows), device=q.device)
    qn = q[:, r].float().norm(dim=-1)                 # [B, R, H]
    kn = k.float().norm(dim=-1).amax(dim=1)           # [B, H]
    tol = LSE_ABS + 2.0 ** -9 * scale * qn * kn[:, None, :]
    return tol.permute(0, 2, 1).cpu().numpy().astype(np.float64)   # [B, H, R]


def oshape(s):
    return orc.Shape(s.B, s.N, s.n_h, s.n_w, s.n_special, s.H, s.D, s.s_h, s.s_w,
                     s.keep_first_frame, s.flags, s.scale, s.mean_logit_bias)


def say(msg):
    print(msg, flush=True)


def check_subsample(shape, buf, kb, vb):
    """idx / Kc / Vc bit-exact, means close; returns the oracle's pieces."""
    o = oshape(shape)
    idx = orc.kept_indices(o)
    M, nd = orc.counts(o)
    assert (buf.M, buf.n_dropped) == (M, nd)
    assert (buf.idx.cpu().numpy() == idx).all(), "kept index list differs"
    Kc, Vc = orc.gather(o, kb, vb, idx)
    got_k = harness.decode_compact(buf.Kc, shape.B, shape.H, M, buf.M_pad, "k")
    got_v = harness.decode_compact(buf.Vc, shape.B, shape.H, M, buf.M_pad, "v")
    assert (inputs.bf16_bits(got_k[:, :, :M]) == Kc).all(), "compacted K differs"
    assert (inputs.bf16_bits(got_v[:, :, :M]) == Vc).all(), "compacted V differs"
    if buf.M_pad > M:  # padding rows are zeros
        assert (inputs.bf16_bits(got_k[:, :, M:]) == 0).all()
        assert (inputs.bf16_bits(got_v[:, :, M:]) == 0).all()
    km, vm = orc.mean(o, kb, vb)
    gk = buf.kmean.cpu().numpy().astype(np.float64)
    gv = buf.vmean.cpu().numpy().astype(np.float64)
    assert (np.abs(gk - km) <= 1e-6 + 1e-5 * np.abs(km)).all(), np.abs(gk - km).max()
    assert (np.abs(gv - vm) <= 1e-6 + 1e-5 * np.abs(vm)).all(), np.abs(gv - vm).max()
    return idx, nd, Kc, Vc, km, vm


def check_output(got_o, got_lse, want_o, want_lse, rows, what, q=None, k=None, scale=0.125):
    g = got_o[:, rows].float().cpu().numpy().astype(np.float64)
    err = np.abs(g - want_o)
    assert np.isfinite(g).all(), what
    assert err.max() <= MAX_ABS, (what, err.max())
    assert err.mean() <= MEAN_ABS, (what, err.mean())
    if got_lse is not None:
        gl = got_lse[:, :, rows].cpu().numpy().astype(np.float64)
        lse_err = np.abs(gl - want_lse)
        tol = lse_tolerance(q, k, scale, rows)
        say("%s: lse max-abs error %.3e (largest share of its bound %.2f)" % (
            what, lse_err.max(), (lse_err / tol).max()))
        assert (lse_err <= tol).all(), (what, lse_err.max(), (lse_err / tol).max())
    return err.max(), err.mean()


def run_case(shape, q, k, v, rows=None, what=""):
    say("case %s: B=%d N=%d grid=%dx%d P=%d H=%d strides=(%d,%d) keep_first=%d flags=%d bias=%g" % (
        what, shape.B, shape.N, shape.n_h, shape.n_w, shape.n_special, shape.H, shape.s_h,
        shape.s_w, shape.keep_first_frame, shape.flags, shape.mean_logit_bias))
    buf = harness.sga_forward(shape, q, k, v, poison=True)
    torch.cuda.synchronize()
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    idx, nd, Kc, Vc, km, vm = check_subsample(shape, buf, kb, vb)
    if rows is None:
        rows = np.arange(shape.NQ, dtype=np.int64)
    want_o, want_lse, _ = orc.attn_rows(oshape(shape), qb, kb, vb, Kc, Vc, km, vm, nd, rows)
    return check_output(buf.O, buf.lse, want_o, want_lse, rows, what, q, k, shape.scale)


# ----------------------------------------------------------------------------
# Tiny configuration: every flag combination, both first-frame rules, every sigma
# ----------------------------------------------------------------------------
@pytest.fixture(scope="module")
def tiny_qkv():
    w = inputs.WORKLOADS["tiny"]
    return w, inputs.make_qkv(w, "cuda")


@pytest.mark.parametrize("sigma", [1, 2, 4, 6, 9])
@pytest.mark.parametrize("keep_first", [0, 1])
def test_tiny_all_flags(tiny_qkv, sigma, keep_first):
    w, (q, k, v) = tiny_qkv
    s_h, s_w = agg.agg_sigma_to_strides(sigma)
    for flags in (0, agg.AGG_DIAG, agg.AGG_MEAN, agg.AGG_DIAG | agg.AGG_MEAN):
        shape = harness.shape_of(w, flags=flags, s_h=s_h, s_w=s_w, keep_first_frame=keep_first)
        run_case(shape, q, k, v, what="tiny sigma=%d" % sigma)


def test_tiny_dense_baseline_and_stride_one_agree(tiny_qkv):
    w, (q, k, v) = tiny_qkv
    shape = harness.shape_of(w)
    O, lse = harness.dense_forward(shape, q, k, v)
    torch.cuda.synchronize()
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    rows = np.arange(shape.NQ, dtype=np.int64)
    want_o, want_lse = orc.dense_rows(oshape(shape), qb, kb, vb, rows)
    check_output(O, lse, want_o, want_lse, rows, "dense tiny", q, k, shape.scale)
    # strides (1,1) through the SGA entry point is the same computation, bit for bit
    s1 = harness.shape_of(w, s_h=1, s_w=1)
    buf = harness.sga_forward(s1, q, k, v)
    torch.cuda.synchronize()
    assert torch.equal(buf.O.view(torch.int16), O.view(torch.int16))
    assert torch.equal(buf.lse, lse)


def test_mean_logit_bias(tiny_qkv):
    w, (q, k, v) = tiny_qkv
    _, nd = agg.agg_kv_count(harness.shape_of(w))
    shape = harness.shape_of(w, flags=agg.AGG_MEAN, mean_logit_bias=math.log(nd))
    run_case(shape, q, k, v, what="tiny bias=ln|D|")


# ----------------------------------------------------------------------------
# Ragged shapes: head counts that do not fill a head group, batch > 1, grids
# that leave partial windows, compacted sets shorter than one tile, query
# counts that are not a multiple of the 256-row query tile.
# ----------------------------------------------------------------------------
RAGGED = [
    # B, N, n_h, n_w, P, H, s_h, s_w, keep_first
    (2, 3, 5, 7, 2, 3, 2, 3, 1),
    (1, 1, 4, 4, 1, 1, 3, 3, 0),     # M = 5 rows: far less than one tile
    (1, 2, 9, 11, 0, 5, 2, 2, 0),    # no special tokens
    (2, 5, 13, 17, 5, 2, 3, 3, 1),   # NQ = 1130 = 4*256 + 106
    (1, 4, 8, 8, 5, 16, 1, 2, 1),
    (1, 3, 6, 6, 5, 4, 7, 7, 0),     # strides larger than the grid: one patch per frame
    (1, 1, 6, 6, 5, 4, 2, 2, 1),     # single frame kept whole: nothing dropped
    (1, 2, 4, 5, 70, 2, 2, 2, 1),    # more special tokens than a 64-row tile
    (1, 2, 11, 4, 1, 2, 5, 1, 0),    # stride along the rows only
]


@pytest.mark.parametrize("case", RAGGED)
def test_ragged_shapes(case):
    B, N, n_h, n_w, P, H, s_h, s_w, kf = case
    shape = agg.make_shape(B, N, n_h, n_w, P, H, 64, s_h, s_w, kf)
    q, k, v = inputs.iid_qkv(B, shape.NQ, H, 64, seed=500 + N * 7 + H, device="cuda")
    run_case(shape, q, k, v, what="ragged")
    O, lse = harness.dense_forward(shape, q, k, v)
    torch.cuda.synchronize()
    rows = np.arange(shape.NQ, dtype=np.int64)
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    want_o, want_lse = orc.dense_rows(oshape(shape), qb, kb, vb, rows)
    check_output(O, lse, want_o, want_lse, rows, "ragged dense", q, k, shape.scale)


def test_large_logits_stay_finite():
    """Peaked rows: queries aligned with their own key at 6x scale (logits near 50); the
    sums have to grow a long way between tiles without overflow."""
    w = inputs.WORKLOADS["tiny"]
    q, k, v = inputs.make_qkv(w, "cuda")
    q = (6.0 * k.float()).to(torch.bfloat16)
    shape = harness.shape_of(w)
    run_case(shape, q, k, v, what="peaked")


@pytest.mark.parametrize("kind", ["huge_positive", "all_negative", "mixed_rows"])
def test_extreme_logits_take_the_general_path(kind):
    """Logits of several hundred nats: exp2 of the raw scores overflows (or every
    probability of a row underflows), so the kernel's unreferenced fast path must hand
    the workgroup to its running-maximum path.  Ragged sizes on purpose."""
    shape = agg.make_shape(1, 3, 9, 7, 5, 3, 64, 2, 2, 1)
    q, k, v = inputs.iid_qkv(1, shape.NQ, 3, 64, seed=4242, device="cuda")
    if kind == "huge_positive":      # own key at ~320 nats, everything else far below
        q = (40.0 * k.float()).to(torch.bfloat16)
    elif kind == "all_negative":     # every logit near -240 nats
        u = torch.ones(64, device="cuda")
        k = (u + 0.05 * k.float()).to(torch.bfloat16)
        q = (-30.0 * u).expand_as(q).to(torch.bfloat16).contiguous()
    else:                            # only some rows are extreme
        qf = q.float()
        qf[:, ::7] = 40.0 * k.float()[:, ::7]
        q = qf.to(torch.bfloat16)
    run_case(shape, q, k, v, what="extreme " + kind)
    O, lse = harness.dense_forward(shape, q, k, v)
    torch.cuda.synchronize()
    rows = np.arange(shape.NQ, dtype=np.int64)
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    want_o, want_lse = orc.dense_rows(oshape(shape), qb, kb, vb, rows)
    check_output(O, lse, want_o, want_lse, rows, "extreme dense " + kind, q, k, shape.scale)


def test_small_row_sums_with_padding():
    """Rows whose softmax denominator is far below the number of zero-padded keys of the
    last tile (every logit around -14 nats): the padded keys' unit contributions must
    not swamp the sum."""
    shape = agg.make_shape(1, 2, 6, 6, 5, 2, 64, 2, 2, 1)  # M = 55: 9 padded rows
    q, k, v = inputs.iid_qkv(1, shape.NQ, 2, 64, seed=77, device="cuda")
    u = torch.ones(64, device="cuda")
    k = (u + 0.05 * k.float()).to(torch.bfloat16)
    q = (-1.75 * u).expand_as(q).to(torch.bfloat16).contiguous()
    # all logits sit near -14 nats while lse is near -10: scale the bound by the logits
    run_case(shape, q, k, v, what="small sums")


def test_bitwise_reproducible(tiny_qkv):
    w, (q, k, v) = tiny_qkv
    shape = harness.shape_of(w)
    a = harness.sga_forward(shape, q, k, v, poison=True)
    b = harness.sga_forward(shape, q, k, v, poison=True)
    torch.cuda.synchronize()
    for x, y in ((a.O, b.O), (a.Kc, b.Kc), (a.Vc, b.Vc)):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))
    for x, y in ((a.lse, b.lse), (a.kmean, b.kmean), (a.vmean, b.vmean), (a.idx, b.idx)):
        assert torch.equal(x, y)


# ----------------------------------------------------------------------------
# Full-size workloads, in the launch configuration the benchmark times: index
# list, compacted copies and means in full; attention on a stratified row sample
# (every query row is independent) against the full compacted set.
# ----------------------------------------------------------------------------
def sample_rows(w, tile=256, extra=12, seed=0):
    L, NQ = w.L, w.NQ
    rows = set()
    frames = sorted({0, 1, w.N // 2, w.N - 1})
    cells = [(0, 0), (0, 1), (1, 0), (1, 1), (2, 2), (2, 3), (w.n_h - 1, w.n_w - 1),
             (w.n_h - 1, 0), (0, w.n_w - 1), (w.n_h // 2, w.n_w // 2 + 1)]
    for f in frames:
        for t in range(w.n_special):
            rows.add(f * L + t)
        for r, c in cells:
            rows.add(f * L + w.n_special + r * w.n_w + c)
    last_tile = (NQ // tile) * tile
    for r in (tile - 1, tile, last_tile - 1, last_tile, NQ - 1, NQ - 2):
        if 0 <= r < NQ:
            rows.add(r)
    rng = np.random.default_rng(seed)
    rows.update(int(x) for x in rng.integers(0, NQ, size=extra))
    return np.array(sorted(rows), dtype=np.int64)


@pytest.mark.parametrize("name,part,parts", [("f100", 0, 1), ("f300", 0, 2), ("f300", 1, 2),
                                             ("f800", 0, 2), ("f800", 1, 2)])
def test_full_size_workloads(name, part, parts):
    """The launch configuration bench.py times.  Sampled query rows (special tokens, kept and
    dropped patches, grid corners and edges, first / middle / last frame, both sides of a query
    tile boundary, the tail tile, plus 2000 random rows: more than 2048 per workload, split over
    two test cases at the larger sizes to keep each case's oracle time near a minute) against the
    oracle over the FULL compacted set; the index list and both compacted tensors bit-exact over
    all rows; and two properties of every output row."""
    w = inputs.WORKLOADS[name]
    say("generating %s" % name)
    q, k, v = inputs.make_qkv(w, "cuda")
    shape = harness.shape_of(w)
    rows = sample_rows(w, extra=2000)
    assert len(rows) >= 2048
    rows = rows[part::parts]
    mx, mn = run_case(shape, q, k, v, rows=rows, what=name)
    say("%s part %d/%d: %d sampled rows, max-abs %.3e mean-abs %.3e" % (
        name, part + 1, parts, len(rows), mx, mn))
    # properties that hold at any size, checked on all NQ rows: an output row is a convex
    # combination of value rows (kept rows, the query's own row, the mean of rows), so it stays
    # inside the per-channel range of V up to bf16 rounding; and nothing is NaN or infinite
    buf = harness.sga_forward(shape, q, k, v)
    torch.cuda.synchronize()
    vmax = v.float().amax(dim=1, keepdim=True)
    vmin = v.float().amin(dim=1, keepdim=True)
    o = buf.O.float()
    slack = 2.0 ** -7 * torch.maximum(vmax.abs(), vmin.abs()) + 1e-6
    assert bool(torch.isfinite(o).all()) and bool(torch.isfinite(buf.lse).all())
    assert bool((o <= vmax + slack).all()) and bool((o >= vmin - slack).all())


def test_mid_size_batch_of_three():
    """Three scenes in one call (B = 3, 12 frames of the benchmark's 37 x 37 + 5 tokens, 16 heads,
    pi^3 rule): every (batch, head) pair is its own key stream, numbered over the XCD slots;
    distinct data per scene, 300 sampled rows against the oracle, then the index-driven path."""
    shape = agg.make_shape(3, 12, 37, 37, 5, 16, 64, 2, 2, 0)
    q, k, v = inputs.iid_qkv(3, shape.NQ, 16, 64, seed=31337, device="cuda")
    rng = np.random.default_rng(12)
    rows = np.unique(np.concatenate([rng.integers(0, shape.NQ, 290), [0, 255, 256, shape.NQ - 1]]))
    mx, mn = run_case(shape, q, k, v, rows=rows.astype(np.int64), what="B=3")
    say("B=3: %d rows, max-abs %.3e mean-abs %.3e" % (len(rows), mx, mn))
    _idx_case(shape, q, k, v, "B=3")


def test_full_size_dense_baseline():
    w = inputs.WORKLOADS["f100"]
    q, k, v = inputs.make_qkv(w, "cuda")
    shape = harness.shape_of(w)
    O, lse = harness.dense_forward(shape, q, k, v)
    torch.cuda.synchronize()
    rows = sample_rows(w)[:: 4]
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    want_o, want_lse = orc.dense_rows(oshape(shape), qb, kb, vb, rows)
    check_output(O, lse, want_o, want_lse, rows, "dense f100", q, k, shape.scale)


# ----------------------------------------------------------------------------
# The same attention with the kernel fetching the kept rows of K/V in place through the index
# list (no compacted copy): identical arithmetic on identical operands, so bit-identical results.
# ----------------------------------------------------------------------------
def _idx_case(shape, q, k, v, what):
    say("idx case %s: N=%d grid=%dx%d H=%d strides=(%d,%d) keep_first=%d flags=%d" % (
        what, shape.N, shape.n_h, shape.n_w, shape.H, shape.s_h, shape.s_w, shape.keep_first_frame,
        shape.flags))
    ref = harness.sga_forward(shape, q, k, v, poison=True)
    got = harness.alloc(shape, "cuda", poison=True)
    # index list and mean terms only: no compacted tensors are written or read
    agg.agg_kv_subsample(shape, k, v, None, None, got.idx, got.kmean, got.vmean, got.workspace,
                         got.workspace.numel())
    harness.attend_idx(got, q, k, v)
    torch.cuda.synchronize()
    assert torch.equal(ref.idx, got.idx)
    assert torch.equal(ref.kmean, got.kmean) and torch.equal(ref.vmean, got.vmean)
    assert torch.isnan(got.Kc.float()).all() and torch.isnan(got.Vc.float()).all()  # untouched
    assert torch.equal(ref.O.view(torch.int16), got.O.view(torch.int16)), what
    assert torch.equal(ref.lse, got.lse), what


@pytest.mark.parametrize("sigma,keep_first,flags", [(2, 1, 3), (4, 0, 3), (9, 1, 1), (6, 0, 2),
                                                    (4, 1, 0), (1, 1, 3)])
def test_idx_path_matches_compacted_path_tiny(tiny_qkv, sigma, keep_first, flags):
    w, (q, k, v) = tiny_qkv
    s_h, s_w = agg.agg_sigma_to_strides(sigma)
    _idx_case(harness.shape_of(w, flags=flags, s_h=s_h, s_w=s_w, keep_first_frame=keep_first),
              q, k, v, "tiny")


@pytest.mark.parametrize("case", RAGGED)
def test_idx_path_matches_compacted_path_ragged(case):
    B, N, n_h, n_w, P, H, s_h, s_w, kf = case
    shape = agg.make_shape(B, N, n_h, n_w, P, H, 64, s_h, s_w, kf)
    q, k, v = inputs.iid_qkv(B, shape.NQ, H, 64, seed=500 + N * 7 + H, device="cuda")
    _idx_case(shape, q, k, v, "ragged")


def test_idx_path_extreme_logits():
    """The general path of the index-driven kernel (own key at several hundred nats)."""
    shape = agg.make_shape(1, 3, 9, 7, 5, 3, 64, 2, 2, 1)
    q, k, v = inputs.iid_qkv(1, shape.NQ, 3, 64, seed=4242, device="cuda")
    qf = q.float()
    qf[:, ::5] = 40.0 * k.float()[:, ::5]
    _idx_case(shape, qf.to(torch.bfloat16), k, v, "extreme")


def test_idx_path_full_size():
    """100 frames, every output row: bit-identical to the compacted path."""
    w = inputs.WORKLOADS["f100"]
    q, k, v = inputs.make_qkv(w, "cuda")
    _idx_case(harness.shape_of(w), q, k, v, "f100")


# ----------------------------------------------------------------------------
# Key counts around the tile edges: the key loop walks 64-key tiles through three LDS buffers
# (unrolled by three), masks the tail of the last tile only, and checks its row sums every 24
# tiles.  One frame with strides (1,1) makes every token a key, so M = NQ can be set at will:
# 1..8 tiles and two counts beyond the first sum check, each with a full, a one-key and a
# 63-key last tile, through all three ways the kernel fetches its tiles.
# ----------------------------------------------------------------------------
TILE_EDGE_COUNTS = [64 * t + r for t in (0, 1, 2, 3, 4, 5, 6, 7, 24, 25) for r in (0, 1, 63)
                    if 64 * t + r > 0]


@pytest.mark.parametrize("nkeys", TILE_EDGE_COUNTS)
def test_key_counts_around_tile_edges(nkeys):
    H = 2
    shape = agg.make_shape(1, 1, 1, nkeys, 0, H, 64, 1, 1, 1, flags=0)
    assert shape.NQ == nkeys and agg.agg_kv_count(shape) == (nkeys, 0)
    q, k, v = inputs.iid_qkv(1, nkeys, H, 64, seed=9000 + nkeys, device="cuda")
    say("tile-edge case: %d keys = %d tiles, %d in the last" % (nkeys, (nkeys + 63) // 64,
                                                               (nkeys - 1) % 64 + 1))
    O, lse = harness.dense_forward(shape, q, k, v)          # rows of K/V in place
    torch.cuda.synchronize()
    rows = np.arange(nkeys, dtype=np.int64)
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    want_o, want_lse = orc.dense_rows(oshape(shape), qb, kb, vb, rows)
    check_output(O, lse, want_o, want_lse, rows, "tile edge %d" % nkeys, q, k, shape.scale)
    ref = harness.sga_forward(shape, q, k, v, poison=True)  # compacted copy
    got = harness.alloc(shape, "cuda", poison=True)         # through the index list
    agg.agg_kv_subsample(shape, k, v, None, None, got.idx, got.kmean, got.vmean, got.workspace,
                         got.workspace.numel())
    harness.attend_idx(got, q, k, v)
    torch.cuda.synchronize()
    for name, other in (("compacted", ref), ("index-driven", got)):
        assert torch.equal(other.O.view(torch.int16), O.view(torch.int16)), (name, nkeys)
        assert torch.equal(other.lse, lse), (name, nkeys)


@pytest.mark.parametrize("nq", [1, 2, 31, 32, 33, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1025])
def test_query_counts_around_tile_edges(nq):
    """Query counts around the 32-query block, the 64-query wavefront and the 256-query
    workgroup tile, with a subsampled key set (one frame, pi^3 rule, strides (1,3)) and both
    extras: whole path against the oracle, then the index-driven path against the first."""
    shape = agg.make_shape(1, 1, 1, nq, 0, 3, 64, 1, 3, 0)
    q, k, v = inputs.iid_qkv(1, nq, 3, 64, seed=7000 + nq, device="cuda")
    run_case(shape, q, k, v, what="query edge %d" % nq)
    _idx_case(shape, q, k, v, "query edge %d" % nq)


@pytest.mark.parametrize("H", [33, 40])
def test_more_than_32_heads(H):
    """Rows wider than 256 sixteen-byte chunks: the mean pass covers a row with two workgroups
    side by side, the gather has a ragged last head group (33), and heads no longer divide
    evenly over the XCD slots.  Whole path, index-driven path, dense baseline, frame attention."""
    shape = agg.make_shape(1, 2, 6, 5, 1, H, 64, 2, 2, 1)
    q, k, v = inputs.iid_qkv(1, shape.NQ, H, 64, seed=3300 + H, device="cuda")
    run_case(shape, q, k, v, what="H=%d" % H)
    _idx_case(shape, q, k, v, "H=%d" % H)
    rows = np.arange(shape.NQ, dtype=np.int64)
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    O, lse = harness.dense_forward(shape, q, k, v)
    torch.cuda.synchronize()
    want_o, want_lse = orc.dense_rows(oshape(shape), qb, kb, vb, rows)
    check_output(O, lse, want_o, want_lse, rows, "dense H=%d" % H, q, k, shape.scale)
    O, lse = harness.frame_forward(shape, q, k, v)
    torch.cuda.synchronize()
    want_o, want_lse = orc.frame_rows(oshape(shape), qb, kb, vb, rows)
    err = np.abs(O.float().cpu().numpy().astype(np.float64) - want_o)
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (H, err.max(), err.mean())


# ----------------------------------------------------------------------------
# Frame attention (Global-to-Frame conversion of early global blocks)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("case", [(2, 3, 5, 7, 2, 3), (1, 4, 16, 16, 5, 16), (1, 2, 37, 37, 5, 2)])
def test_frame_attention(case):
    B, N, n_h, n_w, P, H = case
    shape = agg.make_shape(B, N, n_h, n_w, P, H, 64, 2, 2, 1)
    q, k, v = inputs.iid_qkv(B, shape.NQ, H, 64, seed=900 + N + H, device="cuda")
    O, lse = harness.frame_forward(shape, q, k, v)
    torch.cuda.synchronize()
    rows = np.arange(shape.NQ, dtype=np.int64)
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    want_o, want_lse = orc.frame_rows(oshape(shape), qb, kb, vb, rows)
    # library lse is [B*N, H, L]; the oracle's is [B, H, N*L]
    L = shape.L
    got_lse = lse.view(B, N, H, L).permute(0, 2, 1, 3).reshape(B, H, N * L)
    check_output(O, got_lse, want_o, want_lse, rows, "frame attention", q, k, shape.scale)


def test_full_size_frame_attention():
    w = inputs.WORKLOADS["f100"]
    q, k, v = inputs.make_qkv(w, "cuda")
    shape = harness.shape_of(w)
    O, _ = harness.frame_forward(shape, q, k, v, with_lse=False)
    torch.cuda.synchronize()
    rows = sample_rows(w)[:: 3]
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    want_o, _ = orc.frame_rows(oshape(shape), qb, kb, vb, rows)
    check_output(O, None, want_o, None, rows, "frame f100")


# ----------------------------------------------------------------------------
# The calls only enqueue kernels (no allocation, no synchronisation, no memset), so a
# layer can be captured into a HIP graph; every replay must reproduce the eager result.
# ----------------------------------------------------------------------------
def test_hip_graph_replays_match_eager(tiny_qkv):
    w, (q, k, v) = tiny_qkv
    shape = harness.shape_of(w)
    eager = harness.sga_forward(shape, q, k, v)
    torch.cuda.synchronize()
    buf = harness.alloc(shape, "cuda", poison=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):   # warm-up on the capture stream
        harness.subsample(buf, k, v)
        harness.attend(buf, q, k, v)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        harness.subsample(buf, k, v)
        harness.attend(buf, q, k, v)
    for replay in range(3):
        for t in (buf.O, buf.Kc, buf.Vc, buf.kmean, buf.vmean):
            t.fill_(float("nan"))   # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(buf.O.view(torch.int16), eager.O.view(torch.int16)), replay
        assert torch.equal(buf.lse, eager.lse), replay
        assert torch.equal(buf.kmean, eager.kmean) and torch.equal(buf.idx, eager.idx)


# ----------------------------------------------------------------------------
# One whole global-attention block: LayerNorm, Q/K/V projections, attention (subsampled,
# per-frame or dense), output projection, residual -- against the block oracle.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("mode", [agg.AGG_BLOCK_SGA, agg.AGG_BLOCK_FRAME, agg.AGG_BLOCK_DENSE])
def test_global_block(mode):
    from oracle import block_oracle as blk

    shape = agg.make_shape(1, 3, 9, 7, 5, 16, 64, 2, 2, 1)   # NQ = 204: ragged everywhere
    C = shape.H * 64
    wts = inputs.block_weights(C, seed=321, device="cuda")
    x = inputs.block_input(1, shape.NQ, C, seed=321, device="cuda")
    y, _ = harness.block_forward(shape, mode, wts, x)
    torch.cuda.synchronize()
    host = {k: (v.double().cpu().numpy() if torch.is_tensor(v) else v) for k, v in wts.items()}
    want = blk.block(oshape(shape), mode, inputs.bf16_bits(x), host)
    got = y.double().cpu().numpy()
    err = np.abs(got - want)
    # y = x + projection: bf16 storage of values up to ~4 gives an ulp of 2^-6; the attention
    # tolerance (2e-2) passes through a projection with unit gain
    assert np.isfinite(got).all()
    assert err.max() <= 6e-2 and err.mean() <= 4e-3, (mode, err.max(), err.mean())


BLOCK_MAX, BLOCK_MEAN = 6e-2, 4e-3   # one block: see test_global_block


def test_global_block_with_33_heads():
    """A block whose width (2112) is not a multiple of the projection kernel's 256-column tile:
    the last column tile of every projection is partial, and so is the last head group."""
    from oracle import block_oracle as blk

    shape = agg.make_shape(1, 2, 7, 6, 3, 33, 64, 2, 2, 1)
    C = shape.H * 64
    wts = inputs.block_weights(C, seed=777, device="cuda")
    x = inputs.block_input(1, shape.NQ, C, seed=777, device="cuda")
    y, _ = harness.block_forward(shape, agg.AGG_BLOCK_SGA, wts, x)
    torch.cuda.synchronize()
    host = {k: (v.double().cpu().numpy() if torch.is_tensor(v) else v) for k, v in wts.items()}
    want = blk.block(oshape(shape), agg.AGG_BLOCK_SGA, inputs.bf16_bits(x), host)
    got = y.double().cpu().numpy()
    err = np.abs(got - want)
    say("block with 33 heads: max %.3e mean %.3e" % (err.max(), err.mean()))
    assert np.isfinite(got).all()
    assert err.max() <= BLOCK_MAX and err.mean() <= BLOCK_MEAN, (err.max(), err.mean())



def _host_weights(wts):
    return {k: (v.double().cpu().numpy() if torch.is_tensor(v) else v) for k, v in wts.items()}


def test_block_stack_chained():
    """Four blocks chained the way an aggregator pass chains them (Sec. 4.2: an early global block
    as frame attention, then subsampled blocks; a dense block last for the third mode), each with
    its own weights, on one workspace.  Every block is checked in its chained position against
    the block oracle fed with the library's previous output (one block's tolerance), and the
    end of the chain against the oracle chained on its own outputs (the blocks' tolerances
    add up along the residual stream)."""
    from oracle import block_oracle as blk

    shape = agg.make_shape(1, 3, 9, 7, 5, 16, 64, 2, 2, 1)   # NQ = 204
    C = shape.H * 64
    modes = [agg.AGG_BLOCK_FRAME, agg.AGG_BLOCK_SGA, agg.AGG_BLOCK_SGA, agg.AGG_BLOCK_DENSE]
    layers = [inputs.block_weights(C, seed=700 + i, device="cuda") for i in range(len(modes))]
    cws = [agg.make_block_weights(l["ln_gamma"], l["ln_beta"], l["ln_eps"], l["w_q"], l["w_k"],
                                  l["w_v"], l["w_o"], l["b_q"], l["b_k"], l["b_v"], l["b_o"])
           for l in layers]
    nws = max(agg.agg_block_workspace_bytes(shape, m) for m in set(modes))
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    x0 = inputs.block_input(1, shape.NQ, C, seed=700, device="cuda")
    outs, src = [], x0
    for i, m in enumerate(modes):
        ws.fill_(0xFF)   # nothing may survive in the workspace from the previous block
        dst = torch.full_like(x0, float("nan"))
        say("stack block %d mode %d" % (i, m))
        agg.agg_global_block_fwd(shape, m, cws[i], src, dst, ws, nws)
        outs.append(dst)
        src = dst
    torch.cuda.synchronize()
    chained = inputs.bf16_bits(x0)
    prev = x0
    for i, m in enumerate(modes):
        host = _host_weights(layers[i])
        got = outs[i].double().cpu().numpy()
        assert np.isfinite(got).all(), i
        want_here = blk.block(oshape(shape), m, inputs.bf16_bits(prev), host)
        err = np.abs(got - want_here)
        say("stack block %d in place: max %.3e mean %.3e" % (i, err.max(), err.mean()))
        assert err.max() <= BLOCK_MAX and err.mean() <= BLOCK_MEAN, (i, err.max(), err.mean())
        want_chain = blk.block(oshape(shape), m, chained, host)
        chained = blk.to_bf16_bits(want_chain)
        err = np.abs(got - want_chain)
        say("stack block %d chained: max %.3e mean %.3e" % (i, err.max(), err.mean()))
        assert err.max() <= (i + 1) * BLOCK_MAX and err.mean() <= (i + 1) * BLOCK_MEAN, (
            i, err.max(), err.mean())
        prev = outs[i]


@pytest.mark.parametrize("mode", [agg.AGG_BLOCK_SGA, agg.AGG_BLOCK_FRAME])
def test_block_full_width_many_row_tiles(mode):
    """A block at the full width (C = 1024: four column tiles per projection) with 2530 rows:
    ten 256-row tiles, so the projection kernel's tile numbering wraps around the eight XCD
    slots and has fully interior tiles as well as a ragged last one; every row compared."""
    from oracle import block_oracle as blk

    shape = agg.make_shape(1, 2, 35, 36, 5, 16, 64, 2, 2, 1)   # NQ = 2 * 1265 = 2530
    C = shape.H * 64
    assert shape.NQ > 9 * 256
    wts = inputs.block_weights(C, seed=811, device="cuda")
    x = inputs.block_input(1, shape.NQ, C, seed=811, device="cuda")
    y, _ = harness.block_forward(shape, mode, wts, x)
    torch.cuda.synchronize()
    want = blk.block(oshape(shape), mode, inputs.bf16_bits(x), _host_weights(wts))
    got = y.double().cpu().numpy()
    err = np.abs(got - want)
    say("block C=1024 rows=%d mode %d: max %.3e mean %.3e" % (shape.NQ, mode, err.max(), err.mean()))
    assert np.isfinite(got).all()
    assert err.max() <= BLOCK_MAX and err.mean() <= BLOCK_MEAN, (mode, err.max(), err.mean())


def test_linear_and_layernorm_ragged_rows():
    """Row counts that are not a multiple of the 128-row GEMM tile or the 4-row LayerNorm
    group, exercised through the dense block on a 1-frame shape."""
    from oracle import block_oracle as blk

    shape = agg.make_shape(2, 1, 11, 13, 4, 2, 64, 1, 1, 1)  # B=2, NQ = 147, C = 128
    C = 128
    wts = inputs.block_weights(C, seed=99, device="cuda")
    x = inputs.block_input(2, shape.NQ, C, seed=99, device="cuda")
    y, _ = harness.block_forward(shape, agg.AGG_BLOCK_DENSE, wts, x)
    torch.cuda.synchronize()
    host = {k: (v.double().cpu().numpy() if torch.is_tensor(v) else v) for k, v in wts.items()}
    want = blk.block(oshape(shape), blk.DENSE, inputs.bf16_bits(x), host)
    err = np.abs(y.double().cpu().numpy() - want)
    assert err.max() <= 6e-2 and err.mean() <= 4e-3, (err.max(), err.mean())


# ----------------------------------------------------------------------------
# Caller-supplied kept lists and the selection rules of the token-selection ablation
# ----------------------------------------------------------------------------
def lshape(s):
    from oracle import list_oracle  # noqa: F401  (same field names as the C oracle's Shape)
    return oshape(s)


def check_list_case(shape, lst, q, k, v, rows=None, what=""):
    """Runs the list path and checks every product against the list oracle."""
    from oracle import list_oracle as lo

    say("list case %s: B=%d N=%d grid=%dx%d P=%d H=%d M_list=%d flags=%d" % (
        what, shape.B, shape.N, shape.n_h, shape.n_w, shape.n_special, shape.H, lst.shape[1],
        shape.flags))
    buf = harness.list_forward(shape, lst, q, k, v, poison=True)
    torch.cuda.synchronize()
    host_list = lst.cpu().numpy()
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    B, H, NQ, M = shape.B, shape.H, shape.NQ, lst.shape[1]
    # compacted copies: row m of batch b is token list[b, m], bit for bit; padding zero
    got_k = inputs.bf16_bits(harness.decode_compact(buf.Kc, B, H, M, buf.M_pad, "k"))
    got_v = inputs.bf16_bits(harness.decode_compact(buf.Vc, B, H, M, buf.M_pad, "v"))
    k4, v4 = kb.reshape(B, NQ, H, 64), vb.reshape(B, NQ, H, 64)
    for b in range(B):
        assert (got_k[b, :, :M] == k4[b, host_list[b]].transpose(1, 0, 2)).all(), "Kc differs"
        assert (got_v[b, :, :M] == v4[b, host_list[b]].transpose(1, 0, 2)).all(), "Vc differs"
    assert (got_k[:, :, M:] == 0).all() and (got_v[:, :, M:] == 0).all()
    # membership bitmap
    words = buf.kept_bits.cpu().numpy().view(np.uint32)
    for b in range(B):
        want = np.zeros(words.shape[1] * 32, dtype=bool)
        want[host_list[b]] = True
        got = ((words[b][:, None] >> np.arange(32, dtype=np.uint32)[None, :]) & 1).astype(bool).ravel()
        assert (got == want).all(), "kept_bits differ"
    if rows is None:
        rows = np.arange(NQ, dtype=np.int64)
    want_o, want_lse, km, vm, nd = lo.attn_rows(lshape(shape), host_list, qb, kb, vb, rows)
    assert (buf.n_dropped.cpu().numpy() == nd).all(), (buf.n_dropped.cpu().numpy(), nd)
    gk = buf.kmean.cpu().numpy().astype(np.float64)
    gv = buf.vmean.cpu().numpy().astype(np.float64)
    assert (np.abs(gk - km) <= 1e-6 + 1e-5 * np.abs(km)).all(), np.abs(gk - km).max()
    assert (np.abs(gv - vm) <= 1e-6 + 1e-5 * np.abs(vm)).all(), np.abs(gv - vm).max()
    check_output(buf.O, buf.lse, want_o, want_lse, rows, what, q, k, shape.scale)
    return buf


@pytest.mark.parametrize("keep_first", [0, 1])
def test_selection_rules_match_oracle(keep_first):
    from oracle import list_oracle as lo

    shape = agg.make_shape(2, 3, 7, 8, 5, 4, 64, 3, 3, keep_first)
    q, k, v = inputs.iid_qkv(2, shape.NQ, 4, 64, seed=700 + keep_first, device="cuda")
    kb = inputs.bf16_bits(k)
    first = harness.select(shape, agg.AGG_SELECT_FIRST, 0, k).cpu().numpy()
    assert (first == agg.agg_kv_indices_host(shape)[None, :]).all()
    for seed in (0, 77, (5 << 32) + 9):
        got = harness.select(shape, agg.AGG_SELECT_RANDOM, seed, k).cpu().numpy()
        want, _ = lo.select(lshape(shape), lo.RANDOM, seed, None)
        assert (got == want).all(), seed
    for rule, orule in ((agg.AGG_SELECT_HIGH, lo.HIGH), (agg.AGG_SELECT_LOW, lo.LOW)):
        got = harness.select(shape, rule, 0, k).cpu().numpy()
        want, cands = lo.select(lshape(shape), orule, 0, kb)
        # the kernel ranks float32 sums of squares: where it differs from the float64 choice the
        # two magnitudes must agree to float32 rounding of a 256-term sum
        for b, m in zip(*np.nonzero(got != want)):
            cells, mags = cands[b][m]
            assert got[b, m] in cells
            assert abs(mags[cells.index(got[b, m])] - mags[cells.index(want[b, m])]) <= \
                1e-5 * abs(mags[cells.index(want[b, m])])
        assert (got != want).mean() < 0.01


@pytest.mark.parametrize("rule", [0, 1, 2, 3])
@pytest.mark.parametrize("flags", [0, 3])
def test_list_path_on_selected_lists(rule, flags):
    shape = agg.make_shape(2, 3, 9, 7, 5, 3, 64, 2, 2, 1, flags=flags)
    q, k, v = inputs.iid_qkv(2, shape.NQ, 3, 64, seed=710 + rule, device="cuda")
    lst = harness.select(shape, rule, 31, k)
    check_list_case(shape, lst, q, k, v, what="rule %d" % rule)


def test_list_first_rule_agrees_with_grid_path(tiny_qkv):
    w, (q, k, v) = tiny_qkv
    shape = harness.shape_of(w)
    lst = harness.select(shape, agg.AGG_SELECT_FIRST, 0, k)
    a = harness.list_forward(shape, lst, q, k, v)
    b = harness.sga_forward(shape, q, k, v)
    torch.cuda.synchronize()
    assert torch.equal(a.Kc.view(torch.int16), b.Kc.view(torch.int16))
    assert torch.equal(a.Vc.view(torch.int16), b.Vc.view(torch.int16))
    assert int(a.n_dropped[0]) == b.n_dropped
    # the two mean reductions group their float32 partial sums differently
    assert (a.kmean - b.kmean).abs().max() < 1e-6
    assert (a.O.float() - b.O.float()).abs().max() <= 2.0 ** -7
    assert (a.lse - b.lse).abs().max() < 1e-5


def test_list_arbitrary_entries():
    """Different lists per batch element, in random order, one leaving out special tokens,
    one shorter than a tile of 64, and a list with a repeated token."""
    from oracle import list_oracle as lo  # noqa: F401

    shape = agg.make_shape(2, 2, 6, 5, 3, 2, 64, 2, 2, 0)
    NQ = shape.NQ
    q, k, v = inputs.iid_qkv(2, NQ, 2, 64, seed=720, device="cuda")
    rng = np.random.default_rng(3)
    for M in (40, 64, 65):
        lists = np.stack([rng.choice(NQ, M, replace=False) for _ in range(2)]).astype(np.int32)
        check_list_case(shape, torch.from_numpy(lists).cuda(), q, k, v, what="random M=%d" % M)
    repeated = np.stack([rng.choice(NQ, 50, replace=True) for _ in range(2)]).astype(np.int32)
    assert len(set(repeated[0].tolist())) < 50
    check_list_case(shape, torch.from_numpy(repeated).cuda(), q, k, v, what="repeated ids")
    everything = np.stack([rng.permutation(NQ), rng.permutation(NQ)]).astype(np.int32)
    buf = check_list_case(shape, torch.from_numpy(everything).cuda(), q, k, v, what="all tokens")
    assert (buf.n_dropped == 0).all()


def test_list_path_with_33_heads():
    """The list-driven pass where a row is wider than one workgroup's 256 chunks (the mean role
    runs two workgroups side by side and only the first writes the run's count)."""
    shape = agg.make_shape(2, 2, 6, 5, 3, 33, 64, 2, 2, 0)
    q, k, v = inputs.iid_qkv(2, shape.NQ, 33, 64, seed=733, device="cuda")
    rng = np.random.default_rng(33)
    lists = np.stack([rng.choice(shape.NQ, 21, replace=False) for _ in range(2)]).astype(np.int32)
    check_list_case(shape, torch.from_numpy(lists).cuda(), q, k, v, what="33 heads")


def test_list_full_size_random_rule():
    """100 frames: one random token per window, sampled query rows against the oracle."""
    w = inputs.WORKLOADS["f100"]
    shape = harness.shape_of(w)
    q, k, v = inputs.make_qkv(w, "cuda")
    lst = harness.select(shape, agg.AGG_SELECT_RANDOM, 2024, k)
    rows = np.array([0, 1373, 1374, 1379, 1380, 70000, 137399, 98765], dtype=np.int64)
    check_list_case(shape, lst, q, k, v, rows=rows, what="f100 random")


def _capture(fn):
    """Warm up fn on a side stream, capture it into a graph on that stream, return the graph."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fn()
    return graph


def test_hip_graph_of_static_subsample_and_index_driven_attention():
    """The pair of calls a caller under graph capture would use: the subsample call whose scratch
    lives inside the library (index list and mean terms only) and the attention that reads the
    kept rows in place.  Each replay reproduces the eager result of the ordinary path."""
    w = inputs.WORKLOADS["tiny"]
    shape = harness.shape_of(w)
    q, k, v = inputs.make_qkv(w, "cuda")
    eager = harness.sga_forward(shape, q, k, v)
    torch.cuda.synchronize()
    buf = harness.alloc(shape, "cuda", poison=True)

    def run():
        agg.agg_kv_subsample_static(shape, k, v, None, None, buf.idx, buf.kmean, buf.vmean)
        harness.attend_idx(buf, q, k, v)

    graph = _capture(run)
    for replay in range(3):
        for t in (buf.O, buf.lse, buf.kmean, buf.vmean):
            t.fill_(float("nan"))
        buf.idx.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(buf.idx, eager.idx), replay
        assert torch.equal(buf.kmean, eager.kmean) and torch.equal(buf.vmean, eager.vmean), replay
        assert torch.equal(buf.O.view(torch.int16), eager.O.view(torch.int16)), replay
        assert torch.equal(buf.lse, eager.lse), replay


def test_hip_graph_replays_of_block_and_list_paths():
    """Every launch of the multi-kernel entry points is capturable (they clear with kernels,
    not memsets) and each replay reproduces the eager result bit for bit."""
    shape = agg.make_shape(1, 3, 9, 7, 5, 4, 64, 2, 2, 1)
    C = shape.H * 64
    wts = inputs.block_weights(C, seed=11, device="cuda")
    x = inputs.block_input(1, shape.NQ, C, seed=11, device="cuda")
    for mode in (agg.AGG_BLOCK_SGA, agg.AGG_BLOCK_FRAME):
        eager, _ = harness.block_forward(shape, mode, wts, x)
        torch.cuda.synchronize()
        cw = agg.make_block_weights(wts["ln_gamma"], wts["ln_beta"], wts["ln_eps"], wts["w_q"],
                                    wts["w_k"], wts["w_v"], wts["w_o"], wts["b_q"], wts["b_k"],
                                    wts["b_v"], wts["b_o"])
        nws = agg.agg_block_workspace_bytes(shape, mode)
        ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(x)
        graph = _capture(lambda: agg.agg_global_block_fwd(shape, mode, cw, x, y, ws, nws))
        for replay in range(3):
            y.fill_(float("nan"))
            ws.fill_(0xFF)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y.view(torch.int16), eager.view(torch.int16)), (mode, replay)

    q, k, v = inputs.iid_qkv(1, shape.NQ, shape.H, 64, seed=12, device="cuda")
    lst = harness.select(shape, agg.AGG_SELECT_HIGH, 0, k)
    eager = harness.list_forward(shape, lst, q, k, v)
    torch.cuda.synchronize()
    buf = harness.list_forward(shape, lst, q, k, v, poison=True)
    torch.cuda.synchronize()
    M = lst.shape[1]

    def run():
        agg.agg_select_kv_indices(shape, agg.AGG_SELECT_HIGH, 0, k, lst)
        agg.agg_kv_subsample_list(shape, lst, M, k, v, buf.Kc, buf.Vc, buf.kmean, buf.vmean,
                                  buf.kept_bits, buf.n_dropped, buf.workspace, buf.workspace.numel())
        agg.agg_global_attn_fwd_list(shape, M, q, k, v, buf.Kc, buf.Vc, buf.kmean, buf.vmean,
                                     buf.kept_bits, buf.n_dropped, buf.O, buf.lse)

    graph = _capture(run)
    for replay in range(3):
        buf.O.fill_(float("nan"))
        buf.kept_bits.fill_(-1)
        buf.n_dropped.fill_(-7)
        buf.workspace.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(buf.O.view(torch.int16), eager.O.view(torch.int16)), replay
        assert torch.equal(buf.lse, eager.lse) and torch.equal(buf.n_dropped, eager.n_dropped)
        assert torch.equal(buf.kept_bits, eager.kept_bits) and torch.equal(buf.kmean, eager.kmean)


@pytest.mark.parametrize("case", [(2, 3, 7, 8, 5, 4, 3, 3, 1), (1, 2, 16, 16, 5, 16, 2, 2, 0),
                                  (1, 3, 5, 7, 2, 3, 1, 2, 1), (1, 2, 6, 5, 1, 33, 2, 2, 1)])
def test_cell_mean_pooling(case):
    """agg_kv_pool: rows are window means (one bf16 rounding), and attention over them without
    extras matches plain attention over the oracle's pooled rows."""
    from oracle import list_oracle as lo

    B, N, n_h, n_w, P, H, s_h, s_w, kf = case
    shape = agg.make_shape(B, N, n_h, n_w, P, H, 64, s_h, s_w, kf)
    q, k, v = inputs.iid_qkv(B, shape.NQ, H, 64, seed=740 + n_h, device="cuda")
    buf = harness.pool_forward(shape, q, k, v)
    torch.cuda.synchronize()
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    kp, vp, groups = lo.pool(lshape(shape), kb, vb)
    M = len(groups)
    assert M == buf.M
    got_k = harness.decode_compact(buf.Kc, B, H, M, buf.M_pad, "k").double().cpu().numpy()
    got_v = harness.decode_compact(buf.Vc, B, H, M, buf.M_pad, "v").double().cpu().numpy()
    assert (got_k[:, :, M:] == 0).all() and (got_v[:, :, M:] == 0).all()
    # float32 mean rounded once against float64 mean rounded once: at most one bf16 step apart
    for got, want in ((got_k[:, :, :M], kp), (got_v[:, :, :M], vp)):
        assert (np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-30).all()
        exact = got == lo.round_to_bf16(want)
        assert exact.mean() > 0.999
    single = np.array([len(g) == 1 for g in groups])
    assert np.array_equal(got_k[:, :, :M][:, :, single], kp[:, :, single])   # copies are exact
    rows = np.arange(shape.NQ, dtype=np.int64)
    want_o, want_lse = lo.attn_over_rows(lshape(shape), qb, lo.round_to_bf16(kp),
                                         lo.round_to_bf16(vp), rows)
    check_output(buf.O, buf.lse, want_o, want_lse, rows, "cell mean", q, k, shape.scale)


def test_list_path_with_extreme_logits():
    """The general (running-maximum) path with membership taken from the bitmap: own key at
    several hundred nats for every query, list chosen by the lowest-magnitude rule."""
    shape = agg.make_shape(2, 3, 9, 7, 5, 3, 64, 2, 2, 1)
    q, k, v = inputs.iid_qkv(2, shape.NQ, 3, 64, seed=4343, device="cuda")
    q = (40.0 * k.float()).to(torch.bfloat16)
    lst = harness.select(shape, agg.AGG_SELECT_LOW, 0, k)
    from oracle import list_oracle as lo

    buf = harness.list_forward(shape, lst, q, k, v, poison=True)
    torch.cuda.synchronize()
    rows = np.arange(shape.NQ, dtype=np.int64)
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    want_o, want_lse, _, _, _ = lo.attn_rows(lshape(shape), lst.cpu().numpy(), qb, kb, vb, rows)
    check_output(buf.O, buf.lse, want_o, want_lse, rows, "list extreme", q, k, shape.scale)
