"""Pins for the CPU oracle: everything here runs without a GPU and compares the
oracle with something other than itself -- values the paper prints, textbook
attention, masked dense attention written a second way, closed forms and
invariants (AVGGT paper, Sec. 4.1, 4.2, 4.3 and its FLOPs tables)."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import sga_oracle as orc
from paper_2512_02541_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def small_shape(**kw):
    base = dict(B=1, N=3, n_h=5, n_w=7, n_special=2, H=2, D=8, s_h=2, s_w=3,
                keep_first_frame=1, flags=orc.DIAG | orc.MEAN, scale=float(np.float32(1.0 / math.sqrt(8.0))),  # the ABI carries float32
                mean_logit_bias=0.0)
    base.update(kw)
    return orc.Shape(**base)


def draw(shape, seed=7):
    q, k, v = inputs.iid_qkv(shape.B, shape.NQ, shape.H, shape.D, seed)
    return q, k, v


def bits(t):
    return inputs.bf16_bits(t)


# ----------------------------------------------------------------------------
# A second, independent statement of the kept set: enumerate windows, mark the
# first token of each (Sec. 4.3: the first patch token of every s_h x s_w window is kept).
# ----------------------------------------------------------------------------
def kept_mask_by_windows(shape):
    L = shape.L
    mask = np.zeros(shape.NQ, dtype=bool)
    for f in range(shape.N):
        base = f * L
        mask[base:base + shape.n_special] = True
        if f == 0 and shape.keep_first_frame:
            mask[base:base + L] = True
            continue
        for top in range(0, shape.n_h, shape.s_h):
            for left in range(0, shape.n_w, shape.s_w):
                window = [(r, c) for r in range(top, min(top + shape.s_h, shape.n_h))
                          for c in range(left, min(left + shape.s_w, shape.n_w))]
                r, c = window[0]  # row-major first
                mask[base + shape.n_special + r * shape.n_w + c] = True
    return mask


def masked_dense_reference(shape, q, k, v, kept, with_self, with_mean, beta=0.0):
    """softmax over an explicit (NQ x (NQ+1)) masked logit matrix in float64; the
    last column is the mean pair.  Never builds a compacted copy."""
    qd, kd, vd = (t.to(torch.float64).numpy() for t in (q, k, v))
    B, NQ, H, D = qd.shape
    dropped = ~kept
    out = np.zeros((B, NQ, H, D))
    lse = np.zeros((B, H, NQ))
    probs = np.zeros((B, H, NQ, NQ + 1))
    for b in range(B):
        for h in range(H):
            kk = kd[b, :, h, :]
            vv = vd[b, :, h, :]
            if dropped.any():
                kbar = kk[dropped].mean(axis=0)
                vbar = vv[dropped].mean(axis=0)
            else:
                kbar = np.zeros(D)
                vbar = np.zeros(D)
            k_aug = np.concatenate([kk, kbar[None]], axis=0)
            v_aug = np.concatenate([vv, vbar[None]], axis=0)
            logits = shape.scale * qd[b, :, h, :] @ k_aug.T
            logits[:, NQ] += beta
            allow = np.zeros((NQ, NQ + 1), dtype=bool)
            allow[:, :NQ] = kept[None, :]
            if with_self:
                allow[np.arange(NQ), np.arange(NQ)] |= dropped
            if with_mean and dropped.any():
                allow[:, NQ] = True
            logits = np.where(allow, logits, -np.inf)
            mx = logits.max(axis=1, keepdims=True)
            e = np.exp(logits - mx)
            den = e.sum(axis=1, keepdims=True)
            p = e / den
            out[b, :, h, :] = p @ v_aug
            lse[b, h] = (mx + np.log(den))[:, 0]
            probs[b, h] = p
    return out, lse, probs


# ----------------------------------------------------------------------------
# sigma table and window rule, as printed
# ----------------------------------------------------------------------------
def test_sigma_table_matches_paper():
    rows = _read_table("sigma_table.txt")
    assert len(rows) == 4
    for sigma, sh, sw in rows:
        assert orc.sigma_to_strides(int(sigma)) == (int(sh), int(sw))
        assert int(sh) * int(sw) == int(sigma)
    with pytest.raises(ValueError):
        orc.sigma_to_strides(3)


@pytest.mark.parametrize("n_h,n_w,s_h,s_w", [(5, 7, 2, 3), (4, 4, 2, 2), (3, 5, 1, 2), (7, 7, 3, 3),
                                               (2, 3, 3, 3), (6, 1, 2, 2)])
@pytest.mark.parametrize("keep_first", [0, 1])
def test_kept_set_is_first_token_of_each_window(n_h, n_w, s_h, s_w, keep_first):
    shape = small_shape(n_h=n_h, n_w=n_w, s_h=s_h, s_w=s_w, keep_first_frame=keep_first)
    want = kept_mask_by_windows(shape)
    got = np.array([orc.is_kept(shape, t) for t in range(shape.NQ)])
    assert (got == want).all()
    idx = orc.kept_indices(shape)
    assert (idx == np.nonzero(want)[0]).all()
    assert (np.diff(idx) > 0).all()
    kept, dropped = orc.counts(shape)
    per_frame = math.ceil(n_h / s_h) * math.ceil(n_w / s_w)
    f0 = 1 if keep_first else 0
    assert kept == f0 * shape.L + (shape.N - f0) * (shape.n_special + per_frame)
    assert kept + dropped == shape.NQ
    # every window of a subsampled frame holds exactly one kept patch
    for f in range(f0, shape.N):
        for top in range(0, n_h, s_h):
            for left in range(0, n_w, s_w):
                cnt = sum(want[f * shape.L + shape.n_special + r * n_w + c]
                          for r in range(top, min(top + s_h, n_h))
                          for c in range(left, min(left + s_w, n_w)))
                assert cnt == 1


def test_kept_counts_reproduce_paper_flops_tables():
    """The FLOPs columns of the paper's 800- and 333-frame tables fix the count
    formula: ceil windows, first frame whole, special tokens kept."""
    table = {}
    for frames, sigma, flops in _read_table("flops_tables.txt"):
        table[(int(frames), int(sigma))] = float(flops)
    C = 1024
    for frames, sigmas in ((800, (2, 4, 6, 9)), (334, (2, 4))):
        base = orc.Shape(1, frames, 28, 37, 5, 16, 64, 1, 1, 1, 0, 0.125)
        NQ = base.NQ
        other_parts = table[(frames, 1)] - 24 * 2 * NQ * NQ * C / 1e15
        frame_layers = 9 * 2 * frames * base.L * base.L * C / 1e15
        for sigma in sigmas:
            sh, sw = orc.sigma_to_strides(sigma)
            shape = orc.Shape(1, frames, 28, 37, 5, 16, 64, sh, sw, 1, 0, 0.125)
            M, _ = orc.counts(shape)
            resid = table[(frames, sigma)] - 15 * 2 * NQ * M * C / 1e15
            assert abs(resid - other_parts - frame_layers) < 1.2e-3, (frames, sigma, resid)
            # the two nearest misreadings are rejected by the same numbers
            shape_all = orc.Shape(1, frames, 28, 37, 5, 16, 64, sh, sw, 0, 0, 0.125)
            M_all, _ = orc.counts(shape_all)
            resid_all = table[(frames, sigma)] - 15 * 2 * NQ * M_all * C / 1e15
            assert abs(resid_all - other_parts - frame_layers) > 2.5e-3
            M_floor = base.L + (frames - 1) * (5 + (28 // sh) * (37 // sw))
            if M_floor != M:
                resid_floor = table[(frames, sigma)] - 15 * 2 * NQ * M_floor * C / 1e15
                assert abs(resid_floor - other_parts - frame_layers) > 2e-2


def test_bench_geometry_counts():
    # sizes of the measured workloads: 37x37 grid, 5 special tokens, VGGT rule
    expect = {"tiny": (522, 330, 192), "f100": (137400, 71466, 65934),
              "f300": (412200, 110808, 301392), "f333": (457542, 122886, 334656),
              "f800": (1099200, 140400, 958800)}
    for name, (nq, m, nd) in expect.items():
        w = inputs.WORKLOADS[name]
        shape = orc.Shape(w.B, w.N, w.n_h, w.n_w, w.n_special, w.H, w.D, w.s_h, w.s_w,
                          w.keep_first_frame, 3, 0.125)
        assert shape.NQ == nq
        assert orc.counts(shape) == (m, nd)


# ----------------------------------------------------------------------------
# s = 1 and the dense routine against textbook attention
# ----------------------------------------------------------------------------
def textbook_attention_loops(q, k, v, scale):
    """Triple loop, float64, for tiny inputs only."""
    B, NQ, H, D = q.shape
    out = np.zeros((B, NQ, H, D))
    for b in range(B):
        for h in range(H):
            for i in range(NQ):
                logit = [scale * sum(q[b, i, h, d] * k[b, j, h, d] for d in range(D))
                         for j in range(NQ)]
                mx = max(logit)
                w = [math.exp(x - mx) for x in logit]
                den = sum(w)
                for d in range(D):
                    out[b, i, h, d] = sum(w[j] * v[b, j, h, d] for j in range(NQ)) / den
    return out


def test_dense_rows_equal_textbook_attention():
    shape = small_shape(N=2, n_h=3, n_w=3, s_h=1, s_w=1, flags=0)
    q, k, v = draw(shape, seed=3)
    rows = np.arange(shape.NQ)
    O, lse = orc.dense_rows(shape, bits(q), bits(k), bits(v), rows)
    want = textbook_attention_loops(*(t.to(torch.float64).numpy() for t in (q, k, v)), shape.scale)
    assert np.abs(O - want).max() < 1e-12
    # library cross-check: torch's scaled_dot_product_attention in float64
    qt, kt, vt = (t.to(torch.float64).permute(0, 2, 1, 3) for t in (q, k, v))
    sd = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, scale=shape.scale)
    assert np.abs(O - sd.permute(0, 2, 1, 3).numpy()).max() < 1e-12
    ref_lse = torch.logsumexp(shape.scale * qt @ kt.transpose(-1, -2), dim=-1).numpy()
    assert np.abs(lse - ref_lse).max() < 1e-12


@pytest.mark.parametrize("flags", [0, orc.DIAG, orc.MEAN, orc.DIAG | orc.MEAN])
def test_strides_one_reduce_to_dense(flags):
    shape = small_shape(s_h=1, s_w=1, flags=flags, B=2)
    q, k, v = draw(shape, seed=11)
    res = orc.sga(shape, bits(q), bits(k), bits(v))
    assert res["n_dropped"] == 0 and len(res["idx"]) == shape.NQ
    O, lse = orc.dense_rows(shape, bits(q), bits(k), bits(v), np.arange(shape.NQ))
    assert np.abs(res["O"] - O).max() < 1e-12
    assert np.abs(res["lse"] - lse).max() < 1e-12


def test_single_frame_with_reference_rule_is_dense():
    shape = small_shape(N=1, keep_first_frame=1)
    q, k, v = draw(shape, seed=12)
    res = orc.sga(shape, bits(q), bits(k), bits(v))
    O, _ = orc.dense_rows(shape, bits(q), bits(k), bits(v), np.arange(shape.NQ))
    assert res["n_dropped"] == 0
    assert np.abs(res["O"] - O).max() < 1e-12


# ----------------------------------------------------------------------------
# subset, self term, mean term against masked dense attention
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("flags", [0, orc.DIAG, orc.MEAN, orc.DIAG | orc.MEAN])
@pytest.mark.parametrize("keep_first", [0, 1])
@pytest.mark.parametrize("strides", [(1, 2), (2, 2), (2, 3), (3, 3)])
def test_sga_equals_masked_dense_attention(flags, keep_first, strides):
    shape = small_shape(s_h=strides[0], s_w=strides[1], keep_first_frame=keep_first, flags=flags,
                        B=2, mean_logit_bias=0.25 if flags & orc.MEAN else 0.0)
    q, k, v = draw(shape, seed=21 + flags)
    res = orc.sga(shape, bits(q), bits(k), bits(v), want_p=True)
    kept = kept_mask_by_windows(shape)
    want_o, want_lse, want_p = masked_dense_reference(
        shape, q, k, v, kept, bool(flags & orc.DIAG), bool(flags & orc.MEAN),
        beta=shape.mean_logit_bias)
    assert np.abs(res["O"] - want_o).max() < 1e-11
    assert np.abs(res["lse"] - want_lse).max() < 1e-11
    # probabilities, column by column: kept columns, then self, then mean
    P = res["P"]
    M = len(res["idx"])
    assert np.abs(P[..., :M] - want_p[..., res["idx"]]).max() < 1e-12
    NQ = shape.NQ
    diag = want_p[:, :, np.arange(NQ), np.arange(NQ)] * (~kept)[None, None, :]
    if not flags & orc.DIAG:
        diag = np.zeros_like(diag)
    assert np.abs(P[..., M] - diag).max() < 1e-12
    assert np.abs(P[..., M + 1] - want_p[..., NQ]).max() < 1e-12
    # shared normalisation: the concatenated list sums to one
    assert np.abs(P.sum(axis=-1) - 1.0).max() < 1e-12


def test_explicit_compacted_copy_and_mean():
    shape = small_shape(B=2)
    q, k, v = draw(shape, seed=31)
    kb, vb = bits(k), bits(v)
    idx = orc.kept_indices(shape)
    Kc, Vc = orc.gather(shape, kb, vb, idx)
    assert Kc.shape == (shape.B, shape.H, len(idx), shape.D)
    assert (Kc == kb[:, idx].transpose(0, 2, 1, 3)).all()
    assert (Vc == vb[:, idx].transpose(0, 2, 1, 3)).all()
    km, vm = orc.mean(shape, kb, vb)
    kept = kept_mask_by_windows(shape)
    want_k = k.to(torch.float64).numpy()[:, ~kept].mean(axis=1)
    want_v = v.to(torch.float64).numpy()[:, ~kept].mean(axis=1)
    assert np.abs(km - want_k).max() < 1e-13
    assert np.abs(vm - want_v).max() < 1e-13


def test_identical_dropped_tokens_closed_form():
    """If every dropped patch carries the same (k*, v*), the mean column with
    logit bias ln|D| carries exactly the dropped mass: SGA (mean on, self off)
    equals dense attention for every query."""
    shape = small_shape(flags=orc.MEAN, s_h=2, s_w=2, n_h=4, n_w=6)
    q, k, v = draw(shape, seed=41)
    kept = kept_mask_by_windows(shape)
    k = k.clone()
    v = v.clone()
    drop_ids = torch.from_numpy(np.nonzero(~kept)[0])
    k[:, drop_ids] = k[:, drop_ids[0]].clone().unsqueeze(1)
    v[:, drop_ids] = v[:, drop_ids[0]].clone().unsqueeze(1)
    n_dropped = int((~kept).sum())
    shape.mean_logit_bias = float(np.float32(math.log(n_dropped)))
    res = orc.sga(shape, bits(q), bits(k), bits(v))
    dense_o, dense_lse = orc.dense_rows(shape, bits(q), bits(k), bits(v), np.arange(shape.NQ))
    # bias is stored as float32, so agreement is to float32 rounding of ln|D|
    assert np.abs(res["O"] - dense_o).max() < 1e-6
    assert np.abs(res["lse"] - dense_lse).max() < 1e-6
    # with bias 0 it equals dense attention whose dropped set is one column
    shape.mean_logit_bias = 0.0
    res0 = orc.sga(shape, bits(q), bits(k), bits(v))
    first = np.nonzero(~kept)[0][0]
    collapsed = kept.copy()
    collapsed[first] = True
    ref, _, _ = masked_dense_reference(shape, q, k, v, collapsed, False, False)
    assert np.abs(res0["O"] - ref).max() < 1e-11


def test_self_term_dominates_when_query_is_aligned_with_own_key():
    shape = small_shape(flags=orc.DIAG, scale=1.0)
    q, k, v = draw(shape, seed=51)
    kept = kept_mask_by_windows(shape)
    # equal-norm keys and q_i = 200 k_i: <q_i, k_i> = 200 |k|^2 exceeds every other
    # logit 200 <k_i, k_j> by Cauchy-Schwarz, by tens of nats for distinct directions
    k = (3.0 * k.float() / k.float().norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    q = (200.0 * k.float()).to(torch.bfloat16)
    res = orc.sga(shape, bits(q), bits(k), bits(v))
    vd = v.to(torch.float64).numpy()
    dropped = np.nonzero(~kept)[0]
    assert len(dropped) > 0
    assert np.abs(res["O"][:, dropped] - vd[:, dropped]).max() < 1e-6
    # a kept query gets no second copy of itself: with the flag on or off it is unchanged
    shape_off = small_shape(flags=0, scale=1.0)
    res_off = orc.sga(shape_off, bits(q), bits(k), bits(v))
    kept_ids = np.nonzero(kept)[0]
    assert np.abs(res["O"][:, kept_ids] - res_off["O"][:, kept_ids]).max() == 0.0


def test_shared_softmax_merge_rule():
    """Joint result == log-sum-exp merge of (kept set only) with (extras only)."""
    shape = small_shape()
    q, k, v = draw(shape, seed=61)
    joint = orc.sga(shape, bits(q), bits(k), bits(v), want_p=True)
    kept_only = orc.sga(small_shape(flags=0), bits(q), bits(k), bits(v))
    kept = kept_mask_by_windows(shape)
    qd, kd, vd = (t.to(torch.float64).numpy() for t in (q, k, v))
    kbar = kd[:, ~kept].mean(axis=1)
    vbar = vd[:, ~kept].mean(axis=1)
    for b in range(shape.B):
        for h in range(shape.H):
            for i in range(shape.NQ):
                l_mean = shape.scale * qd[b, i, h] @ kbar[b, h]
                parts = [(l_mean, vbar[b, h])]
                if not kept[i]:
                    parts.append((shape.scale * qd[b, i, h] @ kd[b, i, h], vd[b, i, h]))
                l1 = kept_only["lse"][b, h, i]
                lse = np.logaddexp.reduce([l1] + [p[0] for p in parts])
                o = math.exp(l1 - lse) * kept_only["O"][b, i, h]
                for lg, vec in parts:
                    o = o + math.exp(lg - lse) * vec
                assert abs(joint["lse"][b, h, i] - lse) < 1e-12
                assert np.abs(joint["O"][b, i, h] - o).max() < 1e-12


def test_rows_subset_matches_full_run():
    shape = small_shape(B=2)
    q, k, v = draw(shape, seed=71)
    full = orc.sga(shape, bits(q), bits(k), bits(v))
    rows = np.array([0, 1, 2, 5, shape.L, shape.L + 3, shape.NQ - 1, 17])
    part = orc.sga(shape, bits(q), bits(k), bits(v), rows=rows)
    assert (part["O"] == full["O"][:, rows]).all()
    assert (part["lse"] == full["lse"][:, :, rows]).all()


# ----------------------------------------------------------------------------
# symmetries and bounds
# ----------------------------------------------------------------------------
def test_frame_permutation_equivariance():
    shape = small_shape(N=4, keep_first_frame=1)
    q, k, v = draw(shape, seed=81)
    L = shape.L
    perm_frames = [0, 3, 1, 2]  # frame 0 is special under the VGGT rule; permute the rest
    tok = np.concatenate([np.arange(f * L, (f + 1) * L) for f in perm_frames])
    a = orc.sga(shape, bits(q), bits(k), bits(v))
    b = orc.sga(shape, bits(q[:, tok]), bits(k[:, tok]), bits(v[:, tok]))
    assert np.abs(b["O"] - a["O"][:, tok]).max() < 1e-12
    shape_pi = small_shape(N=4, keep_first_frame=0)
    perm_all = [2, 0, 3, 1]
    tok = np.concatenate([np.arange(f * L, (f + 1) * L) for f in perm_all])
    a = orc.sga(shape_pi, bits(q), bits(k), bits(v))
    b = orc.sga(shape_pi, bits(q[:, tok]), bits(k[:, tok]), bits(v[:, tok]))
    assert np.abs(b["O"] - a["O"][:, tok]).max() < 1e-12


def test_output_is_convex_combination_and_linear_in_v():
    shape = small_shape()
    q, k, v = draw(shape, seed=91)
    res = orc.sga(shape, bits(q), bits(k), bits(v))
    vd = v.to(torch.float64).numpy()
    lo = vd.min(axis=1)[:, None]
    hi = vd.max(axis=1)[:, None]
    assert (res["O"] >= lo - 1e-12).all() and (res["O"] <= hi + 1e-12).all()
    res2 = orc.sga(shape, bits(q), bits(k), bits((2.0 * v).to(torch.bfloat16)))  # exact in bf16
    assert np.abs(res2["O"] - 2.0 * res["O"]).max() < 1e-12
    assert np.abs(res2["lse"] - res["lse"]).max() == 0.0


def test_extras_add_at_most_two_columns():
    # Sec. 4.3: the enhancement costs O(N) extra work -- two columns per query
    shape = small_shape()
    q, k, v = draw(shape, seed=95)
    res = orc.sga(shape, bits(q), bits(k), bits(v), want_p=True)
    M = len(res["idx"])
    assert res["P"].shape[-1] == M + 2
    kept = kept_mask_by_windows(shape)
    assert (res["P"][..., np.nonzero(kept)[0], M] == 0).all()
    assert (res["P"][..., np.nonzero(~kept)[0], M] > 0).all()
    assert (res["P"][..., M + 1] > 0).all()


# ----------------------------------------------------------------------------
# planted mistakes: each plausible error must trip at least one pin above.
# The mistakes live here, in reference code on the CPU, never in a kernel.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("mistake", ["self_for_all", "mean_per_frame", "mean_includes_kept",
                                      "floor_windows", "window_last_token"])
def test_pins_discriminate_planted_mistakes(mistake):
    shape = small_shape(N=3, n_h=5, n_w=7, s_h=2, s_w=3)
    q, k, v = draw(shape, seed=101)
    res = orc.sga(shape, bits(q), bits(k), bits(v))
    kept = kept_mask_by_windows(shape)
    qd, kd, vd = (t.to(torch.float64).numpy() for t in (q, k, v))
    NQ, L = shape.NQ, shape.L
    if mistake in ("floor_windows", "window_last_token"):
        wrong = np.zeros(NQ, dtype=bool)
        for f in range(shape.N):
            base = f * L
            wrong[base:base + shape.n_special] = True
            if f == 0:
                wrong[base:base + L] = True
                continue
            for top in range(0, shape.n_h, shape.s_h):
                for left in range(0, shape.n_w, shape.s_w):
                    rr = list(range(top, min(top + shape.s_h, shape.n_h)))
                    cc = list(range(left, min(left + shape.s_w, shape.n_w)))
                    if mistake == "floor_windows" and (len(rr) < shape.s_h or len(cc) < shape.s_w):
                        continue
                    r, c = (rr[0], cc[0]) if mistake == "floor_windows" else (rr[-1], cc[-1])
                    wrong[base + shape.n_special + r * shape.n_w + c] = True
        assert (wrong != kept).any()
        assert not np.array_equal(np.nonzero(wrong)[0], res["idx"])
        return
    # value-level mistakes, built as variants of the masked dense reference
    b, h = 0, 1
    kk, vv = kd[b, :, h], vd[b, :, h]
    dropped = ~kept
    if mistake == "mean_includes_kept":
        kbar, vbar = kk.mean(axis=0), vv.mean(axis=0)
    elif mistake == "mean_per_frame":
        sel = dropped.copy()
        sel[: 2 * L] = False  # last frame's dropped tokens only
        kbar, vbar = kk[sel].mean(axis=0), vv[sel].mean(axis=0)
    else:
        kbar, vbar = kk[dropped].mean(axis=0), vv[dropped].mean(axis=0)
    k_aug = np.concatenate([kk, kbar[None]])
    v_aug = np.concatenate([vv, vbar[None]])
    logits = shape.scale * qd[b, :, h] @ k_aug.T
    allow = np.zeros((NQ, NQ + 1), dtype=bool)
    allow[:, :NQ] = kept[None, :]
    allow[:, NQ] = True
    if mistake == "self_for_all":
        # wrong: a kept query counted twice -> emulate by doubling its own weight
        pass
    allow[np.arange(NQ), np.arange(NQ)] |= dropped
    logits = np.where(allow, logits, -np.inf)
    e = np.exp(logits - logits.max(axis=1, keepdims=True))
    if mistake == "self_for_all":
        ids = np.nonzero(kept)[0]
        e[ids, ids] *= 2.0
    p = e / e.sum(axis=1, keepdims=True)
    wrong_o = p @ v_aug
    assert np.abs(wrong_o - res["O"][b, :, h]).max() > 1e-4


# ----------------------------------------------------------------------------
# frame attention (Sec. 4.2): block-diagonal dense attention
# ----------------------------------------------------------------------------
def test_frame_attention_is_block_diagonal_dense_attention():
    shape = small_shape(B=2, N=3, flags=0)
    q, k, v = draw(shape, seed=111)
    rows = np.arange(shape.NQ)
    O, lse = orc.frame_rows(shape, bits(q), bits(k), bits(v), rows)
    qd, kd, vd = (t.to(torch.float64).numpy() for t in (q, k, v))
    L = shape.L
    frame_of = np.arange(shape.NQ) // L
    for b in range(shape.B):
        for h in range(shape.H):
            logits = shape.scale * qd[b, :, h] @ kd[b, :, h].T
            logits = np.where(frame_of[:, None] == frame_of[None, :], logits, -np.inf)
            mx = logits.max(axis=1, keepdims=True)
            e = np.exp(logits - mx)
            den = e.sum(axis=1, keepdims=True)
            assert np.abs(O[b, :, h] - (e / den) @ vd[b, :, h]).max() < 1e-12
            assert np.abs(lse[b, h] - (mx + np.log(den))[:, 0]).max() < 1e-12
    # one frame: frame attention is global attention
    one = small_shape(N=1, flags=0)
    q, k, v = draw(one, seed=112)
    Of, _ = orc.frame_rows(one, bits(q), bits(k), bits(v), np.arange(one.NQ))
    Od, _ = orc.dense_rows(one, bits(q), bits(k), bits(v), np.arange(one.NQ))
    assert np.abs(Of - Od).max() == 0.0


# ----------------------------------------------------------------------------
# block oracle: its pieces against library routines, its composition against a
# second way of writing it
# ----------------------------------------------------------------------------
def test_block_oracle_pieces_and_composition():
    from oracle import block_oracle as blk

    rng = np.random.default_rng(5)
    # bf16 rounding helper: round-to-nearest-even, ties checked on exact halves
    vals = np.array([1.0, 1.00390625, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5, 3.0e38, 1e-40])
    want = torch.tensor(vals, dtype=torch.float64).to(torch.float32).to(torch.bfloat16)
    got = blk.from_bf16_bits(blk.to_bf16_bits(vals))
    assert np.array_equal(got, want.to(torch.float64).numpy())
    # LayerNorm and linear against torch in float64
    x = rng.standard_normal((3, 7, 128))
    gamma, beta = rng.standard_normal(128), rng.standard_normal(128)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (128,), torch.from_numpy(gamma),
                                         torch.from_numpy(beta), eps=1e-6).numpy()
    assert np.abs(blk.layernorm(x, gamma, beta, 1e-6) - ref).max() < 1e-12
    w, b = rng.standard_normal((64, 128)), rng.standard_normal(64)
    ref = torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b))
    assert np.abs(blk.linear(x, w, b) - ref.numpy()).max() < 1e-12
    # composition: with identity projections, unit LayerNorm scale and zero biases the block is
    # x + Attn(LN(x), LN(x), LN(x)) on the bf16-rounded LayerNorm output
    shape = small_shape(B=1, N=2, n_h=3, n_w=4, H=2, D=8, flags=orc.DIAG | orc.MEAN)
    C = shape.H * shape.D
    xb = blk.to_bf16_bits(rng.standard_normal((1, shape.NQ, C)))
    eye = np.eye(C)
    wts = dict(ln_gamma=np.ones(C), ln_beta=np.zeros(C), ln_eps=1e-6, w_q=eye, w_k=eye, w_v=eye,
               w_o=eye)
    for mode in (blk.SGA, blk.FRAME, blk.DENSE):
        y = blk.block(shape, mode, xb, wts)
        x = blk.from_bf16_bits(xb)
        xn = blk.to_bf16_bits(blk.layernorm(x, 1.0, 0.0, 1e-6)).reshape(1, shape.NQ, shape.H, shape.D)
        rows = np.arange(shape.NQ)
        if mode == blk.SGA:
            o = orc.sga(shape, xn, xn, xn)["O"]
        elif mode == blk.FRAME:
            o, _ = orc.frame_rows(shape, xn, xn, xn, rows)
        else:
            o, _ = orc.dense_rows(shape, xn, xn, xn, rows)
        o = blk.from_bf16_bits(blk.to_bf16_bits(o)).reshape(1, shape.NQ, C)
        assert np.array_equal(y, blk.from_bf16_bits(blk.to_bf16_bits(x + o)))
    # distinct random projections and biases, dense mode, against the formula written out with
    # torch float64 ops (catches swapped projections, a transposed weight, a dropped bias or
    # residual)
    t = torch.from_numpy
    rb = lambda a: blk.from_bf16_bits(blk.to_bf16_bits(a))
    wts = dict(ln_gamma=1.0 + 0.1 * rng.standard_normal(C), ln_beta=0.1 * rng.standard_normal(C),
               ln_eps=1e-6)
    for name in "qkvo":
        wts["w_" + name] = rb(rng.standard_normal((C, C)) / np.sqrt(C))
        wts["b_" + name] = 0.05 * rng.standard_normal(C)
    y = blk.block(shape, blk.DENSE, xb, wts)
    x = t(blk.from_bf16_bits(xb))
    xn = t(rb(torch.nn.functional.layer_norm(x, (C,), t(wts["ln_gamma"]), t(wts["ln_beta"]),
                                             eps=1e-6).numpy()))
    proj = {n: t(rb(torch.nn.functional.linear(xn, t(wts["w_" + n]), t(wts["b_" + n])).numpy()))
            .view(1, shape.NQ, shape.H, shape.D).permute(0, 2, 1, 3) for n in "qkv"}
    att = torch.nn.functional.scaled_dot_product_attention(proj["q"], proj["k"], proj["v"],
                                                           scale=shape.scale)
    att = t(rb(att.permute(0, 2, 1, 3).reshape(1, shape.NQ, C).numpy()))
    want = rb((x + torch.nn.functional.linear(att, t(wts["w_o"]), t(wts["b_o"]))).numpy())
    # float64 sums in a different order can flip a bf16 rounding on a handful of entries
    assert (y != want).mean() < 2e-3 and np.abs(y - want).max() < 2.0 ** -6


# ----------------------------------------------------------------------------
# List-driven oracle (token-selection ablation of the supplementary material)
# ----------------------------------------------------------------------------
def _list_shape(**kw):
    return small_shape(**kw)


@pytest.mark.parametrize("keep_first", [0, 1])
def test_list_first_rule_is_the_grid_rule(keep_first):
    from oracle import list_oracle as lo

    shape = _list_shape(B=2, keep_first_frame=keep_first)
    q, k, v = draw(shape, seed=61)
    lst, _ = lo.select(shape, lo.FIRST, 0, None)
    assert (lst == orc.kept_indices(shape)[None, :]).all()
    rows = np.arange(shape.NQ)
    O, lse, km, vm, nd = lo.attn_rows(shape, lst, bits(q), bits(k), bits(v), rows)
    res = orc.sga(shape, bits(q), bits(k), bits(v))
    assert (nd == res["n_dropped"]).all()
    assert np.abs(O - res["O"]).max() < 1e-11
    assert np.abs(lse - res["lse"]).max() < 1e-11
    assert np.abs(km - res["kmean"]).max() < 1e-12 and np.abs(vm - res["vmean"]).max() < 1e-12


def test_list_of_all_tokens_is_dense_attention_and_order_is_irrelevant():
    from oracle import list_oracle as lo

    shape = _list_shape()
    q, k, v = draw(shape, seed=62)
    rows = np.arange(shape.NQ)
    rng = np.random.default_rng(5)
    everything = rng.permutation(shape.NQ).astype(np.int32)[None, :]
    O, lse, _, _, nd = lo.attn_rows(shape, everything, bits(q), bits(k), bits(v), rows)
    want = torch.nn.functional.scaled_dot_product_attention(
        q.double().permute(0, 2, 1, 3), k.double().permute(0, 2, 1, 3), v.double().permute(0, 2, 1, 3),
        scale=shape.scale).permute(0, 2, 1, 3).numpy()
    assert nd[0] == 0
    assert np.abs(O - want).max() < 1e-11
    # a shuffled subset gives the same result as the sorted one
    sub = np.sort(rng.choice(shape.NQ, size=shape.NQ // 3, replace=False)).astype(np.int32)
    a = lo.attn_rows(shape, sub[None, :], bits(q), bits(k), bits(v), rows)
    b = lo.attn_rows(shape, rng.permutation(sub)[None, :], bits(q), bits(k), bits(v), rows)
    assert np.abs(a[0] - b[0]).max() < 1e-12 and np.abs(a[1] - b[1]).max() < 1e-12


@pytest.mark.parametrize("flags", [0, 1, 2, 3])
def test_list_attention_equals_masked_dense_attention(flags):
    """Random lists that contain every special token (so that 'unlisted' and 'unlisted patch'
    coincide) against the masked dense reference; batch elements get different lists."""
    from oracle import list_oracle as lo

    shape = _list_shape(B=2, flags=flags)
    q, k, v = draw(shape, seed=63 + flags)
    rng = np.random.default_rng(11 + flags)
    L, P = shape.L, shape.n_special
    special = np.array([f * L + p for f in range(shape.N) for p in range(P)])
    patches = np.array([t for t in range(shape.NQ) if t % L >= P])
    n_pick = 17
    lists = np.stack([np.concatenate([special, rng.choice(patches, n_pick, replace=False)])
                      for _ in range(shape.B)]).astype(np.int32)
    rows = np.arange(shape.NQ)
    O, lse, _, _, nd = lo.attn_rows(shape, lists, bits(q), bits(k), bits(v), rows)
    assert (nd == len(patches) - n_pick).all()
    for b in range(shape.B):
        kept = np.zeros(shape.NQ, dtype=bool)
        kept[lists[b]] = True
        one = orc.Shape(**{**shape.__dict__, "B": 1})
        wo, wl, _ = masked_dense_reference(one, q[b:b + 1], k[b:b + 1], v[b:b + 1], kept,
                                           bool(flags & 1), bool(flags & 2))
        assert np.abs(O[b] - wo[0]).max() < 1e-11
        assert np.abs(lse[b] - wl[0]).max() < 1e-11


def test_list_unlisted_special_token_gets_self_term_but_is_not_averaged():
    from oracle import list_oracle as lo

    shape = _list_shape(N=1, n_h=2, n_w=2, n_special=1, H=1, keep_first_frame=0)
    q, k, v = draw(shape, seed=64)          # tokens: 0 special, 1..4 patches
    lst = np.array([[1, 3]], dtype=np.int32)
    O, lse, km, vm, nd = lo.attn_rows(shape, lst, bits(q), bits(k), bits(v), [0, 2])
    kd, vd, qd = (t.double().numpy()[0, :, 0] for t in (k, v, q))
    assert nd[0] == 2 and np.allclose(km[0, 0], (kd[2] + kd[4]) / 2, atol=1e-15)
    for r, i in enumerate((0, 2)):
        cols_k = np.stack([kd[1], kd[3], kd[i], (kd[2] + kd[4]) / 2])
        cols_v = np.stack([vd[1], vd[3], vd[i], (vd[2] + vd[4]) / 2])
        z = shape.scale * cols_k @ qd[i]
        p = np.exp(z - z.max())
        p /= p.sum()
        assert np.abs(O[0, r, 0] - p @ cols_v).max() < 1e-13


def test_selection_rules_pick_inside_their_window():
    from oracle import list_oracle as lo

    shape = _list_shape(B=2, N=4, n_h=7, n_w=8, s_h=3, s_w=3, keep_first_frame=1)
    q, k, v = draw(shape, seed=65)
    grid = orc.kept_indices(shape)
    L, P = shape.L, shape.n_special
    kd = k.double().numpy().reshape(shape.B, shape.NQ, -1)
    mag = (kd * kd).sum(-1)
    for rule in (lo.RANDOM, lo.HIGH, lo.LOW):
        lst, _ = lo.select(shape, rule, 1234, bits(k))
        assert lst.shape == (shape.B, len(grid))
        for b in range(shape.B):
            assert len(set(lst[b].tolist())) == len(grid)   # one distinct token per position
            for m, g in enumerate(grid):
                t = int(lst[b, m])
                if g % L < P or g // L == 0:
                    assert t == g                             # special tokens, reference frame
                    continue
                assert t // L == g // L
                gr, gc = divmod(g % L - P, shape.n_w)
                tr, tc = divmod(t % L - P, shape.n_w)
                assert gr <= tr < min(gr + shape.s_h, shape.n_h)
                assert gc <= tc < min(gc + shape.s_w, shape.n_w)
                if rule != lo.RANDOM:                         # explicit loop over the window
                    window = [g // L * L + P + r * shape.n_w + c
                              for r in range(gr, min(gr + shape.s_h, shape.n_h))
                              for c in range(gc, min(gc + shape.s_w, shape.n_w))]
                    best = max(window, key=lambda x: mag[b, x]) if rule == lo.HIGH else \
                        min(window, key=lambda x: mag[b, x])
                    assert mag[b, t] == mag[b, best]


def test_random_rule_is_uniform_over_cells_and_depends_on_seed():
    from oracle import list_oracle as lo

    counts = np.zeros(4)
    for w in range(4000):
        counts[lo.random_cell(99, 0, 1 + w % 7, w, 8, 4)] += 1
    assert (np.abs(counts - 1000) < 130).all(), counts          # ~4.7 sigma of a fair draw
    a = [lo.random_cell(1, 0, 1, w, 8, 9) for w in range(64)]
    b = [lo.random_cell(2, 0, 1, w, 8, 9) for w in range(64)]
    c = [lo.random_cell(1 + (1 << 32), 0, 1, w, 8, 9) for w in range(64)]
    assert a != b and a != c
    assert all(0 <= x < 9 for x in a)


def test_cell_mean_pooling_oracle():
    from oracle import list_oracle as lo

    shape = _list_shape(B=2, N=3, n_h=5, n_w=7, s_h=2, s_w=3, keep_first_frame=1)
    q, k, v = draw(shape, seed=66)
    kp, vp, groups = lo.pool(shape, bits(k), bits(v))
    grid = orc.kept_indices(shape)
    assert kp.shape == (shape.B, shape.H, len(grid), shape.D)
    assert [g[0] for g in groups] == grid.tolist()           # a row stands where its first token stood
    kd = k.double().numpy()
    L, P = shape.L, shape.n_special
    for m, g0 in enumerate(grid):                             # explicit loop over each window
        if g0 % L < P or g0 // L == 0:
            assert np.array_equal(kp[:, :, m], kd[:, g0])
            continue
        r0, c0 = divmod(g0 % L - P, shape.n_w)
        acc = np.zeros_like(kd[:, 0])
        n = 0
        for r in range(r0, min(r0 + shape.s_h, shape.n_h)):
            for c in range(c0, min(c0 + shape.s_w, shape.n_w)):
                acc += kd[:, g0 // L * L + P + r * shape.n_w + c]
                n += 1
        assert n == len(groups[m]) and np.abs(kp[:, :, m] - acc / n).max() < 1e-14
    # every patch of a subsampled frame is averaged exactly once
    seen = sorted(t for g in groups for t in g)
    assert seen == list(range(shape.NQ))
    # strides (1,1): nothing is pooled, attention over the rows is dense attention
    one = _list_shape(B=1, s_h=1, s_w=1)
    q1, k1, v1 = draw(one, seed=67)
    kp1, vp1, _ = lo.pool(one, bits(k1), bits(v1))
    assert np.array_equal(kp1, k1.double().numpy().transpose(0, 2, 1, 3))
    rows = np.arange(one.NQ)
    O, lse = lo.attn_over_rows(one, bits(q1), kp1, vp1, rows)
    want, want_lse = orc.dense_rows(one, bits(q1), bits(k1), bits(v1), rows)
    assert np.abs(O - want).max() < 1e-11 and np.abs(lse - want_lse).max() < 1e-11
    # K and V constant inside every window: the mean is the first token, and the result is the
    # subsample-only variant of the grid rule
    kc, vc = k.clone(), v.clone()
    for g in groups:
        kc[:, g] = k[:, g[0]:g[0] + 1]
        vc[:, g] = v[:, g[0]:g[0] + 1]
    kp2, vp2, _ = lo.pool(shape, bits(kc), bits(vc))
    O2, _ = lo.attn_over_rows(shape, bits(q), kp2, vp2, np.arange(shape.NQ))
    plain = orc.Shape(**{**shape.__dict__, "flags": 0})
    assert np.abs(O2 - orc.sga(plain, bits(q), bits(kc), bits(vc))["O"]).max() < 1e-11
    # rounding helper: exact on representable values, nearest-even otherwise
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -0.3])
    r = lo.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2.0 ** -6 and abs(r[3] + 0.3) < 2.0 ** -9 * 0.3 * 2


def test_shift_of_keys_orthogonal_to_the_query_changes_nothing():
    """Adding to EVERY key a vector orthogonal to q_i shifts none of row i's logits (kept columns,
    self column, mean column alike), so o_i is unchanged; values are dyadic so that the shifted
    keys are exact in bf16."""
    shape = small_shape(H=1, flags=orc.DIAG | orc.MEAN, mean_logit_bias=0.5)
    rng = np.random.default_rng(17)
    NQ, D = shape.NQ, shape.D
    k = torch.tensor(rng.integers(-16, 17, size=(1, NQ, 1, D)) / 8.0, dtype=torch.float32)
    v = torch.tensor(rng.integers(-16, 17, size=(1, NQ, 1, D)) / 8.0, dtype=torch.float32)
    q = torch.tensor(rng.integers(-8, 9, size=(1, NQ, 1, D)) / 8.0, dtype=torch.float32)
    u = torch.zeros(D)
    rows = [3, 20, shape.L + shape.n_special + 1, NQ - 1]     # special, frame-0, dropped, last
    for i in rows:
        q[0, i, 0] = torch.tensor([1.0, 1.0, 0.5, -0.5] + [0.0] * (D - 4))
    u[:4] = torch.tensor([1.0, -1.0, 1.0, 1.0])               # q_i . u = 1 - 1 + 0.5 - 0.5 = 0
    k2 = k + u.view(1, 1, 1, D)
    qb, vb = bits(q.to(torch.bfloat16)), bits(v.to(torch.bfloat16))
    assert torch.equal(k2.to(torch.bfloat16).float(), k2)     # still exact
    a = orc.sga(shape, qb, bits(k.to(torch.bfloat16)), vb, rows=np.array(rows))
    b = orc.sga(shape, qb, bits(k2.to(torch.bfloat16)), vb, rows=np.array(rows))
    assert np.abs(a["O"] - b["O"]).max() < 1e-13
    assert np.abs(a["lse"] - b["lse"]).max() < 1e-13
    # a shift that is NOT orthogonal does change the dropped query's row (the pin has teeth)
    k3 = k + torch.tensor([1.0] + [0.0] * (D - 1)).view(1, 1, 1, D) * (torch.arange(NQ) % 2).view(1, NQ, 1, 1)
    c = orc.sga(shape, qb, bits(k3.to(torch.bfloat16)), vb, rows=np.array(rows))
    assert np.abs(a["O"] - c["O"]).max() > 1e-3
