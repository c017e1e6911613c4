"""CPU oracle for attention over a caller-supplied kept list -- TEST INFRASTRUCTURE ONLY.

Plain numpy in float64; shares nothing with the HIP path.  Covers the token-selection
ablation of the AVGGT paper's supplementary material ("Effect of the Grid-Based
Subsampling Strategy"): within each s_h x s_w window keep, instead of the first token, a
random one, the one with the highest or the one with the lowest feature magnitude; the
attention itself is Sec. 4.3's -- kept set, self term, mean component, one softmax.

Definitions used here (the readings are listed with the other readings of the paper):
  * a list may hold any tokens in any order; the self term goes to every query whose token
    is not listed; the mean component averages K resp. V over the patch tokens (slot >=
    n_special) that are not listed and exists when there is at least one;
  * feature magnitude of a token = sum of squares of its K row over all heads;
  * the random choice is a counter-based hash of (seed, batch, frame, window), written out
    in ``random_cell`` below, taken modulo the number of cells of the (clipped) window.

The paper prints no number that depends on the definition of "feature magnitude", on the
random generator or on how an arbitrary list treats unlisted special tokens: parity unpinned
for those three choices (the attention over a given list is pinned as below).

Pins (tests/test_oracle_pins.py): the FIRST rule reproduces the grid rule's index list and
the C oracle's outputs; a list of all tokens gives dense attention; list order does not
matter; brute-force masked dense attention on random lists; window membership, one pick per
window and uniformity of the random rule; HIGH/LOW against an explicit loop.
"""
from __future__ import annotations

import numpy as np

FIRST, RANDOM, HIGH, LOW = 0, 1, 2, 3
DIAG, MEAN = 1, 2
_M32 = 0xFFFFFFFF


def _widen(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _mix(x: int) -> int:
    x &= _M32
    x ^= x >> 16
    x = (x * 0x7FEB352D) & _M32
    x ^= x >> 15
    x = (x * 0x846CA68B) & _M32
    x ^= x >> 16
    return x


def random_cell(seed: int, b: int, frame: int, window: int, n_frames: int, cells: int) -> int:
    s = (seed & _M32) ^ (((seed >> 32) & _M32) * 0x9E3779B1 & _M32)
    x = _mix(s ^ (((b * n_frames + frame) * 0x85EBCA77) & _M32))
    x = _mix(x ^ ((window * 0xC2B2AE3D) & _M32))
    return x % cells


def windows(shape):
    """[(row0, col0, rows, cols)] of a frame's windows in row-major window order (windows are
    anchored at the grid origin; edge windows are clipped, Sec. 4.3)."""
    out = []
    for r0 in range(0, shape.n_h, shape.s_h):
        for c0 in range(0, shape.n_w, shape.s_w):
            out.append((r0, c0, min(shape.s_h, shape.n_h - r0), min(shape.s_w, shape.n_w - c0)))
    return out


def select(shape, rule: int, seed: int, k_bits: np.ndarray):
    """int32 [B, M]: per batch element the kept tokens, position by position in the order of the
    grid rule's ascending list.  Also returns, for HIGH/LOW, each window's candidate tokens and
    float64 magnitudes so that a test can accept near-ties."""
    P, T = shape.n_special, shape.n_h * shape.n_w
    L = P + T
    NQ = shape.N * L
    wins = windows(shape)
    mag = None
    if rule in (HIGH, LOW):
        k = _widen(k_bits).reshape(shape.B, NQ, -1)
        mag = (k * k).sum(axis=2)
    lists, cands = [], []
    for b in range(shape.B):
        row, cb = [], []
        for f in range(shape.N):
            base = f * L
            row.extend(range(base, base + P))
            cb.extend([None] * P)
            if f == 0 and shape.keep_first_frame:
                row.extend(range(base + P, base + L))
                cb.extend([None] * T)
                continue
            for w, (r0, c0, nr, nc) in enumerate(wins):
                cells = [base + P + (r0 + i) * shape.n_w + (c0 + j) for i in range(nr) for j in range(nc)]
                if rule == FIRST:
                    pick = 0
                elif rule == RANDOM:
                    pick = random_cell(seed, b, f, w, shape.N, len(cells))
                else:
                    m = mag[b, cells]
                    pick = int(np.argmax(m)) if rule == HIGH else int(np.argmin(m))  # first on ties
                row.append(cells[pick])
                cb.append((cells, None if mag is None else mag[b, cells]))
        lists.append(row)
        cands.append(cb)
    return np.asarray(lists, dtype=np.int32), cands


def mean_terms(shape, kv_list: np.ndarray, k_bits, v_bits):
    """kmean, vmean float64 [B, H, D] over the unlisted patch tokens, and their count [B]."""
    P, L = shape.n_special, shape.n_special + shape.n_h * shape.n_w
    NQ = shape.N * L
    k = _widen(k_bits).reshape(shape.B, NQ, shape.H, shape.D)
    v = _widen(v_bits).reshape(shape.B, NQ, shape.H, shape.D)
    km = np.zeros((shape.B, shape.H, shape.D))
    vm = np.zeros_like(km)
    nd = np.zeros(shape.B, dtype=np.int64)
    for b in range(shape.B):
        listed = np.zeros(NQ, dtype=bool)
        listed[kv_list[b]] = True
        dropped = [t for t in range(NQ) if (t % L) >= P and not listed[t]]
        nd[b] = len(dropped)
        if dropped:
            km[b] = k[b, dropped].sum(axis=0) / len(dropped)
            vm[b] = v[b, dropped].sum(axis=0) / len(dropped)
    return km, vm, nd


def attn_rows(shape, kv_list: np.ndarray, q_bits, k_bits, v_bits, rows):
    """O float64 [B, nrows, H, D] and lse [B, H, nrows] for the listed query rows."""
    L = shape.n_special + shape.n_h * shape.n_w
    NQ = shape.N * L
    B, H, D = shape.B, shape.H, shape.D
    q = _widen(q_bits).reshape(B, NQ, H, D)
    k = _widen(k_bits).reshape(B, NQ, H, D)
    v = _widen(v_bits).reshape(B, NQ, H, D)
    km, vm, nd = mean_terms(shape, kv_list, k_bits, v_bits)
    rows = np.asarray(rows, dtype=np.int64)
    scale = float(np.float32(shape.scale))
    O = np.zeros((B, len(rows), H, D))
    lse = np.zeros((B, H, len(rows)))
    for b in range(B):
        listed = np.zeros(NQ, dtype=bool)
        listed[kv_list[b]] = True
        use_mean = bool(shape.flags & MEAN) and nd[b] > 0
        for h in range(H):
            kc = k[b, kv_list[b], h]          # explicit compacted copy [M, D]
            vc = v[b, kv_list[b], h]
            for r, i in enumerate(rows):
                logits = [scale * (kc @ q[b, i, h])]
                values = [vc]
                if (shape.flags & DIAG) and not listed[i]:
                    logits.append(np.array([scale * (k[b, i, h] @ q[b, i, h])]))
                    values.append(v[b, i, h][None, :])
                if use_mean:
                    logits.append(np.array([scale * (km[b, h] @ q[b, i, h]) +
                                            float(np.float32(shape.mean_logit_bias))]))
                    values.append(vm[b, h][None, :])
                z = np.concatenate(logits)
                vals = np.concatenate(values, axis=0)
                mx = z.max()
                e = np.exp(z - mx)
                den = e.sum()
                O[b, r, h] = (e / den) @ vals
                lse[b, h, r] = mx + np.log(den)
    return O, lse, km, vm, nd


def pool(shape, k_bits, v_bits):
    """Cell-mean variant of the same ablation: float64 [B, H, M, D] key and value rows where a
    window's row is the mean over the window's tokens; special tokens and a whole-kept frame 0
    are copied.  Rows are in the order of the grid rule's ascending list."""
    P, T = shape.n_special, shape.n_h * shape.n_w
    L = P + T
    NQ = shape.N * L
    k = _widen(k_bits).reshape(shape.B, NQ, shape.H, shape.D)
    v = _widen(v_bits).reshape(shape.B, NQ, shape.H, shape.D)
    groups = []                       # token ids averaged into each row
    for f in range(shape.N):
        base = f * L
        groups.extend([[base + p] for p in range(P)])
        if f == 0 and shape.keep_first_frame:
            groups.extend([[base + P + t] for t in range(T)])
            continue
        for (r0, c0, nr, nc) in windows(shape):
            groups.append([base + P + (r0 + i) * shape.n_w + (c0 + j)
                           for i in range(nr) for j in range(nc)])
    kp = np.stack([k[:, g].mean(axis=1) for g in groups], axis=2)   # [B, H, M, D]
    vp = np.stack([v[:, g].mean(axis=1) for g in groups], axis=2)
    return kp, vp, groups


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float64 -> nearest bf16 value (ties to even), returned as float64."""
    f = x.astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def attn_over_rows(shape, q_bits, kp, vp, rows):
    """Plain softmax attention of the listed queries over given key/value rows [B, H, M, D]."""
    L = shape.n_special + shape.n_h * shape.n_w
    NQ = shape.N * L
    q = _widen(q_bits).reshape(shape.B, NQ, shape.H, shape.D)
    rows = np.asarray(rows, dtype=np.int64)
    scale = float(np.float32(shape.scale))
    O = np.zeros((shape.B, len(rows), shape.H, shape.D))
    lse = np.zeros((shape.B, shape.H, len(rows)))
    for b in range(shape.B):
        for h in range(shape.H):
            z = scale * (q[b, rows, h] @ kp[b, h].T)          # [nrows, M]
            mx = z.max(axis=1, keepdims=True)
            e = np.exp(z - mx)
            den = e.sum(axis=1, keepdims=True)
            O[b, :, h] = (e / den) @ vp[b, h]
            lse[b, h] = (mx + np.log(den))[:, 0]
    return O, lse
