"""Host-side behaviour of libagg.so, checked without a GPU: exported symbols,
counts and index lists against the oracle's enumeration, the fragment-order
offset maps, and every error path that is decided before a launch."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

from oracle import sga_oracle as orc
from paper_2512_02541_amd import binding as agg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def oshape(s):
    return orc.Shape(s.B, s.N, s.n_h, s.n_w, s.n_special, s.H, s.D, s.s_h, s.s_w,
                     s.keep_first_frame, s.flags, s.scale, s.mean_logit_bias)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "agg.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(agg_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = agg.lib()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(agg.EXPORTS)


def test_sigma_table():
    assert agg.agg_sigma_to_strides(2) == (1, 2)
    assert agg.agg_sigma_to_strides(4) == (2, 2)
    assert agg.agg_sigma_to_strides(6) == (2, 3)
    assert agg.agg_sigma_to_strides(9) == (3, 3)
    assert agg.agg_sigma_to_strides(1) == (1, 1)
    for s in (2, 4, 6, 9):
        assert agg.agg_sigma_to_strides(s) == orc.sigma_to_strides(s)
    with pytest.raises(agg.AggError) as e:
        agg.agg_sigma_to_strides(5)
    assert e.value.status == -2


GRIDS = [(1, 1), (1, 5), (4, 4), (5, 7), (7, 3), (16, 16), (37, 37), (28, 37)]
STRIDES = [(1, 1), (1, 2), (2, 2), (2, 3), (3, 3), (4, 1), (5, 9)]


@pytest.mark.parametrize("keep_first", [0, 1])
@pytest.mark.parametrize("n_special", [0, 5])
def test_counts_and_indices_match_oracle_enumeration(keep_first, n_special):
    for (n_h, n_w) in GRIDS:
        for (s_h, s_w) in STRIDES:
            for N in (1, 2, 5):
                s = agg.make_shape(1, N, n_h, n_w, n_special, 16, 64, s_h, s_w, keep_first)
                o = oshape(s)
                M, nd = agg.agg_kv_count(s)
                assert (M, nd) == orc.counts(o), (n_h, n_w, s_h, s_w, N)
                idx = agg.agg_kv_indices_host(s)
                assert (idx == orc.kept_indices(o)).all()
                dropped = agg.agg_dropped_indices_host(s)
                want = np.setdiff1d(np.arange(s.NQ, dtype=np.int32), idx)
                assert (dropped == want).all(), (n_h, n_w, s_h, s_w, N)
                nbytes, m_pad = agg.agg_kv_compact_bytes(s)
                assert m_pad % 64 == 0 and 0 <= m_pad - M < 64
                assert nbytes == s.B * s.H * m_pad * 64 * 2


def test_workload_counts():
    from paper_2512_02541_amd.inputs import WORKLOADS

    want = {"tiny": (330, 192), "f100": (71466, 65934), "f300": (110808, 301392),
            "f333": (122886, 334656), "f800": (140400, 958800)}
    for name, w in WORKLOADS.items():
        s = agg.make_shape(w.B, w.N, w.n_h, w.n_w, w.n_special, w.H, w.D, w.s_h, w.s_w,
                           w.keep_first_frame)
        assert agg.agg_kv_count(s) == want[name]


def test_fragment_order_offsets_are_tile_bijections():
    for fn in (agg.agg_kc_offset, agg.agg_vc_offset):
        seen = np.zeros(2 * 4096, dtype=np.int32)
        for m in range(128):
            for d in range(64):
                off = fn(m, d)
                assert (m // 64) * 4096 <= off < (m // 64 + 1) * 4096
                seen[off] += 1
        assert (seen == 1).all()
    # 16-byte operand groups: K keeps 8 consecutive channels of a row together,
    # V keeps 8 rows of one channel together
    for m in range(64):
        for d0 in range(0, 64, 8):
            offs = [agg.agg_kc_offset(m, d0 + e) for e in range(8)]
            assert offs == list(range(offs[0], offs[0] + 8)) and offs[0] % 8 == 0
    for d in range(64):
        for t in range(4):
            for g in range(2):
                rows = [16 * t + 8 * (e // 4) + 4 * g + e % 4 for e in range(8)]
                offs = [agg.agg_vc_offset(r, d) for r in rows]
                assert offs == list(range(offs[0], offs[0] + 8)) and offs[0] % 8 == 0


def test_error_paths_before_any_launch():
    lib = agg.lib()
    good = agg.make_shape(1, 2, 16, 16, 5, 16, 64, 2, 2)
    m = ctypes.c_int64(0)

    def count_status(**kw):
        s = agg.make_shape(1, 2, 16, 16, 5, 16, 64, 2, 2)
        for k, v in kw.items():
            setattr(s, k, v)
        return lib.agg_kv_count(ctypes.byref(s), ctypes.byref(m), None)

    assert count_status() == 0
    assert lib.agg_kv_count(None, ctypes.byref(m), None) == -1
    assert count_status(N=0) == -2
    assert count_status(s_h=0) == -2
    assert count_status(flags=4) == -2
    assert count_status(keep_first_frame=2) == -2
    assert count_status(scale=0.0) == -2
    assert count_status(scale=float("nan")) == -2
    assert count_status(D=128) == -3
    assert count_status(N=2000000, n_h=37, n_w=37) == -6
    assert "NULL" in agg.status_string(-1)
    assert agg.status_string(0) == "ok"

    fake = ctypes.c_void_p(0x1000)  # aligned, never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1008)
    ws = agg.agg_workspace_bytes(good)
    assert ws > 0
    sub = lib.agg_kv_subsample
    assert sub(ctypes.byref(good), None, fake, fake, fake, None, fake, fake, fake, ws, None) == -1
    assert sub(ctypes.byref(good), fake, fake, fake, fake, None, None, fake, fake, ws, None) == -1
    assert sub(ctypes.byref(good), odd, fake, fake, fake, None, fake, fake, fake, ws, None) == -4
    assert sub(ctypes.byref(good), fake, fake, fake, fake, None, fake, fake, fake, ws - 1, None) == -5
    att = lib.agg_global_attn_fwd
    assert att(ctypes.byref(good), fake, fake, fake, fake, fake, fake, fake, None, None, None) == -1
    assert att(ctypes.byref(good), fake, fake, odd, fake, fake, fake, fake, fake, None, None) == -4
    bad = agg.make_shape(1, 2, 16, 16, 5, 16, 32, 2, 2)
    assert att(ctypes.byref(bad), fake, fake, fake, fake, fake, fake, fake, fake, None, None) == -3
    den = lib.agg_dense_global_attn_fwd
    assert den(ctypes.byref(good), fake, fake, fake, None, None, None) == -1
    assert den(ctypes.byref(good), fake, fake, fake, odd, None, None) == -4
    assert den(ctypes.byref(bad), fake, fake, fake, fake, None, None) == -3

    # frame attention, the index-driven call and the block: same validation before any launch
    fr = lib.agg_frame_attn_fwd
    assert fr(ctypes.byref(good), fake, fake, None, fake, None, None) == -1
    assert fr(ctypes.byref(good), fake, odd, fake, fake, None, None) == -4
    ix = lib.agg_global_attn_fwd_idx
    assert ix(ctypes.byref(good), fake, fake, fake, None, fake, fake, fake, None, None) == -1
    assert ix(ctypes.byref(good), fake, fake, fake, fake, fake, odd, fake, None, None) == -4
    far = agg.make_shape(1, 13000, 37, 37, 5, 16, 64, 2, 2)   # 17.9 M tokens: beyond 24-bit ids
    assert ix(ctypes.byref(far), fake, fake, fake, fake, fake, fake, fake, None, None) == -6
    # the subsample call takes both compacted tensors or neither
    assert sub(ctypes.byref(good), fake, fake, None, fake, None, fake, fake, fake, ws, None) == -1
    w = agg.agg_block_weights(0x1000, 0x1000, 1e-6, 0x1000, 0x1000, 0x1000, 0x1000, None, None,
                              None, None)
    blk = lib.agg_global_block_fwd
    for mode in (agg.AGG_BLOCK_SGA, agg.AGG_BLOCK_FRAME, agg.AGG_BLOCK_DENSE):
        bws = agg.agg_block_workspace_bytes(good, mode)
        assert bws >= 5 * 522 * 1024 * 2   # five activations; SGA adds its compacted set
        other = ctypes.c_void_p(0x2000)
        assert blk(ctypes.byref(good), mode, ctypes.byref(w), fake, other, fake, bws - 1, None) == -5
        assert blk(ctypes.byref(good), mode, ctypes.byref(w), None, other, fake, bws, None) == -1
        assert blk(ctypes.byref(good), mode, None, fake, other, fake, bws, None) == -1
        assert blk(ctypes.byref(good), mode, ctypes.byref(w), fake, fake, fake, bws, None) == -2  # y aliases x
    assert agg.agg_block_workspace_bytes(good, 7) == 0
    wide = agg.make_shape(1, 2, 16, 16, 5, 65, 64, 2, 2)    # 4160 channels: beyond the LayerNorm's row
    assert blk(ctypes.byref(wide), agg.AGG_BLOCK_SGA, ctypes.byref(w), fake, ctypes.c_void_p(0x2000),
               fake, 1 << 40, None) == -3
    assert blk(ctypes.byref(good), 7, ctypes.byref(w), fake, fake, fake, 1 << 40, None) == -2

    # caller-supplied lists
    nbytes, m_pad = agg.agg_list_compact_bytes(good, 65)
    assert (nbytes, m_pad) == (1 * 16 * 128 * 64 * 2, 128)
    sz, mp = ctypes.c_size_t(0), ctypes.c_int64(0)
    assert lib.agg_list_compact_bytes(ctypes.byref(good), 0, ctypes.byref(sz), ctypes.byref(mp)) == -2
    lws = agg.agg_list_workspace_bytes(good)
    assert lws > 0
    sel = lib.agg_select_kv_indices
    assert sel(ctypes.byref(good), 9, 0, fake, fake, None) == -2
    assert sel(ctypes.byref(good), agg.AGG_SELECT_HIGH, 0, None, fake, None) == -1
    assert sel(ctypes.byref(good), agg.AGG_SELECT_RANDOM, 0, None, None, None) == -1
    sl = lib.agg_kv_subsample_list
    assert sl(ctypes.byref(good), fake, 65, fake, fake, fake, fake, fake, fake, fake, fake, fake,
              lws - 1, None) == -5
    assert sl(ctypes.byref(good), None, 65, fake, fake, fake, fake, fake, fake, fake, fake, fake,
              lws, None) == -1
    assert sl(ctypes.byref(good), fake, 0, fake, fake, fake, fake, fake, fake, fake, fake, fake,
              lws, None) == -2
    pool = lib.agg_kv_pool
    assert pool(ctypes.byref(good), fake, fake, fake, None, None) == -1
    assert pool(ctypes.byref(good), fake, odd, fake, fake, None) == -4
    assert pool(ctypes.byref(bad), fake, fake, fake, fake, None) == -3
    al = lib.agg_global_attn_fwd_list
    assert al(ctypes.byref(good), 65, fake, fake, fake, fake, fake, fake, fake, None, fake, fake,
              None, None) == -1
    assert al(ctypes.byref(good), 65, fake, fake, fake, fake, odd, fake, fake, fake, fake, fake,
              None, None) == -4


def test_missing_library_is_an_error(monkeypatch):
    monkeypatch.setattr(agg, "_lib", None)
    monkeypatch.setattr(agg, "LIB_PATH", os.path.join(ROOT, "does_not_exist", "libagg.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        agg.lib()


def test_decode_compact_inverts_the_documented_layout():
    import torch

    from paper_2512_02541_amd import harness

    M_pad = 128
    for which, fn in (("k", agg.agg_kc_offset), ("v", agg.agg_vc_offset)):
        flat = torch.zeros(2 * 4096, dtype=torch.float32)
        for m in range(M_pad):
            for d in range(64):
                flat[fn(m, d)] = m * 64 + d
        dec = harness.decode_compact(flat, 1, 1, M_pad, M_pad, which)
        assert torch.equal(dec.reshape(-1), torch.arange(M_pad * 64, dtype=torch.float32))


def test_product_and_oracle_share_nothing():
    """The library, its binding and the benchmark's product path never reach into oracle/, and
    the oracle never reaches into the package (only the input generators serve both)."""
    pkg = os.path.join(ROOT, "paper_2512_02541_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for name in files:
            if not name.endswith((".py", ".cpp", ".hip", ".h")):
                continue
            text = open(os.path.join(dirpath, name)).read()
            assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), name
            assert "sga_oracle" not in text and "block_oracle" not in text and \
                "list_oracle" not in text, name
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", name)).read()
            assert "paper_2512_02541_amd" not in text and "agg.h" not in text and \
                "agg_internal" not in text, name
    # bench.py touches the oracle only inside its CPU-baseline leg
    bench = open(os.path.join(ROOT, "bench.py")).read()
    for m in re.finditer(r"^\s*(from|import)\s+oracle\b.*$", bench, flags=re.M):
        last_def = re.findall(r"^def (\w+)\(", bench[:m.start()], flags=re.M)[-1]
        assert last_def == "cpu_baseline", (m.group(0), last_def)


def test_attention_kernel_leaves_m0_to_its_copy_statements(tmp_path):
    """The attention kernel's global->LDS copies set the M0 register inside assembly statements
    without declaring it (the compiler rejects M0 as a clobber).  That is sound only while no
    compiler-emitted instruction of those kernels uses M0: compile the file to assembly and
    look at every instruction outside the statements."""
    import subprocess

    from paper_2512_02541_amd import build as b

    out = tmp_path / "agg_attn.s"
    cmd = [b.HIPCC, *b.FLAGS, "-I", os.path.join(ROOT, "include"), "-I", b.CSRC, "-S",
           "--cuda-device-only", os.path.join(b.CSRC, "agg_attn.hip"), "-o", str(out)]
    subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
    inside, seen_copy, offenders = False, 0, []
    for line in out.read_text().splitlines():
        text = line.split(";")[0] if not line.lstrip().startswith(";;#") else line
        if "#ASMSTART" in line:
            inside = True
        elif "#ASMEND" in line:
            inside = False
        elif inside:
            seen_copy += "global_load_lds_dwordx4" in text
        elif re.search(r"\bm0\b", text):
            offenders.append(line.strip())
    assert seen_copy >= 4, "the copy statements were not found"
    assert not offenders, offenders[:5]
