"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, evaluates its closed forms, and rejects bad arguments
before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2605_16439_amd import kvcapsule as kv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def header_functions():
    txt = ""
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if name.endswith(".h"):
            txt += open(os.path.join(ROOT, "include", name)).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(kvc_[a-z_0-9]+)\s*\(", txt)))


def test_library_loads_and_exports_every_declared_symbol():
    L = kv.lib()
    names = header_functions()
    assert "kvc_compress" in names and "kvc_reconstruct_attend_decode" in names
    for name in names:
        assert hasattr(L, name), name
    assert sorted(kv.EXPORTS) == names
    assert re.match(r"^\d+\.\d+$", kv.version())


def test_compressed_len_matches_paper_formula():
    with open(os.path.join(GOLDEN, "compressed_len.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                n, c, m = line.split()
                assert kv.kvc_compressed_len(int(n), float(c)) == int(m), line
    assert kv.kvc_compressed_len(0, 0.5) == 0


def test_memory_footprint_closed_form():
    # App. C eqs. 1-2 by hand: B=1, H_kv=4, one image n=1024 -> m=410, d=128, bf16
    s = kv.make_shape(1, 28, 4, 128, 1024, 1, 410, kv.KVC_BF16)
    full, caps = kv.kvc_memory_footprint(s, 0, 0)
    assert full == 2097152 and caps == 839680 + 3358720 + 3358720 + 1024
    s8 = kv.make_shape(4, 28, 4, 128, 1024, 8, 410, kv.KVC_BF16)
    full, caps = kv.kvc_memory_footprint(s8, 0, 512)
    assert full == 2 * 4 * 4 * (8192 + 512) * 128 * 2
    assert caps == 2 * 4 * 4 * (8 * 410 + 512) * 128 * 2 + 2 * 3358720 + 1024


def _valid():
    s = kv.make_shape(2, 8, 2, 64, 48, 2, 20, kv.KVC_F32)
    p = kv.KvcParams(0x1000, 0x2000, 0x3000, 0x4000)
    return s, p


def _decode(s, p, q=0x10000, Kc=0x20000, Vc=0x30000, Kt=0x40000, Vt=0x50000, t=4, cap=8,
            kn=None, vn=None, scale=0.0, out=0x60000, lse=None, ws=0x70000, wsb=1 << 30):
    return kv.lib().kvc_reconstruct_attend_decode(
        ctypes.byref(s) if s is not None else None, ctypes.byref(p) if p is not None else None,
        q, Kc, Vc, Kt, Vt, t, cap, kn, vn, ctypes.c_float(scale), out, lse, ws, wsb, None)


def test_decode_rejects_bad_arguments_before_any_launch():
    """Fake (never dereferenced) device addresses: every call below must fail validation."""
    s, p = _valid()
    assert _decode(None, p) == kv.KVC_ERR_NULL
    assert _decode(s, None) == kv.KVC_ERR_NULL
    assert _decode(s, p, q=None) == kv.KVC_ERR_NULL
    assert _decode(s, p, out=None) == kv.KVC_ERR_NULL
    assert _decode(s, p, Kc=None) == kv.KVC_ERR_NULL
    assert _decode(s, p, Kt=None) == kv.KVC_ERR_NULL
    assert _decode(s, p, kn=0x80000) == kv.KVC_ERR_NULL          # k_new without v_new
    assert _decode(s, p, t=9) == kv.KVC_ERR_SHAPE                  # text_len > text_cap
    assert _decode(s, p, t=8, kn=0x80000, vn=0x90000) == kv.KVC_ERR_SHAPE   # append beyond cap
    assert _decode(s, p, t=-1) == kv.KVC_ERR_SHAPE
    assert _decode(s, p, q=0x10004) == kv.KVC_ERR_ALIGN
    assert _decode(s, p, ws=None) == kv.KVC_ERR_WORKSPACE
    assert _decode(s, p, wsb=16) == kv.KVC_ERR_WORKSPACE
    assert _decode(s, p, scale=-1.0) == kv.KVC_ERR_SHAPE
    bad = kv.make_shape(2, 8, 3, 64, 48, 2, 20, kv.KVC_F32)       # H_q % H_kv != 0
    assert _decode(bad, p) == kv.KVC_ERR_SHAPE
    bad = kv.make_shape(2, 8, 2, 64, 48, 2, 49, kv.KVC_F32)       # m > n
    assert _decode(bad, p) == kv.KVC_ERR_SHAPE
    bad = kv.make_shape(2, 8, 2, 64, 48, 2, 0, kv.KVC_F32)        # m < 1
    assert _decode(bad, p) == kv.KVC_ERR_SHAPE
    bad = kv.make_shape(2, 8, 2, 60, 48, 2, 20, kv.KVC_F32)       # d % 8
    assert _decode(bad, p) == kv.KVC_ERR_SHAPE
    bad = kv.make_shape(2, 8, 2, 512, 48, 2, 20, kv.KVC_F32)
    assert _decode(bad, p) == kv.KVC_ERR_UNSUPPORTED
    bad = kv.make_shape(2, 8, 2, 64, 48, 2, 20, 7)
    assert _decode(bad, p) == kv.KVC_ERR_DTYPE
    empty = kv.make_shape(2, 8, 2, 64, 48, 0, 20, kv.KVC_F32)     # no vision and no text row
    assert _decode(empty, p, t=0, cap=0, Kt=None, Vt=None) == kv.KVC_ERR_SHAPE


def test_compress_rejects_bad_arguments_before_any_launch():
    s, p = _valid()

    def comp(s=s, p=p, K=0x10000, V=0x20000, sb=2 * 100 * 64, sh=100 * 64, ss=64, vis=2,
             Kc=0x30000, Vc=0x40000, S=100):
        return kv.lib().kvc_compress(ctypes.byref(s) if s is not None else None,
                                     ctypes.byref(p) if p is not None else None, K, V, sb, sh, ss,
                                     vis, S, Kc, Vc, None, 0, None)
    assert comp(s=None) == kv.KVC_ERR_NULL
    assert comp(K=None) == kv.KVC_ERR_NULL
    assert comp(Vc=None) == kv.KVC_ERR_NULL
    assert comp(p=kv.KvcParams(None, 0x2000, 0x3000, 0x4000)) == kv.KVC_ERR_NULL   # no mask
    assert comp(vis=-1) == kv.KVC_ERR_SHAPE
    assert comp(vis=5) == kv.KVC_ERR_SHAPE            # 5 + 2 * 48 rows do not fit a sequence of 100
    assert comp(S=97) == kv.KVC_ERR_SHAPE
    assert comp(ss=32) == kv.KVC_ERR_SHAPE            # rows overlap
    assert comp(ss=68) == kv.KVC_ERR_ALIGN
    assert comp(K=0x10002) == kv.KVC_ERR_ALIGN


def test_workspace_size_and_status_strings():
    s, _ = _valid()
    a = kv.kvc_workspace_bytes(s, 8)
    b = kv.kvc_workspace_bytes(s, 800)
    assert 0 < a < b
    assert kv.kvc_workspace_bytes(kv.make_shape(0, 8, 2, 64, 48, 2, 20, kv.KVC_F32), 8) == 0
    seen = {kv.status_string(c) for c in range(-7, 1)}
    assert len(seen) == 8 and kv.status_string(kv.KVC_OK) == "ok"
    assert kv.status_string(-99) == "unknown status"


def test_probe_read_rejects_bad_arguments_before_touching_the_device():
    L = kv.lib()
    fake = ctypes.c_void_p(0x10000)
    assert L.kvc_probe_read(None, 1024, fake, None) == kv.KVC_ERR_NULL
    assert L.kvc_probe_read(fake, 1024, None, None) == kv.KVC_ERR_NULL
    assert L.kvc_probe_read(ctypes.c_void_p(0x10008), 1024, fake, None) == kv.KVC_ERR_ALIGN
    assert L.kvc_probe_read(fake, 1000, fake, None) == kv.KVC_ERR_ALIGN
    assert L.kvc_probe_read(fake, 0, fake, None) == kv.KVC_OK


def test_capsule_value_offset_is_the_documented_blocked_layout():
    """Rows in blocks of 8, a block channel-major [d][w] with w = 8 (m % 8 for a shorter last block): the
    offsets of all (j, c) are a permutation of 0 .. m*d - 1 and 8 consecutive rows of a channel are contiguous."""
    L = kv.lib()
    for m, d in ((1, 8), (8, 16), (13, 8), (410, 128)):
        offs = [L.kvc_capsule_value_offset(j, c, m, d) for j in range(m) for c in range(d)]
        assert sorted(offs) == list(range(m * d))
        for j in range(0, m - 1):
            if j % 8 != 7:
                assert L.kvc_capsule_value_offset(j + 1, 3, m, d) == L.kvc_capsule_value_offset(j, 3, m, d) + 1
        w = min(8, m)
        assert L.kvc_capsule_value_offset(0, 1, m, d) == w
    assert L.kvc_capsule_value_offset(5, 0, 5, 8) == -1 and L.kvc_capsule_value_offset(0, 8, 5, 8) == -1
    fake = ctypes.c_void_p(0x10000)
    assert L.kvc_unpack_values(None, fake, 1, 8, 8, kv.KVC_BF16, None) == kv.KVC_ERR_NULL
    assert L.kvc_unpack_values(fake, fake, 1, 0, 8, kv.KVC_BF16, None) == kv.KVC_ERR_SHAPE
    assert L.kvc_unpack_values(fake, fake, 1, 8, 8, 9, None) == kv.KVC_ERR_DTYPE


def test_pack_theta_rejects_bad_arguments_before_any_launch():
    s, p = _valid()
    L = kv.lib()
    fake, fake2 = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x20000)
    assert L.kvc_pack_theta(None, fake, fake2, None) == kv.KVC_ERR_NULL
    assert L.kvc_pack_theta(ctypes.byref(s), None, fake2, None) == kv.KVC_ERR_NULL
    assert L.kvc_pack_theta(ctypes.byref(s), fake, None, None) == kv.KVC_ERR_NULL
    assert L.kvc_pack_theta(ctypes.byref(s), fake, fake, None) == kv.KVC_ERR_SHAPE          # in place
    assert L.kvc_pack_theta(ctypes.byref(s), ctypes.c_void_p(0x10008), fake2, None) == kv.KVC_ERR_ALIGN
    # a misaligned packed theta in the parameters of a decode call is refused like any other pointer
    bad = kv.KvcParams(p.key_idx, p.theta, p.U, p.mu, 0x50004)
    assert _decode(s, bad) == kv.KVC_ERR_ALIGN


def test_packed_theta_layout_is_the_value_layout_with_positions_for_channels():
    """Element (row j, position pos) of a record of m x n elements, rows in blocks of 8, each block [n][w]."""
    m, n = 19, 24
    seen = set()
    for j in range(m):
        for pos in range(n):
            w = min(8, m - 8 * (j // 8))
            off = kv.lib().kvc_capsule_value_offset(j, pos, m, n)
            assert off == (j // 8) * 8 * n + pos * w + j % 8
            seen.add(off)
    assert seen == set(range(m * n))          # a permutation of the record: same size as theta


def test_pack_u_rejects_bad_arguments_before_any_launch():
    s, p = _valid()
    L = kv.lib()
    fake, fake2 = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x20000)
    assert L.kvc_pack_u(None, fake, fake2, None) == kv.KVC_ERR_NULL
    assert L.kvc_pack_u(ctypes.byref(s), None, fake2, None) == kv.KVC_ERR_NULL
    assert L.kvc_pack_u(ctypes.byref(s), fake, fake, None) == kv.KVC_ERR_SHAPE              # in place
    assert L.kvc_pack_u(ctypes.byref(s), fake, ctypes.c_void_p(0x20008), None) == kv.KVC_ERR_ALIGN
    odd = kv.make_shape(2, 8, 2, 64, 50, 2, 20, kv.KVC_F32)                                 # n not a multiple of 8
    assert L.kvc_pack_u(ctypes.byref(odd), fake, fake2, None) == kv.KVC_ERR_UNSUPPORTED
    bad = kv.KvcParams(p.key_idx, p.theta, p.U, p.mu, None, 0x50004)
    assert _decode(s, bad) == kv.KVC_ERR_ALIGN
