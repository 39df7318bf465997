"""The C-ABI library loads, exports every declared symbol and rejects bad
arguments on the host without touching a device (no compute calls here)."""

import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _fa():
    import paper_2506_11886_amd as fa
    return fa


def test_library_exports_every_declared_symbol():
    fa = _fa()
    hdr = open(os.path.join(ROOT, "include", "fourier_attn.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(fa_[a-z_0-9]+)\s*\(", hdr))
    assert {"fa_compress", "fa_decode", "fa_compress_workspace_bytes",
            "fa_decode_workspace_bytes", "fa_decode_default_splits", "fa_status_string",
            "fa_append", "fa_select_dims", "fa_select_workspace_bytes", "fa_decode_mq", "fa_compress_kv", "fa_decode_varlen", "fa_append_varlen",
            "fa_compress_kv_workspace_bytes", "fa_decode_static", "fa_compress_workspace_bytes_for",
            "fa_compress_kv_workspace_bytes_for", "fa_legt_compress", "fa_legt_mse",
            "fa_legt_workspace_bytes"} <= names
    for n in names:
        assert hasattr(fa.lib, n), n


def test_status_strings():
    fa = _fa()
    assert fa.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5, -99):
        assert fa.status_string(code)


FAKE = ctypes.c_void_p(0x10000)   # never dereferenced: validation fails first


def _decode(fa, **kw):
    a = dict(q=FAKE, dtype=1, B=1, Hq=8, Hkv=2, D=128, ck=FAKE, kmask=FAKE, Dkc=96, cv=FAKE,
             vmask=FAKE, Dvc=96, M=32, T=512, t0=0, N=512, k_keep=FAKE, kks=0, v_keep=FAKE, vks=0,
             k_full=FAKE, v_full=FAKE, W=16, fs=0, scale=0.0, splits=0, out=FAKE, ws=FAKE,
             ws_bytes=0, stream=None)
    a.update(kw)
    return fa.lib.fa_decode(a["q"], a["dtype"], a["B"], a["Hq"], a["Hkv"], a["D"], a["ck"], a["kmask"],
                            a["Dkc"], a["cv"], a["vmask"], a["Dvc"], a["M"], a["T"], a["t0"], a["N"],
                            a["k_keep"], a["kks"], a["v_keep"], a["vks"], a["k_full"], a["v_full"],
                            a["W"], a["fs"], a["scale"], a["splits"], a["out"], a["ws"], a["ws_bytes"],
                            a["stream"])


@pytest.mark.parametrize("kw,code", [
    (dict(Hq=7), -2), (dict(Dkc=129), -2), (dict(M=0), -2), (dict(M=600), -2),
    (dict(t0=1), -2), (dict(N=0, W=0), -2), (dict(D=100), -3), (dict(Hq=64, Hkv=2), -3),
    (dict(dtype=7), -3), (dict(q=None), -1), (dict(ck=None), -1), (dict(k_full=None), -1),
    (dict(out=None), -1), (dict(ws_bytes=16), -4), (dict(kks=5), -2), (dict(splits=-1), -2),
])
def test_decode_rejects_bad_arguments(kw, code):
    assert _decode(_fa(), **kw) == code


def _compress(fa, **kw):
    a = dict(x=FAKE, dtype=1, sb=8 * 512 * 128, sh=512 * 128, sn=128, B=1, H=8, N=512, D=128,
             mask=FAKE, Dc=96, M=32, T=512, t0=0, acc=0, coeffs=FAKE, keep=FAKE, layout=0, ks=0,
             koff=0, ws=FAKE, ws_bytes=0, stream=None)
    a.update(kw)
    return fa.lib.fa_compress(a["x"], a["dtype"], a["sb"], a["sh"], a["sn"], a["B"], a["H"], a["N"],
                              a["D"], a["mask"], a["Dc"], a["M"], a["T"], a["t0"], a["acc"], a["coeffs"],
                              a["keep"], a["layout"], a["ks"], a["koff"], a["ws"], a["ws_bytes"],
                              a["stream"])


@pytest.mark.parametrize("kw,code", [
    (dict(Dc=200), -2), (dict(M=513), -2), (dict(t0=4), -2), (dict(sn=100), -2), (dict(sn=132), -2),
    (dict(layout=3), -2), (dict(koff=-1), -2), (dict(D=100, Dc=50), -3), (dict(M=2000, T=4000), -3),
    (dict(x=None), -1), (dict(mask=None), -1), (dict(coeffs=None), -1),
    (dict(N=8192, T=8192, sb=8 * 8192 * 128, sh=8192 * 128, ws_bytes=8), -4),
    (dict(x=ctypes.c_void_p(0x10004)), -2),
])
def test_compress_rejects_bad_arguments(kw, code):
    assert _compress(_fa(), **kw) == code


def test_workspace_queries():
    fa = _fa()
    assert fa.decode_workspace_bytes(1, 32, 8, 128, 96, 96, 256, 31740, 1028, 0) > 0
    assert fa.decode_workspace_bytes(1, 7, 2, 128, 96, 96, 256, 100, 10, 0) == 0
    assert fa.compress_workspace_bytes(8, 32, 4096, 128, 96, 256) >= 256
    assert fa.decode_default_splits(1, 32, 8, 256, 31740, 1028) >= 1
    # the element-type-aware query: never more than the one that covers both, far less for long bf16 segments
    both = fa.compress_workspace_bytes(1, 8, 129020, 128, 112, 512)
    bf16 = fa.compress_workspace_bytes(1, 8, 129020, 128, 112, 512, fa.FA_BF16)
    f32 = fa.compress_workspace_bytes(1, 8, 129020, 128, 112, 512, fa.FA_F32)
    assert 0 < bf16 <= f32 == both and bf16 * 4 < both
    assert fa.compress_kv_workspace_bytes(1, 8, 129020, 128, 112, 112, 512, fa.FA_BF16) < \
        fa.compress_kv_workspace_bytes(1, 8, 129020, 128, 112, 112, 512)
    assert fa.lib.fa_compress_workspace_bytes_for(7, 1, 8, 1000, 128, 96, 64) == 0


def test_append_rejects_bad_arguments_on_the_host():
    fa = _fa()
    a = dict(k_new=FAKE, v_new=FAKE, dtype=1, B=1, Hkv=2, D=64, k_full=FAKE, v_full=FAKE, W=8, fs=0, slot=3,
             evict=1, kmask=FAKE, Dkc=48, vmask=FAKE, Dvc=48, M=16, T=100, n_mid=5, ck=FAKE, cv=FAKE,
             k_keep=FAKE, kks=0, v_keep=FAKE, vks=0, stream=None)

    def call(**kw):
        d = dict(a, **kw)
        return fa.lib.fa_append(d["k_new"], d["v_new"], d["dtype"], d["B"], d["Hkv"], d["D"], d["k_full"],
                                d["v_full"], d["W"], d["fs"], d["slot"], d["evict"], d["kmask"], d["Dkc"],
                                d["vmask"], d["Dvc"], d["M"], d["T"], d["n_mid"], d["ck"], d["cv"], d["k_keep"],
                                d["kks"], d["v_keep"], d["vks"], d["stream"])
    assert call(slot=8) == -2            # slot outside the rows
    assert call(k_new=None) == -1
    assert call(D=60) == -3              # head dim not a multiple of 8
    assert call(n_mid=100) == -2         # position outside the period
    assert call(ck=None) == -1
    assert call(dtype=7) == -3
    assert call(kks=5) == -2             # slab too small for n_mid + 1 rows


def test_select_rejects_bad_arguments_on_the_host():
    fa = _fa()
    a = dict(x=FAKE, dtype=1, sb=8 * 300 * 64, sh=300 * 64, sn=64, B=1, H=8, N=300, D=64, M=32, Dc=48,
             mask=FAKE, mse=None, ws=FAKE, ws_bytes=0, stream=None)

    def call(**kw):
        d = dict(a, **kw)
        return fa.lib.fa_select_dims(d["x"], d["dtype"], d["sb"], d["sh"], d["sn"], d["B"], d["H"], d["N"],
                                     d["D"], d["M"], d["Dc"], d["mask"], d["mse"], d["ws"], d["ws_bytes"],
                                     d["stream"])
    assert call(M=301) == -2             # more basis functions than positions in the period
    assert call(Dc=65) == -2
    assert call(D=60, sn=60) == -3
    assert call(dtype=3) == -3
    assert call(x=None) == -1
    assert call(mask=None) == -1
    assert call(sn=60) == -2             # rows overlap
    assert call() == -4                  # workspace too small
    assert fa.select_workspace_bytes(1, 1, 8, 300, 64, 32) > 4 * 8 * 300 * 64
    assert fa.select_workspace_bytes(0, 1, 8, 300, 64, 32) < fa.select_workspace_bytes(1, 1, 8, 300, 64, 32)


def test_decode_mq_rejects_bad_arguments_on_the_host():
    fa = _fa()

    def call(Tq, Hq=8, Hkv=2, W=16):
        return fa.lib.fa_decode_mq(FAKE, 1, 1, Tq, Hq, Hkv, 128, FAKE, FAKE, 96, FAKE, FAKE, 96, 32, 512, 0, 512,
                                   FAKE, 0, FAKE, 0, FAKE, FAKE, W, 0, 0.0, 0, FAKE, FAKE, 0, None)
    assert call(0) == -2                 # no query token
    assert call(3, W=2) == -2            # more new tokens than full-width rows
    assert call(5) == -3                 # 5 tokens x 4 heads per KV head exceed the group limit
    assert call(4) == -4                 # legal, but the workspace is too small


def test_compress_kv_rejects_bad_arguments_on_the_host():
    fa = _fa()

    def call(**kw):
        d = dict(k=FAKE, v=FAKE, dtype=1, sn=128, N=2048, D=128, Dkc=96, Dvc=96, M=64, ws=FAKE, ws_bytes=1 << 30)
        d.update(kw)
        return fa.lib.fa_compress_kv(d["k"], d["v"], d["dtype"], 8 * d["N"] * d["sn"], d["N"] * d["sn"], d["sn"], 1, 8, d["N"],
                                     d["D"], FAKE, d["Dkc"], FAKE, d["Dvc"], d["M"], d["N"], 0, 0, FAKE, FAKE, FAKE, 0, FAKE, 0, 0,
                                     d["ws"], d["ws_bytes"], None)
    assert call(M=0) == -2
    assert call(Dvc=129) == -2
    assert call(D=100, sn=100) in (-2, -3)
    assert call(ws=None) == -1
    assert call(ws_bytes=16) == -4
    assert call(k=None) == -1
    assert fa.compress_kv_workspace_bytes(1, 8, 31740, 128, 96, 96, 256) >= 2 * fa.compress_workspace_bytes(1, 8, 31740, 128, 96, 256)


def test_static_scratch_refuses_sizes_beyond_the_array():
    from workloads import CONFIGS
    fa = _fa()
    fake = FAKE                          # never dereferenced: the size check comes first
    # 64 sequences x 32 query heads x 256 chunks of middle rows: far more records than 8 MiB hold
    need = fa.decode_workspace_bytes(64, 32, 8, 128, 96, 96, 256, 1 << 20, 1028, 256)
    assert need > fa.FA_STATIC_SCRATCH_BYTES
    st = fa.lib.fa_decode_static(fake, 1, 64, 32, 8, 128, fake, fake, 96, fake, fake, 96, 256, 1 << 20, 0, 1 << 20,
                                 fake, 0, fake, 0, fake, fake, 1028, 0, 0.0, 256, fake, None)
    assert st == fa.FA_ERR_SCRATCH
    assert "scratch" in fa.status_string(st)
    # the benchmark configurations fit
    for c in CONFIGS:
        assert 0 < fa.decode_workspace_bytes(c.B, c.Hq, c.Hkv, c.D, c.Dkc, c.Dvc, c.M, c.N, c.W, c.num_splits) \
            <= fa.FA_STATIC_SCRATCH_BYTES


def test_legt_rejects_bad_arguments_on_the_host():
    fa = _fa()

    def call(**kw):
        d = dict(x=FAKE, dtype=1, sn=64, N=300, D=64, M=32, coeffs=FAKE, ws=FAKE, ws_bytes=1 << 30)
        d.update(kw)
        return fa.lib.fa_legt_compress(d["x"], d["dtype"], 8 * d["N"] * d["sn"], d["N"] * d["sn"], d["sn"], 1, 8, d["N"],
                                       d["D"], d["M"], d["coeffs"], d["ws"], d["ws_bytes"], None)
    assert call(M=301) == -2             # more states than tokens
    assert call(D=60, sn=60) == -3
    assert call(dtype=5) == -3
    assert call(x=None) == -1
    assert call(coeffs=None) == -1
    assert call(sn=32) == -2             # rows overlap
    assert call(ws_bytes=16) == -4
    assert fa.lib.fa_legt_mse(FAKE, 1, 8 * 300 * 64, 300 * 64, 64, 1, 8, 300, 64, 32, FAKE, None, FAKE, 1 << 30, None) == -1
    assert fa.legt_workspace_bytes(1, 8, 300, 64, 32) >= 1 * 8 * 32 * 64 * 4


def test_varlen_entry_points_reject_bad_arguments_on_the_host():
    """fa_decode_varlen validates like fa_decode (N_max, W_max in the place of N, W); fa_append_varlen
    needs both lists and a capacity inside the period."""
    fa = _fa()

    def decode_vl(**kw):
        a = dict(q=FAKE, dtype=1, B=2, Hq=8, Hkv=2, D=128, ck=FAKE, kmask=FAKE, Dkc=96, cv=FAKE, vmask=FAKE,
                 Dvc=96, M=32, T=512, t0=0, N=512, seq_n=FAKE, k_keep=FAKE, kks=0, v_keep=FAKE, vks=0,
                 k_full=FAKE, v_full=FAKE, W=16, seq_w=FAKE, fs=0, scale=0.0, splits=0, out=FAKE, ws=FAKE,
                 ws_bytes=0, stream=None)
        a.update(kw)
        return fa.lib.fa_decode_varlen(a["q"], a["dtype"], a["B"], a["Hq"], a["Hkv"], a["D"], a["ck"], a["kmask"],
                                       a["Dkc"], a["cv"], a["vmask"], a["Dvc"], a["M"], a["T"], a["t0"], a["N"],
                                       a["seq_n"], a["k_keep"], a["kks"], a["v_keep"], a["vks"], a["k_full"],
                                       a["v_full"], a["W"], a["seq_w"], a["fs"], a["scale"], a["splits"], a["out"],
                                       a["ws"], a["ws_bytes"], a["stream"])
    assert decode_vl(Hq=7) == -2 and decode_vl(N=0, W=0) == -2 and decode_vl(q=None) == -1
    assert decode_vl(ws_bytes=16) == -4 and decode_vl(seq_n=None, seq_w=None, ws_bytes=16) == -4

    def append_vl(**kw):
        a = dict(k_new=FAKE, v_new=FAKE, dtype=1, B=2, Hkv=2, D=64, k_full=FAKE, v_full=FAKE, W=8, fs=0,
                 seq_slot=FAKE, kmask=FAKE, Dkc=48, vmask=FAKE, Dvc=48, M=16, T=100, seq_nmid=FAKE, n_cap=50,
                 ck=FAKE, cv=FAKE, k_keep=FAKE, kks=0, v_keep=FAKE, vks=0, stream=None)
        a.update(kw)
        return fa.lib.fa_append_varlen(a["k_new"], a["v_new"], a["dtype"], a["B"], a["Hkv"], a["D"], a["k_full"],
                                       a["v_full"], a["W"], a["fs"], a["seq_slot"], a["kmask"], a["Dkc"], a["vmask"],
                                       a["Dvc"], a["M"], a["T"], a["seq_nmid"], a["n_cap"], a["ck"], a["cv"],
                                       a["k_keep"], a["kks"], a["v_keep"], a["vks"], a["stream"])
    assert append_vl(seq_slot=None) == -1 and append_vl(seq_nmid=None) == -1
    assert append_vl(n_cap=0) == -2 and append_vl(n_cap=101) == -2
    assert append_vl(kks=8) == -2            # a slab pitch below n_cap tokens
    assert append_vl(M=0) == -2 and append_vl(D=60) == -3 and append_vl(kmask=None) == -1
