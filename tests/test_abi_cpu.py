"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, sizes its workspace sanely and rejects bad arguments before
touching the device (so these calls are safe without a GPU)."""
import ctypes as C
import os
import re

import pytest

from paper_2603_09582_amd import binding as ba

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # non-null, 16- and 256-byte aligned; never dereferenced on a failing call


def declared_functions():
    text = open(os.path.join(ROOT, "include", "binattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(binattn_\w+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = ba.lib()
    names = declared_functions()
    assert set(names) == set(ba.EXPORTS)
    for n in names:
        assert hasattr(L, n), n
    assert L.binattn_version() >= 100
    assert L.binattn_strerror(0) == b"ok"
    for code in range(-11, 0):
        assert len(L.binattn_strerror(code)) > 3


def test_workspace_bytes():
    assert ba.workspace_bytes(1, 3, 197, 64) > 2 * 3 * 197 * 64
    assert ba.workspace_bytes(1, 1, 1, 8) > 0
    assert ba.workspace_bytes(2, 16, 16384, 64) < 200 * 2 ** 20
    for bad in [(0, 1, 1, 64), (1, 0, 1, 64), (1, 1, 0, 64), (1, 1, 5, 0), (1, 1, 5, 4),
                (1, 1, 5, 12), (1, 1, 5, 136), (1, 1, 2 ** 24 + 1, 64), (2 ** 16, 2 ** 10, 8, 64)]:
        assert ba.workspace_bytes(*bad) == 0, bad
    # monotone in every argument
    assert ba.workspace_bytes(2, 3, 197, 64) > ba.workspace_bytes(1, 3, 197, 64)
    assert ba.workspace_bytes(1, 3, 300, 64) > ba.workspace_bytes(1, 3, 197, 64)
    assert ba.workspace_bytes(1, 3, 197, 72) > ba.workspace_bytes(1, 3, 197, 64)


def st(*v):
    return (C.c_int64 * 3)(*v)


def pack(q=FAKE, k=FAKE, B=1, H=2, N=16, d=64, qs=None, ks=None, qb=FAKE, kb=FAKE, mq=FAKE, mk=FAKE):
    qs = qs or st(H * N * d, N * d, d)
    ks = ks or st(H * N * d, N * d, d)
    return ba.lib().binattn_pack_qk(q, k, B, H, N, d, qs, ks, qb, kb, mq, mk, None)


def test_pack_qk_rejects_bad_arguments():
    assert pack(q=None) == -1 and pack(kb=None) == -1 and pack(mk=None) == -1
    assert pack(N=0) == -2 and pack(d=12) == -2 and pack(d=256) == -2 and pack(B=-1) == -2
    assert pack(qs=st(2048, 1024, 60)) == -3      # row stride smaller than d
    assert pack(qs=st(2048, 1028, 64)) == -3      # not a multiple of 8
    assert pack(ks=st(-8, 1024, 64)) == -3
    assert pack(q=FAKE + 8) == -4 and pack(mq=FAKE + 2) == -4


def fwd(qb=FAKE, kb=FAKE, mq=FAKE, mk=FAKE, v=FAKE, vs=None, bias=FAKE, bdt=1, bs=None, B=1, H=2,
        N=16, d=64, out=FAKE, os_=None, ws=FAKE, wsb=None, flags=0):
    vs = vs or st(H * N * d, N * d, d)
    os_ = os_ or st(H * N * d, N * d, d)
    bs = bs or st(0, N * N, N)
    if wsb is None:
        wsb = max(ba.workspace_bytes(B, H, N, d), 1)
    return ba.lib().binattn_forward(qb, kb, mq, mk, v, vs, bias, bdt, bs, 0.125, B, H, N, d, out,
                                    os_, ws, wsb, flags, None)


def test_forward_rejects_bad_arguments():
    assert fwd(qb=None) == -1 and fwd(v=None) == -1 and fwd(out=None) == -1
    assert fwd(d=20) == -2 and fwd(N=0) == -2
    assert fwd(vs=st(2048, 1024, 32)) == -3 and fwd(os_=st(2048, 1024, 68)) == -3
    assert fwd(bs=st(0, 256, 8)) == -3             # bias rows overlap
    assert fwd(bs=st(0, -1, 16)) == -3
    assert fwd(v=FAKE + 4) == -4 and fwd(out=FAKE + 2) == -4 and fwd(bias=FAKE + 1) == -4
    assert fwd(bdt=7) == -6
    assert fwd(ws=None) == -5 and fwd(ws=FAKE + 64) == -5 and fwd(wsb=100) == -5
    # a NULL bias or the NO_BIAS flag makes dtype and strides irrelevant: next check is the workspace
    assert fwd(bias=None, bdt=7, wsb=100) == -5
    assert fwd(bdt=7, flags=ba.FLAG_NO_BIAS, wsb=100) == -5


def fwd_axial(by=FAKE, bx=FAKE, Gy=16, Gx=16, N=256, d=64, qb=FAKE, v=FAKE, out=FAKE, ws=FAKE, wsb=1 << 30,
              flags=0):
    B, H = 1, 2
    s3 = st(H * N * d, N * d, d)
    return ba.lib().binattn_forward_axial(qb, FAKE, FAKE, FAKE, v, s3, by, bx, Gy, Gx, 0.125, B, H, N, d,
                                          out, s3, ws, wsb, flags, None)


def test_forward_axial_rejects_bad_arguments():
    assert fwd_axial(by=None) == -1 and fwd_axial(bx=None) == -1 and fwd_axial(qb=None) == -1
    assert fwd_axial(Gx=24, Gy=16, N=384) == -2      # Gx not a power of two
    assert fwd_axial(Gx=8, Gy=32) == -2              # Gx below 16
    assert fwd_axial(Gx=512, Gy=2, N=1024) == -2     # Gx above 256
    assert fwd_axial(Gx=16, Gy=15) == -2             # Gy * Gx != N
    assert fwd_axial(Gx=16, Gy=257, N=16 * 257) == -2
    assert fwd_axial(by=FAKE + 2) == -4 and fwd_axial(bx=FAKE + 1) == -4
    assert fwd_axial(wsb=100) == -5
    L = ba.lib()
    s3 = st(2 * 256 * 64, 256 * 64, 64)
    assert L.binattn_attend_axial(FAKE, FAKE, FAKE, FAKE, FAKE, 16, 16, 0.125, 1, 2, 256, 64, FAKE, s3, FAKE,
                                  100, 0, None) == -5
    assert L.binattn_attend_axial(FAKE, FAKE, FAKE, None, FAKE, 16, 16, 0.125, 1, 2, 256, 64, FAKE, s3, FAKE,
                                  1 << 30, 0, None) == -1


def fwd_relpos(table=FAKE, Gy=16, Gx=16, N=256, d=64, qb=FAKE, v=FAKE, out=FAKE, ws=FAKE, wsb=1 << 30, flags=0):
    B, H = 1, 2
    s3 = st(H * N * d, N * d, d)
    return ba.lib().binattn_forward_relpos(qb, FAKE, FAKE, FAKE, v, s3, table, Gy, Gx, 0.125, B, H, N, d, out,
                                           s3, ws, wsb, flags, None)


def test_forward_relpos_rejects_bad_arguments():
    assert fwd_relpos(table=None) == -1 and fwd_relpos(qb=None) == -1 and fwd_relpos(v=None) == -1
    assert fwd_relpos(Gx=24, Gy=16, N=384) == -2     # Gx not a power of two
    assert fwd_relpos(Gx=8, Gy=32) == -2             # Gx below 16
    assert fwd_relpos(Gx=512, Gy=2, N=1024) == -2    # Gx above 256
    assert fwd_relpos(Gx=16, Gy=257, N=16 * 257) == -2 # Gy above 256
    assert fwd_relpos(Gx=16, Gy=15) == -2            # Gy * Gx != N
    assert fwd_relpos(table=FAKE + 2) == -4
    assert fwd_relpos(wsb=100) == -5
    L = ba.lib()
    s3 = st(2 * 256 * 64, 256 * 64, 64)
    assert L.binattn_attend_relpos(FAKE, FAKE, FAKE, FAKE, 16, 16, 0.125, 1, 2, 256, 64, FAKE, s3, FAKE, 100, 0,
                                   None) == -5
    assert L.binattn_attend_relpos(FAKE, FAKE, FAKE, None, 16, 16, 0.125, 1, 2, 256, 64, FAKE, s3, FAKE, 1 << 30,
                                   0, None) == -1


def fused(q=FAKE, k=FAKE, v=FAKE, out=FAKE, N=200, d=64, bias=FAKE, bdt=1, bs=None, qs=None, mq=FAKE, flags=0):
    B, H = 2, 2
    s3 = st(H * N * d, N * d, d)
    return ba.lib().binattn_forward_fused(q, k, v, qs or s3, s3, s3, bias, bdt, bs or st(0, N * N, N), 0.125, B, H,
                                          N, d, out, s3, mq, None, flags, None)


def test_forward_fused_rejects_bad_arguments():
    assert fused(q=None) == -1 and fused(k=None) == -1 and fused(v=None) == -1 and fused(out=None) == -1
    assert fused(N=257) == -2 and fused(N=0) == -2 and fused(d=20) == -2
    assert fused(qs=st(2048, 1024, 60)) == -3
    assert fused(q=FAKE + 8) == -4 and fused(mq=FAKE + 2) == -4 and fused(out=FAKE + 2) == -4
    assert fused(bdt=9) == -6
    assert fused(bs=st(0, 100, 8)) == -3


def fused_relpos(q=FAKE, v=FAKE, out=FAKE, table=FAKE, Gy=16, Gx=16, N=256, d=64, mq=FAKE):
    B, H = 2, 2
    s3 = st(H * N * d, N * d, d)
    return ba.lib().binattn_forward_fused_relpos(q, FAKE, v, s3, s3, s3, table, Gy, Gx, 0.125, B, H, N, d, out, s3,
                                                 mq, None, 0, None)


def test_forward_fused_relpos_rejects_bad_arguments():
    assert fused_relpos(table=None) == -1 and fused_relpos(q=None) == -1 and fused_relpos(out=None) == -1
    assert fused_relpos(Gy=32, Gx=16, N=512) == -2          # more than two key blocks
    assert fused_relpos(Gy=15) == -2 and fused_relpos(Gx=8, Gy=32) == -2
    assert fused_relpos(table=FAKE + 2) == -4 and fused_relpos(v=FAKE + 8) == -4 and fused_relpos(mq=FAKE + 1) == -4


def attention_relpos(q=FAKE, v=FAKE, out=FAKE, table=FAKE, Gy=32, Gx=64, N=2048, d=64, mq=FAKE, ws=FAKE, wsb=1 << 30):
    B, H = 2, 2
    s3 = st(H * N * d, N * d, d)
    return ba.lib().binattn_attention_relpos(q, FAKE, v, s3, s3, s3, table, Gy, Gx, 0.125, B, H, N, d, out, s3,
                                             mq, None, ws, wsb, 0, None)


def test_attention_relpos_rejects_bad_arguments():
    assert attention_relpos(table=None) == -1 and attention_relpos(q=None) == -1 and attention_relpos(out=None) == -1
    assert attention_relpos(Gy=31) == -2 and attention_relpos(Gx=48, Gy=32, N=1536) == -2   # N = Gy Gx, Gx a power of two
    assert attention_relpos(d=60) == -2
    assert attention_relpos(table=FAKE + 2) == -4 and attention_relpos(v=FAKE + 8) == -4 and attention_relpos(mq=FAKE + 1) == -4
    assert attention_relpos(ws=None) == -5 and attention_relpos(wsb=64) == -5
    # a grid the single launch takes: its checks apply
    assert attention_relpos(Gy=16, Gx=16, N=256, table=None) == -1
    assert attention_relpos(Gy=16, Gx=16, N=256, q=None) == -1


def test_debug_entry_points_reject_bad_arguments():
    L = ba.lib()
    f = lambda **k: L.binattn_logits_debug(
        k.get("qb", FAKE), k.get("kb", FAKE), 1, 2, k.get("N", 16), k.get("d", 64), k.get("r0", 0),
        k.get("r1", 16), k.get("out", FAKE), k.get("variant", 2), k.get("ws", FAKE),
        k.get("wsb", 1 << 30), None)
    assert f(qb=None) == -1 and f(out=None) == -1
    assert f(d=7) == -2
    assert f(r0=-1) == -9 and f(r1=17) == -9 and f(r0=5, r1=4) == -9
    assert f(variant=9) == -8
    assert f(ws=None) == -5 and f(wsb=10) == -5
    g = lambda **k: L.binattn_quant_v_debug(
        k.get("v", FAKE), k.get("vs", st(2048, 1024, 64)), 1, 2, 16, k.get("d", 64),
        k.get("vq", FAKE), k.get("delta", FAKE), k.get("ws", FAKE), k.get("wsb", 1 << 30), None)
    assert g(v=None) == -1 and g(vq=None) == -1 and g(delta=None) == -1
    assert g(d=3) == -2 and g(vs=st(2048, 1024, 63)) == -3 and g(v=FAKE + 2) == -4
    assert g(ws=None) == -5 and g(wsb=8) == -5


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(ba, "_lib", None)
    monkeypatch.setattr(ba, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        ba.lib()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_forward_static_rejects_bad_arguments_before_touching_the_device():
    L = ba.lib()

    def call(qb=FAKE, v=FAKE, out=FAKE, B=1, H=2, N=16, d=64, bias=None, bdt=1, bs=None):
        vs = st(H * N * d, N * d, d)
        return L.binattn_forward_static(qb, FAKE, FAKE, FAKE, v, vs, bias, bdt, bs, 0.125, B, H, N, d, out,
                                        vs, 0, None)

    assert call(qb=None) == -1 and call(out=None) == -1
    assert call(d=20) == -2 and call(N=0) == -2
    assert call(v=FAKE + 8) == -4
    assert call(bias=FAKE, bdt=9, bs=st(0, 256, 16)) == -6
    # a shape whose workspace exceeds the static scratch: refused, nothing launched
    assert ba.workspace_bytes(8, 16, 16384, 64) > ba.STATIC_SCRATCH_BYTES
    assert call(B=8, H=16, N=16384, d=64) == -10
    assert b"static" in L.binattn_strerror(-10)
    # the five benchmark workloads fit
    for (B, H, N, d) in [(1, 3, 197, 64), (64, 12, 197, 64), (32, 16, 256, 72), (8, 16, 1024, 72), (2, 16, 16384, 64)]:
        assert 0 < ba.workspace_bytes(B, H, N, d) <= ba.STATIC_SCRATCH_BYTES


def test_probe_rejects_bad_arguments():
    L = ba.lib()
    assert L.binattn_probe_valu(0, 16, 4, None, None) == -1
    assert L.binattn_probe_valu(0, 0, 4, FAKE, None) == -2 and L.binattn_probe_valu(0, 16, 0, FAKE, None) == -2
    assert L.binattn_probe_valu(0, 16, 4, FAKE + 2, None) == -4
    assert L.binattn_probe_valu(99, 16, 4, FAKE, None) == -8 and L.binattn_probe_valu(2 | (3 << 8), 16, 4, FAKE, None) == -8
