"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments before anything is launched (so no GPU is needed)."""
import ctypes
import os
import re

import pytest

from paper_2505_03803_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # a non-null, 16-byte aligned address that is never dereferenced


def test_exports_match_header():
    hdr = open(os.path.join(ROOT, "include", "rwkvq.h")).read()
    declared = sorted(set(re.findall(r"\b(rwkvq_[a-z0-9_]+)\s*\(", hdr)))
    assert declared == sorted(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert B.version() >= 100


def test_status_strings():
    seen = {B.status_string(i) for i in range(6)}
    assert len(seen) == 6 and B.status_string(0) == "ok" and B.status_string(99) == "unknown status"


def test_matrix_struct_layout_matches_header():
    # ten int32 then four pointers, no padding surprises
    assert ctypes.sizeof(B.rwkvq_matrix) == 10 * 4 + 4 * 8
    assert B.rwkvq_matrix.codes.offset == 40


def sq_gemm(**kw):
    a = dict(codes=FAKE, scales=FAKE, zeros=FAKE, layout=B.CANONICAL, x=FAKE, y=FAKE, M=1, N=1024, K=1024,
             bits=3, group=128, x_dtype=B.F16, y_dtype=B.F32)
    a.update(kw)
    return B.lib().rwkvq_sq_gemm(a["codes"], a["scales"], a["zeros"], a["layout"], a["x"], a["y"], a["M"],
                                 a["N"], a["K"], a["bits"], a["group"], a["x_dtype"], a["y_dtype"], None)


def vq_gemm(**kw):
    a = dict(indices=FAKE, codebooks=FAKE, layout=B.CANONICAL, x=FAKE, y=FAKE, M=1, N=512, K=512, vdim=2,
             kbits=6, br=256, bc=256, x_dtype=B.F16, y_dtype=B.F32)
    a.update(kw)
    return B.lib().rwkvq_vq_gemm(a["indices"], a["codebooks"], a["layout"], a["x"], a["y"], a["M"], a["N"],
                                 a["K"], a["vdim"], a["kbits"], a["br"], a["bc"], a["x_dtype"], a["y_dtype"],
                                 None)


@pytest.mark.parametrize("kw,status", [
    (dict(codes=None), B.ERR_NULL), (dict(scales=None), B.ERR_NULL), (dict(zeros=None), B.ERR_NULL),
    (dict(x=None), B.ERR_NULL), (dict(y=None), B.ERR_NULL),
    (dict(M=0), B.ERR_SHAPE), (dict(N=0), B.ERR_SHAPE), (dict(N=1000), B.ERR_SHAPE),
    (dict(K=1000), B.ERR_SHAPE), (dict(K=128), B.ERR_SHAPE), (dict(K=-256), B.ERR_SHAPE),
    (dict(bits=4), B.ERR_UNSUPPORTED), (dict(group=64), B.ERR_UNSUPPORTED),
    (dict(x_dtype=B.F32), B.ERR_UNSUPPORTED), (dict(y_dtype=7), B.ERR_UNSUPPORTED),
    (dict(layout=5), B.ERR_UNSUPPORTED),
    (dict(layout=B.NATIVE), B.ERR_UNSUPPORTED),          # native layout has no separate zeros buffer
    (dict(codes=FAKE + 4), B.ERR_ALIGN), (dict(x=FAKE + 8), B.ERR_ALIGN), (dict(y=FAKE + 2), B.ERR_ALIGN),
])
def test_sq_gemm_rejects(kw, status):
    assert sq_gemm(**kw) == status


@pytest.mark.parametrize("kw,status", [
    (dict(indices=None), B.ERR_NULL), (dict(codebooks=None), B.ERR_NULL),
    (dict(N=128), B.ERR_SHAPE), (dict(K=384), B.ERR_SHAPE), (dict(M=-1), B.ERR_SHAPE),
    (dict(vdim=4), B.ERR_UNSUPPORTED), (dict(kbits=7), B.ERR_UNSUPPORTED), (dict(br=128), B.ERR_UNSUPPORTED),
    (dict(bc=512), B.ERR_UNSUPPORTED), (dict(codebooks=FAKE + 1), B.ERR_ALIGN),
])
def test_vq_gemm_rejects(kw, status):
    assert vq_gemm(**kw) == status


def test_prepack_and_dequant_reject():
    L = B.lib()
    assert L.rwkvq_sq_prepack(FAKE, FAKE, FAKE, 1024, 1024, 3, 128, None, FAKE, None) == B.ERR_NULL
    assert L.rwkvq_sq_prepack(FAKE, FAKE, FAKE, 1024, 1000, 3, 128, FAKE, FAKE, None) == B.ERR_SHAPE
    assert L.rwkvq_sq_prepack(FAKE, FAKE, FAKE, 1024, 1024, 2, 128, FAKE, FAKE, None) == B.ERR_UNSUPPORTED
    assert L.rwkvq_vq_prepack(FAKE, 512, 512, 2, 6, FAKE + 4, None) == B.ERR_ALIGN
    assert L.rwkvq_vq_prepack(None, 512, 512, 2, 6, FAKE, None) == B.ERR_NULL
    assert L.rwkvq_sq_dequant(FAKE, FAKE, FAKE, 0, 1024, 1024, 3, 128, None, B.F32, None) == B.ERR_NULL
    assert L.rwkvq_sq_dequant(FAKE, FAKE, FAKE, 0, 1024, 1024, 3, 128, FAKE, 9, None) == B.ERR_UNSUPPORTED
    assert L.rwkvq_vq_dequant(FAKE, FAKE, 0, 512, 512, 2, 6, 256, 256, FAKE + 8, B.F32, None) == B.ERR_ALIGN
    assert L.rwkvq_vq_dequant(FAKE, FAKE, 0, 512, 500, 2, 6, 256, 256, FAKE, B.F32, None) == B.ERR_SHAPE


def test_dispatch_rejects():
    L = B.lib()
    d = B.rwkvq_matrix()
    d.kind, d.layout, d.N, d.K, d.bits, d.group = B.SQ, B.CANONICAL, 1024, 1024, 3, 128
    d.codes = d.scales = d.zeros = FAKE
    mats = (B.rwkvq_matrix * 1)(d)
    xs = (ctypes.c_void_p * 1)(FAKE)
    ys = (ctypes.c_void_p * 1)(FAKE)
    assert L.rwkvq_linear_dispatch(None, xs, ys, 1, 1, B.F16, B.F32, None) == B.ERR_NULL
    assert L.rwkvq_linear_dispatch(mats, xs, ys, 0, 1, B.F16, B.F32, None) == B.ERR_SHAPE
    assert L.rwkvq_linear_dispatch(mats, xs, ys, 1, 0, B.F16, B.F32, None) == B.ERR_SHAPE
    ys0 = (ctypes.c_void_p * 1)(None)
    assert L.rwkvq_linear_dispatch(mats, xs, ys0, 1, 1, B.F16, B.F32, None) == B.ERR_NULL
    d.kind = 3
    mats = (B.rwkvq_matrix * 1)(d)
    assert L.rwkvq_linear_dispatch(mats, xs, ys, 1, 1, B.F16, B.F32, None) == B.ERR_UNSUPPORTED


def test_proxy_rejects():
    L = B.lib()
    assert L.rwkvq_proxy_workspace_bytes(1) == 65536 // 8
    assert L.rwkvq_proxy_workspace_bytes(256) == 256 * 65536 // 8
    assert L.rwkvq_proxy_workspace_bytes(0) == 0
    # the general query: 8 KiB per matrix for 16-bit weights; for binary32 two key buffers of the largest
    # matrix, 256 counts per tile of 4096 keys, 256 totals and nine partial sums per 16384 intervals
    sz = lambda Ns, Ks, dt: L.rwkvq_proxy_workspace_size((ctypes.c_int * len(Ns))(*Ns), (ctypes.c_int * len(Ks))(*Ks), len(Ns), dt)
    assert sz([256, 64], [256, 64], B.BF16) == 2 * 8192 and sz([256], [256], B.F16) == 8192
    assert sz([4096, 64], [4096, 64], B.F32) == 2 * 4 * 4096 * 4096 + 4096 * 256 * 4 + 1024 + 1024 * 9 * 8
    assert sz([3], [5], B.F32) == 256 + 256 + 1024 + 1024 + 256            # every part rounded up to 256 bytes
    assert sz([0], [5], B.F32) == 0 and sz([65536], [65536], B.F32) == 0 and sz([4], [4], 7) == 0

    def call(w=FAKE, N=256, K=256, n=1, dt=B.BF16, terms=5, ws=FAKE, out=FAKE, phi=FAKE, null_table=False):
        wp = (ctypes.c_void_p * 2)(w, FAKE)
        Ns = (ctypes.c_int * 2)(N, 256)
        Ks = (ctypes.c_int * 2)(K, 256)
        return L.rwkvq_proxy(None if null_table else wp, Ns, Ks, n, dt, terms, 1.5, 50.0, ws, out, phi, None)

    assert call(null_table=True) == B.ERR_NULL
    assert call(w=None) == B.ERR_NULL
    assert call(ws=None) == B.ERR_NULL
    assert call(out=None) == B.ERR_NULL
    assert call(phi=None) == B.ERR_NULL
    assert call(n=0) == B.ERR_SHAPE
    assert call(dt=7) == B.ERR_UNSUPPORTED
    assert call(terms=1) == B.ERR_UNSUPPORTED
    assert call(terms=9) == B.ERR_UNSUPPORTED
    assert call(N=0) == B.ERR_SHAPE
    assert call(N=1, K=1) == B.ERR_SHAPE                 # fewer than two weights: no interval
    assert call(N=65536, K=65536) == B.ERR_SHAPE          # more than 2^32 - 1 weights
    assert call(w=FAKE + 2) == B.ERR_ALIGN
    assert call(ws=FAKE + 8) == B.ERR_ALIGN
    assert call(phi=FAKE + 2) == B.ERR_ALIGN


def test_encoder_rejects():
    L = B.lib()
    sq = lambda **kw: L.rwkvq_sq_encode(*[kw.get(k, v) for k, v in
                                          [("w", FAKE), ("dt", B.BF16), ("N", 256), ("K", 256), ("bits", 3), ("group", 128),
                                           ("codes", FAKE), ("s", FAKE), ("z", FAKE), ("stream", None)]])
    assert sq(w=None) == B.ERR_NULL and sq(codes=None) == B.ERR_NULL and sq(s=None) == B.ERR_NULL and sq(z=None) == B.ERR_NULL
    assert sq(bits=4) == B.ERR_UNSUPPORTED and sq(group=64) == B.ERR_UNSUPPORTED and sq(dt=7) == B.ERR_UNSUPPORTED
    assert sq(K=200) == B.ERR_SHAPE and sq(N=0) == B.ERR_SHAPE
    assert sq(w=FAKE + 2) == B.ERR_ALIGN and sq(z=FAKE + 8) == B.ERR_ALIGN
    vq = lambda **kw: L.rwkvq_vq_assign(*[kw.get(k, v) for k, v in
                                          [("w", FAKE), ("dt", B.F32), ("cb", FAKE), ("N", 256), ("K", 512), ("vdim", 2),
                                           ("kbits", 6), ("br", 256), ("bc", 256), ("idx", FAKE), ("stream", None)]])
    assert vq(w=None) == B.ERR_NULL and vq(cb=None) == B.ERR_NULL and vq(idx=None) == B.ERR_NULL
    assert vq(vdim=4) == B.ERR_UNSUPPORTED and vq(kbits=7) == B.ERR_UNSUPPORTED and vq(br=128) == B.ERR_UNSUPPORTED
    assert vq(N=300) == B.ERR_SHAPE and vq(K=128) == B.ERR_SHAPE
    assert vq(idx=FAKE + 4) == B.ERR_ALIGN


def test_mu_path_rejects():
    from ctypes import c_int, c_void_p
    L = B.lib()
    cm = lambda **kw: L.rwkvq_clip_mean(*[kw.get(k, v) for k, v in
                                          [("x", FAKE), ("dt", B.BF16), ("B", 128), ("n", 4096), ("p", 1.0), ("out", FAKE),
                                           ("stream", None)]])
    assert cm(x=None) == B.ERR_NULL and cm(out=None) == B.ERR_NULL
    assert cm(dt=9) == B.ERR_UNSUPPORTED and cm(p=-1.0) == B.ERR_UNSUPPORTED and cm(p=50.5) == B.ERR_UNSUPPORTED
    assert cm(p=float("nan")) == B.ERR_UNSUPPORTED
    assert cm(B=0) == B.ERR_SHAPE and cm(B=70000) == B.ERR_SHAPE and cm(n=0) == B.ERR_SHAPE
    assert cm(x=FAKE + 2) == B.ERR_ALIGN and cm(out=FAKE + 2) == B.ERR_ALIGN

    arr = lambda *v: (c_void_p * len(v))(*v)
    cb = lambda **kw: L.rwkvq_mu_codebook(*[kw.get(k, v) for k, v in
                                            [("mus", arr(FAKE)), ("xb", arr(FAKE)), ("n", (c_int * 1)(4096)), ("nt", 1),
                                             ("dt", B.BF16), ("kbits", 6), ("iters", 10), ("cbs", arr(FAKE)),
                                             ("idx", arr(FAKE)), ("stream", None)]])
    assert cb(mus=None) == B.ERR_NULL and cb(idx=None) == B.ERR_NULL and cb(mus=arr(None)) == B.ERR_NULL
    assert cb(nt=0) == B.ERR_SHAPE and cb(n=(c_int * 1)(4097)) == B.ERR_SHAPE and cb(n=(c_int * 1)(0)) == B.ERR_SHAPE
    assert cb(kbits=7) == B.ERR_UNSUPPORTED and cb(dt=9) == B.ERR_UNSUPPORTED and cb(iters=-1) == B.ERR_UNSUPPORTED
    assert cb(iters=1001) == B.ERR_UNSUPPORTED
    assert cb(xb=arr(FAKE + 4)) == B.ERR_ALIGN and cb(cbs=arr(FAKE + 2)) == B.ERR_ALIGN

    mx = lambda **kw: L.rwkvq_token_shift_mix(*[kw.get(k, v) for k, v in
                                                [("x", FAKE), ("xp", FAKE), ("dt", B.F16), ("M", 4), ("d", 4096),
                                                 ("idx", arr(FAKE, FAKE)), ("cbs", arr(FAKE, FAKE)), ("kbits", 6), ("P", 2),
                                                 ("outs", arr(FAKE, FAKE)), ("stream", None)]])
    assert mx(x=None) == B.ERR_NULL and mx(xp=None) == B.ERR_NULL and mx(outs=arr(FAKE, None)) == B.ERR_NULL
    assert mx(dt=B.F32) == B.ERR_UNSUPPORTED and mx(kbits=4) == B.ERR_UNSUPPORTED and mx(P=0) == B.ERR_UNSUPPORTED
    assert mx(P=9) == B.ERR_UNSUPPORTED
    assert mx(M=0) == B.ERR_SHAPE and mx(d=4100) == B.ERR_SHAPE and mx(d=0) == B.ERR_SHAPE
    assert mx(x=FAKE + 8) == B.ERR_ALIGN and mx(idx=arr(FAKE, FAKE + 1)) == B.ERR_ALIGN


def test_dispatch_mixed_rejects():
    L = B.lib()
    good = B.rwkvq_matrix(B.SQ, B.NATIVE, 256, 512, 3, 128, 0, 0, 0, 0, FAKE, FAKE, None, None)
    canon = B.rwkvq_matrix(B.SQ, B.CANONICAL, 256, 512, 3, 128, 0, 0, 0, 0, FAKE, FAKE, FAKE, None)
    mix = lambda **kw: B.rwkvq_mix_input(kw.get("x", FAKE), kw.get("xp", FAKE), kw.get("idx", FAKE), kw.get("cb", FAKE),
                                         kw.get("kbits", 6), 0)
    from ctypes import c_void_p

    def call(mat=good, m=None, y=FAKE, n=1, xdt=B.F16, ydt=B.F32, mats_null=False):
        mats = (B.rwkvq_matrix * 1)(mat)
        mixes = (B.rwkvq_mix_input * 1)(m if m is not None else mix())
        ys = (c_void_p * 1)(y)
        return L.rwkvq_linear_dispatch_mixed(None if mats_null else mats, mixes, ys, n, xdt, ydt, None)

    assert call(mats_null=True) == B.ERR_NULL and call(y=None) == B.ERR_NULL
    assert call(m=mix(x=None)) == B.ERR_NULL and call(m=mix(xp=None)) == B.ERR_NULL
    assert call(m=mix(idx=None)) == B.ERR_NULL and call(m=mix(cb=None)) == B.ERR_NULL
    assert call(n=0) == B.ERR_SHAPE
    assert call(m=mix(kbits=7)) == B.ERR_UNSUPPORTED and call(mat=canon) == B.ERR_UNSUPPORTED
    assert call(xdt=B.F32) == B.ERR_UNSUPPORTED
    assert call(m=mix(xp=FAKE + 2)) == B.ERR_ALIGN and call(y=FAKE + 4) == B.ERR_ALIGN


def test_block_operators_reject():
    L = B.lib()
    wk = lambda **kw: L.rwkvq_wkv(*[kw.get(k, v) for k, v in
                                    [("r", FAKE), ("k", FAKE), ("v", FAKE), ("dt", B.F16), ("M", 1), ("d", 4096), ("w", FAKE),
                                     ("u", FAKE), ("state", FAKE), ("out", FAKE), ("stream", None)]])
    for name in ("r", "k", "v", "w", "u", "state", "out"):
        assert wk(**{name: None}) == B.ERR_NULL
    assert wk(dt=B.F32) == B.ERR_UNSUPPORTED and wk(dt=9) == B.ERR_UNSUPPORTED
    assert wk(M=0) == B.ERR_SHAPE and wk(d=0) == B.ERR_SHAPE
    assert wk(r=FAKE + 2) == B.ERR_ALIGN and wk(out=FAKE + 8) == B.ERR_ALIGN and wk(state=FAKE + 2) == B.ERR_ALIGN
    assert L.rwkvq_relu2(None, B.F16, 8, FAKE, None) == B.ERR_NULL
    assert L.rwkvq_relu2(FAKE, B.F32, 8, FAKE, None) == B.ERR_UNSUPPORTED
    assert L.rwkvq_relu2(FAKE, B.F16, 0, FAKE, None) == B.ERR_SHAPE
    assert L.rwkvq_relu2(FAKE + 2, B.F16, 8, FAKE, None) == B.ERR_ALIGN
    assert L.rwkvq_sigmoid_gate(FAKE, None, B.BF16, 8, FAKE, None) == B.ERR_NULL
    assert L.rwkvq_sigmoid_gate(FAKE, FAKE, 7, 8, FAKE, None) == B.ERR_UNSUPPORTED
    assert L.rwkvq_sigmoid_gate(FAKE, FAKE, B.BF16, -1, FAKE, None) == B.ERR_SHAPE
    assert L.rwkvq_sigmoid_gate(FAKE, FAKE, B.BF16, 8, FAKE + 4, None) == B.ERR_ALIGN


def test_dispatch_post_rejects():
    from ctypes import c_void_p
    L = B.lib()
    good = B.rwkvq_matrix(B.SQ, B.NATIVE, 256, 512, 3, 128, 0, 0, 0, 0, FAKE, FAKE, None, None)
    canon = B.rwkvq_matrix(B.SQ, B.CANONICAL, 256, 512, 3, 128, 0, 0, 0, 0, FAKE, FAKE, FAKE, None)
    mix = lambda **kw: B.rwkvq_mix_input(kw.get("x", FAKE), kw.get("xp", FAKE), kw.get("idx", FAKE), kw.get("cb", FAKE),
                                         kw.get("kbits", 6), 0)

    def call(mat=good, x=FAKE, m=None, op=B.POST_RELU2, gate=None, y=FAKE, n=1, xdt=B.F16, ydt=B.F16, no_x=False,
             no_posts=False, pm=None):
        mats = (B.rwkvq_matrix * 1)(mat)
        xs = None if no_x else (c_void_p * 1)(x)
        mixes = None if m is None else (B.rwkvq_mix_input * 1)(m)
        posts = None if no_posts else (B.rwkvq_post_op * 1)(B._post_op((op, gate) if pm is None else (op, gate, pm[0], pm[1])))
        ys = (c_void_p * 1)(y)
        return L.rwkvq_linear_dispatch_post(mats, xs, mixes, posts, ys, n, xdt, ydt, None)

    assert call(no_posts=True) == B.ERR_NULL and call(no_x=True) == B.ERR_NULL and call(x=None) == B.ERR_NULL
    assert call(y=None) == B.ERR_NULL and call(op=B.POST_SIGMOID_GATE, gate=None) == B.ERR_NULL
    assert call(m=mix(xp=None), no_x=True) == B.ERR_NULL and call(m=mix(x=None)) == B.ERR_NULL
    assert call(op=3) == B.ERR_UNSUPPORTED and call(op=-1) == B.ERR_UNSUPPORTED and call(mat=canon) == B.ERR_UNSUPPORTED
    assert call(m=mix(kbits=5)) == B.ERR_UNSUPPORTED and call(xdt=B.F32) == B.ERR_UNSUPPORTED
    assert call(n=0) == B.ERR_SHAPE
    assert call(op=B.POST_SIGMOID_GATE, gate=FAKE + 2) == B.ERR_ALIGN and call(x=FAKE + 8) == B.ERR_ALIGN
    assert call(m=mix(idx=FAKE + 1)) == B.ERR_ALIGN
    one = [(FAKE, FAKE, 6, FAKE)]
    assert call(pm=(None, one)) == B.ERR_NULL and call(pm=(FAKE, [(None, FAKE, 6, FAKE)])) == B.ERR_NULL
    assert call(pm=(FAKE, [(FAKE, FAKE, 6, None)])) == B.ERR_NULL
    assert call(pm=(FAKE, [(FAKE, FAKE, 7, FAKE)])) == B.ERR_UNSUPPORTED
    assert call(pm=(FAKE, one), ydt=B.F32) == B.ERR_UNSUPPORTED and call(pm=(FAKE, one), m=mix()) == B.ERR_UNSUPPORTED
    assert call(pm=(FAKE + 2, one)) == B.ERR_ALIGN and call(pm=(FAKE, [(FAKE, FAKE, 6, FAKE + 4)])) == B.ERR_ALIGN


def test_rkv_wkv_rejects():
    from ctypes import c_void_p
    L = B.lib()
    good = B.rwkvq_matrix(B.SQ, B.NATIVE, 256, 512, 3, 128, 0, 0, 0, 0, FAKE, FAKE, None, None)
    other_n = B.rwkvq_matrix(B.SQ, B.NATIVE, 512, 512, 3, 128, 0, 0, 0, 0, FAKE, FAKE, None, None)
    canon = B.rwkvq_matrix(B.SQ, B.CANONICAL, 256, 512, 3, 128, 0, 0, 0, 0, FAKE, FAKE, FAKE, None)

    def call(m=(good, good, good), xs=(FAKE, FAKE, FAKE), ys=(FAKE, FAKE, FAKE), w=FAKE, u=FAKE, state=FAKE, out=FAKE,
             xdt=B.F16, ydt=B.F16):
        return L.rwkvq_rkv_wkv((B.rwkvq_matrix * 3)(*m), (c_void_p * 3)(*xs), (c_void_p * 3)(*ys), w, u, state, out, xdt, ydt, None)

    assert call(w=None) == B.ERR_NULL and call(state=None) == B.ERR_NULL and call(out=None) == B.ERR_NULL
    assert call(xs=(FAKE, None, FAKE)) == B.ERR_NULL and call(ys=(None, FAKE, FAKE)) == B.ERR_NULL
    assert call(ydt=B.F32) == B.ERR_UNSUPPORTED and call(xdt=B.F32) == B.ERR_UNSUPPORTED
    assert call(m=(good, canon, good)) == B.ERR_UNSUPPORTED
    assert call(m=(good, good, other_n)) == B.ERR_SHAPE
    assert call(out=FAKE + 2) == B.ERR_ALIGN and call(state=FAKE + 2) == B.ERR_ALIGN and call(xs=(FAKE + 4, FAKE, FAKE)) == B.ERR_ALIGN
