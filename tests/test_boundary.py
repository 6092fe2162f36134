"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, and rejects bad arguments with the documented status before anything is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "parse.h")

pa = pytest.importorskip("paper_2605_08568_amd")
from paper_2605_08568_amd import binding as B  # noqa: E402

FAKE = C.c_void_p(0x1000)      # non-NULL, 16-byte aligned, never dereferenced: every check below fails first
FAKE2 = C.c_void_p(0x2000)
ODD = C.c_void_p(0x1004)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(parse_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = pa.lib()
    names = declared_functions()
    assert {"parse_route", "parse_cache_lookup", "parse_pack_experts", "parse_lowrank_forward"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_status_strings_and_version():
    assert pa.version() >= 100
    for code in range(0, -8, -1):
        assert pa.status_string(code) != "unknown status"
    assert pa.status_string(-99) == "unknown status"


def test_check_offsets():
    assert pa.check_offsets(np.array([0, 3, 5]), 5) == 0
    assert pa.check_offsets(np.array([0, 3, 3, 5]), 5) == -2      # empty prompt
    assert pa.check_offsets(np.array([0, 4, 3, 5]), 5) == -2      # not ascending
    assert pa.check_offsets(np.array([1, 3, 5]), 5) == -2         # does not start at 0
    assert pa.check_offsets(np.array([0, 3, 5]), 6) == -2         # does not end at rows
    assert pa.lib().parse_check_offsets(None, 2, 5) == -1


def test_check_subset():
    assert pa.check_subset(np.array([0, 2, 5]), 6) == 0
    assert pa.check_subset(np.array([0, 2, 6]), 6) == -2          # out of range
    assert pa.check_subset(np.array([2, 2]), 6) == -2             # duplicate
    assert pa.check_subset(np.array([3, 1]), 6) == -2             # not ascending
    assert pa.check_subset(np.arange(7), 6) == -2                 # k > G


def _layer(n=64, m=64, R=32, G=2, dtype=0, layout=0, Vt=FAKE, Ut=FAKE2):
    return B._Layer(n, m, R, G, dtype, layout, Vt.value, Ut.value)


def test_route_rejects_bad_arguments():
    lib = pa.lib()
    ok = dict(X=FAKE, xdt=0, rows=8, off=FAKE, P=2, d=64, Wr=FAKE, G=4, k=2, out=FAKE, stride=2, ws=FAKE, wsb=1 << 20)

    def call(**kw):
        a = dict(ok); a.update(kw)
        return lib.parse_route(a["X"], a["xdt"], a["rows"], a["off"], a["P"], a["d"], a["Wr"], a["G"], a["k"],
                               a["out"], a["stride"], None, None, a["ws"], a["wsb"], None)

    assert call(X=None) == -1 and call(off=None) == -1 and call(Wr=None) == -1 and call(out=None) == -1
    assert call(xdt=7) == -1 and call(rows=0) == -1
    assert call(k=5) == -2 and call(G=65, k=2) == -2 and call(P=9) == -2 and call(stride=1) == -2
    assert call(d=60) == -3 and call(X=ODD) == -3
    assert call(ws=None) == -5 and call(wsb=16) == -5

    def pool(**kw):     # the embedding-only call: the same checks without the router's
        a = dict(ok, emb=FAKE); a.update(kw)
        return lib.parse_pool(a["X"], a["xdt"], a["rows"], a["off"], a["P"], a["d"], a["emb"], a["ws"], a["wsb"], None)

    assert pool(X=None) == -1 and pool(off=None) == -1 and pool(emb=None) == -1
    assert pool(xdt=7) == -1 and pool(rows=0) == -1 and pool(P=0) == -1
    assert pool(P=9) == -2 and pool(d=16392, wsb=1 << 30) == -2
    assert pool(d=60) == -3 and pool(X=ODD) == -3 and pool(emb=ODD) == -3
    assert pool(ws=None) == -5 and pool(wsb=16) == -5


def test_cache_create_rejects_bad_arguments():
    lib = pa.lib()
    h = C.c_void_p()
    assert lib.parse_cache_create(None, 4, 64, 1, 2, 4) == -1
    assert lib.parse_cache_create(C.byref(h), 0, 64, 1, 2, 4) == -1
    assert lib.parse_cache_create(C.byref(h), 4, 62, 1, 2, 4) == -3
    assert lib.parse_cache_create(C.byref(h), 4, 64, 1, 65, 4) == -2
    assert lib.parse_cache_lookup(None, FAKE, 1, 0.9, FAKE, None, None, None) == -1
    assert lib.parse_cache_destroy(None) == -1


def test_pack_and_bucket_reject_bad_arguments():
    lib = pa.lib()
    L = _layer()
    assert lib.parse_pack_experts(C.byref(L), None, 1, FAKE, FAKE, None) == -1
    assert lib.parse_pack_experts(C.byref(L), FAKE, 3, FAKE, FAKE, None) == -2       # k > G
    assert lib.parse_pack_experts(C.byref(L), FAKE, 1, ODD, FAKE, None) == -3
    bad = _layer(R=33)                                                                 # R % G != 0
    assert lib.parse_pack_experts(C.byref(bad), FAKE, 1, FAKE, FAKE, None) == -2
    bad = _layer(n=62)                                                                 # rows not 16-byte multiples
    assert lib.parse_pack_experts(C.byref(bad), FAKE, 1, FAKE, FAKE, None) == -3
    bad = _layer(dtype=0, layout=1)                                                    # operand order is bf16 only
    assert lib.parse_pack_experts(C.byref(bad), FAKE, 1, FAKE, FAKE, None) == -7
    bad = _layer(dtype=1, layout=1, R=32, G=2)                                         # gs = 16 not a multiple of 32
    assert lib.parse_pack_experts(C.byref(bad), FAKE, 1, FAKE, FAKE, None) == -2
    assert lib.parse_layer_to_mfma16(C.byref(_layer(dtype=0)), FAKE, FAKE, None) == -7
    assert lib.parse_bucket_patterns(FAKE, 2000, 2, 2, FAKE, FAKE, FAKE, FAKE, FAKE, None) == -2
    assert lib.parse_bucket_patterns(FAKE, 4, 2, 1, FAKE, FAKE, FAKE, FAKE, FAKE, None) == -2
    assert lib.parse_bucket_patterns(None, 4, 2, 2, FAKE, FAKE, FAKE, FAKE, FAKE, None) == -1


def test_forward_rejects_bad_arguments():
    lib = pa.lib()
    L = _layer()
    pt = B._Patterns(FAKE.value, FAKE.value, FAKE.value, 1, 2, 1)

    def call(mode=0, layer=L, pat=pt, X=FAKE, rows=8, off=FAKE, pid=FAKE, P=2, Y=FAKE, ws=FAKE, wsb=1 << 22):
        return lib.parse_lowrank_forward(mode, C.byref(layer), C.byref(pat), X, rows, off, pid, P, Y, ws, wsb, None)

    assert call(mode=3) == -1 and call(X=None) == -1 and call(Y=None) == -1 and call(pid=None) == -1
    assert call(off=None) == -1 and call(rows=0) == -1
    assert call(P=9) == -2 and call(X=ODD) == -3
    assert call(ws=None) == -5 and call(wsb=8) == -5                     # fp32 prefill needs the Z workspace
    assert call(pat=B._Patterns(FAKE.value, FAKE.value, FAKE.value, 3, 2, 3)) == -2   # k > G
    assert call(layer=_layer(dtype=1, layout=0)) == -7                  # bf16 prefill needs operand order
    assert call(mode=1) == -7                                           # decode is bf16 operand-order only
    Lb = _layer(n=64, m=64, R=64, G=2, dtype=1, layout=1)
    assert call(mode=1, layer=Lb, rows=40, P=20) == -2                  # decode: one token per sequence (rows == P)
    assert call(mode=1, layer=Lb, rows=8, P=4) == -2                    # decode: one row per sequence
    assert lib.parse_lowrank_workspace_bytes(0, C.byref(L), 8, 1, 0, 0) >= 8 * 16 * 4


def test_decode_multi_rejects_bad_arguments():
    lib = pa.lib()
    La = _layer(n=64, m=64, R=64, G=2, dtype=1, layout=1)
    Lb = _layer(n=128, m=64, R=64, G=2, dtype=1, layout=1)
    pt = B._Patterns(None, None, FAKE.value, 1, 2, 1)

    def call(layers, pats, nl, X=FAKE, rows=8, pid=FAKE, ys=None, ws=FAKE, wsb=1 << 24):
        larr = (B._Layer * len(layers))(*layers)
        parr = (B._Patterns * len(pats))(*pats)
        yarr = (C.c_void_p * len(layers))(*(ys if ys is not None else [FAKE.value] * len(layers)))
        return lib.parse_lowrank_decode_multi(larr, parr, nl, X, rows, pid, yarr, ws, wsb, None)

    assert call([La, La], [pt, pt], 0) == -1 and call([La, La], [pt, pt], 2, X=None) == -1
    assert call([La] * 5, [pt] * 5, 5) == -2                       # at most four layers
    assert call([La, Lb], [pt, pt], 2) == -2                       # the layers must share the input width
    assert call([La, _layer(n=64, m=64, R=64, G=2, dtype=1, layout=0)], [pt, pt], 2) == -7
    assert call([La, La], [pt, pt], 2, ys=[FAKE.value, None]) == -1
    assert call([La, La], [pt, pt], 2, wsb=64) == -5
    larr = (B._Layer * 2)(La, La)
    assert lib.parse_lowrank_decode_multi_workspace_bytes(larr, 2) == 2 * lib.parse_lowrank_workspace_bytes(1, C.byref(La), 8, 1, 0, 0)


def test_prefill_multi_rejects_bad_arguments():
    lib = pa.lib()
    La = _layer(n=256, m=256, R=256, G=2, dtype=1, layout=1)          # k*gs = 128
    Lb = _layer(n=512, m=256, R=256, G=2, dtype=1, layout=1)
    Lc = _layer(n=256, m=256, R=128, G=2, dtype=1, layout=1)          # k*gs = 64: not a multiple of 128
    pt = B._Patterns(FAKE.value, FAKE.value, None, 1, 2, 1)

    def call(layers, pats, nl, X=FAKE, rows=8, off=FAKE, pid=FAKE, P=2, ys=None, ws=FAKE, wsb=1 << 24):
        larr = (B._Layer * len(layers))(*layers)
        parr = (B._Patterns * len(pats))(*pats)
        yarr = (C.c_void_p * len(layers))(*(ys if ys is not None else [FAKE.value] * len(layers)))
        return lib.parse_lowrank_prefill_multi(larr, parr, nl, X, rows, off, pid, P, yarr, ws, wsb, None)

    assert call([La, La], [pt, pt], 0) == -1 and call([La, La], [pt, pt], 2, off=None) == -1
    assert call([La] * 5, [pt] * 5, 5) == -2 and call([La, La], [pt, pt], 2, P=9) == -2
    assert call([La, Lb], [pt, pt], 2) == -2                       # the layers must share the input width
    pt_tiles = B._Patterns(FAKE.value, FAKE.value, None, 1, 2, 1, None, None, 0, 2)
    assert call([La, Lc], [pt_tiles, pt_tiles], 2) == -2           # two-launch schedule: selected ranks not a multiple of 128
    pt_fused = B._Patterns(FAKE.value, FAKE.value, None, 1, 2, 1, None, None, 0, 1)
    assert call([La, La], [pt_fused, pt_fused], 2) == -1           # the single-launch kernel takes one layer only
    assert call([La, _layer(n=256, m=256, R=256, G=2, dtype=1, layout=0)], [pt, pt], 2) == -7
    assert call([La, La], [pt, pt], 2, ys=[FAKE.value, None]) == -1
    assert call([La, La], [pt, pt], 2, wsb=64) == -5 and call([La, La], [pt, pt], 2, ws=None) == -5


def test_rank_granular_entry_points_reject_bad_arguments():
    lib = pa.lib()

    def route(X=FAKE, xdt=1, rows=64, off=FAKE, P=2, d=64, Wr=FAKE, G=128, K=32, out=FAKE, stride=32, ws=FAKE, wsb=1 << 24):
        return lib.parse_route_ranks(X, xdt, rows, off, P, d, Wr, G, K, out, stride, None, None, ws, wsb, None)

    assert route(X=None) == -1 and route(K=0) == -1 and route(xdt=5) == -1
    assert route(K=256) == -2 and route(G=9000, K=32) == -2 and route(stride=16) == -2 and route(P=100) == -2
    assert route(d=68) == -3 and route(X=ODD) == -3
    assert route(ws=None) == -5 and route(wsb=64) == -5
    assert lib.parse_route_ranks_workspace_bytes(64, 2, 64, 128) >= 2 * 64 * 4 + 2 * 128 * 4
    rm = _layer(n=64, m=64, R=128, G=128, dtype=1, layout=0)
    assert lib.parse_pack_ranks(C.byref(rm), None, 32, 32, 2, FAKE, FAKE, None) == -1
    assert lib.parse_pack_ranks(C.byref(rm), FAKE, 32, 48, 2, FAKE, FAKE, None) == -2              # K % 32
    assert lib.parse_pack_ranks(C.byref(rm), FAKE, 16, 32, 2, FAKE, FAKE, None) == -2              # stride < K
    assert lib.parse_pack_ranks(C.byref(_layer(n=64, m=64, R=128, G=4, dtype=1, layout=1)), FAKE, 32, 32, 2, FAKE, FAKE, None) == -7
    assert lib.parse_pack_ranks(C.byref(_layer(n=64, m=64, R=128, G=128, dtype=0, layout=0)), FAKE, 32, 32, 2, FAKE, FAKE, None) == -7


def test_router_grad_rejects_bad_arguments():
    lib = pa.lib()
    L = _layer(n=256, m=128, R=64, G=2, dtype=1, layout=1)

    def call(layer=L, U=FAKE, X=FAKE, rows=16, off=FAKE, P=2, yh=FAKE, yd=FAKE, emb=FAKE, sc=FAKE, d=256, k=1,
             tau=1.0, eps=1e-6, grad=FAKE, ws=FAKE, wsb=1 << 24):
        return lib.parse_router_grad(C.byref(layer), U, X, rows, off, P, yh, yd, emb, sc, d, k, tau, eps, None, grad, ws,
                                     wsb, None)

    assert call(U=None) == -1 and call(grad=None) == -1 and call(tau=0.0) == -1 and call(k=0) == -1
    assert call(k=3) == -2 and call(P=17) == -2
    assert call(layer=_layer(n=200, m=128, R=64, G=2, dtype=1, layout=1)) == -2        # n not a multiple of 128
    assert call(layer=_layer(n=256, m=128, R=64, G=2, dtype=1, layout=0)) == -7
    assert call(X=ODD) == -3 and call(ws=None) == -5 and call(wsb=64) == -5
    assert lib.parse_router_grad_workspace_bytes(C.byref(L), 16, 2) >= 16 * 128 * 2 + 2 * 16 * 64 * 2


def test_plan_entry_points_reject_bad_arguments_and_size_their_buffers():
    """Prefill plan, decode plan and the calls that run over them: sizes the host works out, and every rejection that
    happens before a launch."""
    lib = pa.lib()
    lib.parse_prefill_plan_bytes.restype = C.c_size_t
    lib.parse_decode_plan_bytes.restype = C.c_size_t
    # prefill plan: 16 header words, the tile patterns (rounded up to 16), 256 row-map words per tile;
    # capacity = ceil(rows / 256) + min(P, n_patterns + 1)
    def plan_bytes(rows, P, npat):
        cap = (rows + 255) // 256 + min(P, npat + 1)
        words = 16 + (cap + 15) // 16 * 16 + cap * 256
        return (words * 4 + 255) // 256 * 256
    for rows, P, npat in ((4096, 8, 32), (300, 300, 4), (1, 1, 1), (272660, 256, 32)):
        assert lib.parse_prefill_plan_bytes(rows, P, npat) == plan_bytes(rows, P, npat)
    assert lib.parse_prefill_plan_bytes(0, 1, 1) == 0

    def plan(off=FAKE, pid=FAKE, P=8, rows=4096, npat=32, buf=FAKE, nbytes=1 << 24):
        return lib.parse_prefill_plan(off, pid, P, rows, npat, buf, nbytes, None)
    assert plan(off=None) == -1 and plan(pid=None) == -1 and plan(buf=None) == -1 and plan(P=0) == -1
    assert plan(P=5000, rows=4096) == -2                       # more prompts than rows
    assert plan(P=3000, rows=4096) == -2 and plan(npat=3000) == -2   # the plan kernel's table sizes
    assert plan(buf=ODD) == -3 and plan(nbytes=1024) == -5

    # buckets and plan in one launch: the union of the two calls' checks
    def both(sub=FAKE, P=8, k=4, stride=4, outs=(FAKE,) * 5, off=FAKE, pid=FAKE, rows=4096, npat=32, buf=FAKE, nbytes=1 << 24):
        return lib.parse_bucket_and_plan(sub, P, k, stride, *outs, off, pid, rows, npat, buf, nbytes, None)
    assert both(sub=None) == -1 and both(off=None) == -1 and both(pid=None) == -1 and both(buf=None) == -1
    for i in range(5):
        assert both(outs=tuple(None if j == i else FAKE for j in range(5))) == -1
    assert both(P=0) == -1 and both(k=0) == -1 and both(rows=0) == -1 and both(npat=0) == -1
    assert both(P=1025, rows=1 << 20) == -2 and both(k=65, stride=65) == -2 and both(stride=3) == -2
    assert both(P=5000, rows=4096) == -2 and both(npat=3000) == -2
    assert both(buf=ODD) == -3 and both(nbytes=1024) == -5

    # planned prefill of one layer
    L = _layer(n=256, m=256, R=256, G=4, dtype=1, layout=1)           # gs = 64
    pt = B._Patterns(FAKE.value, FAKE.value, None, 2, 4, 2)           # k = 2 -> r_S = 128
    def planned(layer=L, pat=pt, X=FAKE, rows=512, off=FAKE, pid=FAKE, P=2, pl=FAKE, Y=FAKE, ws=FAKE, wsb=1 << 24):
        return lib.parse_lowrank_prefill_planned(C.byref(layer), C.byref(pat), X, rows, off, pid, P, pl, Y, ws, wsb, None)
    assert planned(pl=None) == -1 and planned(off=None) == -1 and planned(Y=None) == -1
    assert planned(layer=_layer(n=256, m=256, R=256, G=4, dtype=1, layout=0)) == -7
    assert planned(layer=_layer(n=256, m=256, R=256, G=4, dtype=0, layout=0)) == -7
    assert planned(P=600) == -2 and planned(layer=_layer(n=80, m=256, R=64, G=2, dtype=1, layout=1)) == -2   # n % 64
    head = B._Patterns(FAKE.value, FAKE.value, None, 2, 4, 2, FAKE.value, FAKE.value, 2, 0)
    assert planned(pat=head) == -2                                    # the shared head must leave groups to the patterns
    assert planned(pat=B._Patterns(FAKE.value, FAKE.value, None, 2, 4, 2, None, None, 1, 0)) == -1   # head without its store
    assert planned(X=ODD) == -3 and planned(pl=ODD) == -3
    assert planned(ws=None) == -5 and planned(wsb=4096) == -5
    lib.parse_lowrank_prefill_planned_workspace_bytes.restype = C.c_size_t
    cap = 2 + 2                                                        # 512 rows, two prompts, four patterns
    assert lib.parse_lowrank_prefill_planned_workspace_bytes(C.byref(L), 512, 2, 2, 4) == cap * 256 * 128 * 2

    # decode plan: 704 words per layer (count, 64 group ids, 64 masks, padding to 192, 512 arrival counters)
    assert lib.parse_decode_plan_bytes(1) == 704 * 4 and lib.parse_decode_plan_bytes(3) == (3 * 704 * 4 + 255) // 256 * 256
    assert lib.parse_decode_plan_bytes(0) == 0 and lib.parse_decode_plan_bytes(5) == 0
    D = _layer(n=256, m=256, R=256, G=4, dtype=1, layout=1)
    dp = B._Patterns(None, None, FAKE.value, 2, 4, 2)
    def dplan(layers=(D,), pats=(dp,), nl=1, pid=FAKE, rows=8, buf=FAKE, nbytes=1 << 16):
        larr = (B._Layer * len(layers))(*layers)
        parr = (B._Patterns * len(pats))(*pats)
        return lib.parse_decode_plan(larr, parr, nl, pid, rows, buf, nbytes, None)
    assert dplan(pid=None) == -1 and dplan(buf=None) == -1 and dplan(rows=0) == -1 and dplan(nl=0) == -1
    assert dplan(rows=33) == -2                                        # a plan covers one panel of 32 sequences
    assert dplan(layers=(D,) * 5, pats=(dp,) * 5, nl=5) == -2
    assert dplan(layers=(_layer(n=256, m=256, R=256, G=4, dtype=1, layout=0),)) == -7
    assert dplan(pats=(B._Patterns(None, None, None, 2, 4, 2),)) == -1  # decode needs the subsets
    assert dplan(buf=ODD) == -3 and dplan(nbytes=512) == -5

    def dstep(layers=(D,), nl=1, X=FAKE, rows=8, pl=FAKE, ys=None, ws=FAKE, wsb=1 << 24):
        larr = (B._Layer * len(layers))(*layers)
        yarr = (C.c_void_p * len(layers))(*(ys if ys is not None else [FAKE.value] * len(layers)))
        return lib.parse_lowrank_decode_planned(larr, nl, X, rows, pl, yarr, ws, wsb, None)
    assert dstep(X=None) == -1 and dstep(pl=None) == -1 and dstep(rows=0) == -1 and dstep(ys=[None]) == -1
    assert dstep(rows=33) == -2 and dstep(X=ODD) == -3 and dstep(pl=ODD) == -3
    assert dstep(ws=None) == -5 and dstep(wsb=64) == -5
    # workspace of a decode call: z as operands (64 bytes per stored rank); partial sums (128 bytes per stored rank and
    # slice) only when the reduction over n is split -- not here (n = 256, few rank blocks -> up to 2 slices of >= 8 steps)
    lib.parse_lowrank_decode_planned_workspace_bytes.restype = C.c_size_t
    larr = (B._Layer * 1)(D)
    need = lib.parse_lowrank_decode_planned_workspace_bytes(larr, 1)
    assert need in (256 * 64, 256 * 64 + 256 * 128 * 2)
    big = (B._Layer * 1)(_layer(n=11008, m=4096, R=2560, G=20, dtype=1, layout=1))
    assert lib.parse_lowrank_decode_planned_workspace_bytes(big, 1) == 2560 * 64 + 2560 * 128 * 3   # three slices of 229-230 steps
    lib.parse_lowrank_decode_static_capacity.restype = C.c_size_t
    assert lib.parse_lowrank_decode_static_capacity() == 4 << 20
