"""The C ABI on a machine without a GPU: the library loads, exports every symbol the header
declares, sizes workspaces with pure host arithmetic, and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2411_10803_amd as md
    return md.library()


def declared_symbols():
    syms = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):       # mustdrop.h and the bench-only mustdrop_bench.h
        if not name.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        syms |= set(re.findall(r"\b(mustdrop_\w+)\s*\(", text))
    return sorted(syms)


def test_every_declared_symbol_is_exported(lib):
    syms = declared_symbols()
    assert {"mustdrop_encode_merge", "mustdrop_prefill_filter", "mustdrop_decode_evict"} <= set(syms)
    for s in syms:
        assert hasattr(lib, s), f"{s} is declared in include/ but not exported"
    from paper_2411_10803_amd import binding
    assert sorted(binding.EXPORTS) == syms


def test_workspace_sizes_are_host_arithmetic(lib):
    a = lib.mustdrop_encode_merge_workspace_bytes(16, 1, 24, 24, 16, 1, 2, 2)
    b = lib.mustdrop_encode_merge_workspace_bytes(32, 1, 24, 24, 16, 1, 2, 2)
    assert 0 < a < b and a % 256 == 0
    assert lib.mustdrop_encode_merge_workspace_bytes(0, 1, 24, 24, 16, 1, 2, 2) == 0
    # 27 x 27 under 2 x 2 windows: 14 x 14 windows (the border ones clipped), more than 27*27 // 4
    assert (lib.mustdrop_encode_merge_workspace_bytes(1, 1, 27, 27, 16, 1, 2, 2)
            > lib.mustdrop_encode_merge_workspace_bytes(1, 1, 26, 26, 16, 1, 2, 2))
    assert lib.mustdrop_prefill_filter_workspace_bytes(16, 576, 64, 32, 192) > 0
    assert lib.mustdrop_decode_evict_workspace_bytes(64, 4352, 32) >= 64 * 4352 * 32 * 4


F = C.c_float
P = C.c_void_p
X = P(0x10000)        # a non-null, 16-byte aligned fake device pointer: never dereferenced on the host


def encode(lib, **kw):
    a = dict(x=X, x_dtype=1, q=X, k=X, qk_dtype=1, mass=None, valid=None, B=2, T=1, Hg=24, Wg=24, D=1024, Hc=16, dc=64,
             kt=1, kh=2, kw=2, tau=0.85, key_budget=32, out_x=P(0x9000000), oi=X, om=X, ok=X, ov=X, oc=X, ki=X,
             ws=P(0x20000000), wsb=1 << 30)
    a.update(kw)
    return lib.mustdrop_encode_merge(a["x"], a["x_dtype"], a["q"], a["k"], a["qk_dtype"], a["mass"], a["valid"],
                                     a["B"], a["T"], a["Hg"], a["Wg"], a["D"], a["Hc"], a["dc"], a["kt"], a["kh"], a["kw"],
                                     F(a["tau"]), a["key_budget"], a["out_x"], a["oi"], a["om"], a["ok"], a["ov"], a["oc"],
                                     a["ki"], None, None, a["ws"], C.c_size_t(a["wsb"]), None)


def test_encode_argument_errors(lib):
    E = dict(OK=0, EINVAL=1, ESHAPE=2, EALIGN=3, EALIAS=4, EWORKSPACE=5, EDTYPE=6)
    assert encode(lib, x=None) == E["EINVAL"] and b"required" in lib.mustdrop_last_error()
    assert encode(lib, B=0) == E["EINVAL"]
    assert encode(lib, x_dtype=7) == E["EDTYPE"]
    assert encode(lib, Hg=25, wsb=1024) == E["EWORKSPACE"]                      # a grid the window does not divide is accepted
    assert encode(lib, kh=8, kw=3, Hg=24, Wg=24) == E["ESHAPE"]                 # 24-token window > limit
    assert encode(lib, key_budget=-1) == E["EINVAL"]
    assert encode(lib, key_budget=577) == E["EINVAL"]
    assert encode(lib, q=None) == E["EINVAL"]
    assert encode(lib, Hc=8) == E["ESHAPE"]                                      # Hc*dc != D
    assert encode(lib, Hc=1024 // 48, dc=48, D=1008) == E["ESHAPE"]             # dc not a power of two
    assert encode(lib, D=1020, Hc=15, dc=68) in (E["EALIGN"], E["ESHAPE"])
    assert encode(lib, x=P(0x10008)) == E["EALIGN"]
    assert encode(lib, out_x=X) == E["EALIAS"]
    assert encode(lib, ws=None) == E["EWORKSPACE"]
    assert encode(lib, wsb=1024) == E["EWORKSPACE"] and b"needed" in lib.mustdrop_last_error()
    assert encode(lib, ws=P(0x20000010)) == E["EALIGN"]
    assert encode(lib, tau=float("nan")) == E["EINVAL"]
    assert encode(lib, key_budget=0) == E["EINVAL"]                              # q/k given without a key budget


def prefill(lib, **kw):
    a = dict(q=P(0x1000000), k=P(0x2000000), v=P(0x8000000), h=P(0x10000000), B=1, Mv=576, N=64, H=32, d=128, C=4096,
             scale=0.088, mode=0, budget=192, gamma=1 / 576, alpha=2 / 640, Rcap=192,
             ho=P(0x20000000), ko=P(0x28000000), vo=P(0x30000000), ki=X, kc=X, ws=P(0x40000000), wsb=1 << 30)
    a.update(kw)
    return lib.mustdrop_prefill_filter(a["q"], a["k"], a["v"], a["h"], None, None, None, a.get("lse"), a["B"], a["Mv"], a["N"], a["H"],
                                       a["d"], a["C"], F(a["scale"]), a["mode"], a["budget"], F(a["gamma"]), F(a["alpha"]),
                                       a["Rcap"], a["ho"], a["ko"], a["vo"], a["ki"], a["kc"], None, None, None, None, None,
                                       a["ws"], C.c_size_t(a["wsb"]), None)


def test_prefill_argument_errors(lib):
    assert prefill(lib, k=None) == 1
    assert prefill(lib, mode=3) == 6
    assert prefill(lib, d=96) == 2
    assert prefill(lib, N=1025) == 2
    assert prefill(lib, C=4100) == 3
    assert prefill(lib, budget=-1) == 1
    assert prefill(lib, gamma=0.0) == 1 and b"gamma" in lib.mustdrop_last_error()
    assert prefill(lib, Rcap=100) == 1
    assert prefill(lib, ko=P(0x2000000)) == 4
    assert prefill(lib, wsb=16) == 5
    assert prefill(lib, q=P(0x1000004)) == 3


ACC, IDS, PROT, LEN = P(0x200000), P(0x300000), P(0x400000), P(0x500000)   # the small state arrays, disjoint


def test_noalloc_rejects_shapes_beyond_the_static_buffer(lib):
    # host-side arithmetic only: the size check comes before anything touches a device
    def call(B, T):
        return lib.mustdrop_encode_merge_noalloc(X, 1, X, X, 1, None, None, B, T, 24, 24, 1024, 16, 64, 1, 2, 2, F(0.9), 32,
                                                 P(0x9000000), X, X, X, X, X, X, None, None, None)
    assert lib.mustdrop_encode_merge_workspace_bytes(64, 8, 24, 24, 16, 1, 2, 2) > (8 << 20)
    assert call(64, 8) == 5 and b"static buffer" in lib.mustdrop_last_error()
    assert call(0, 1) == 1


def decode(lib, **kw):
    a = dict(q=P(0x1000), k=P(0x10000000), v=P(0x80000000), B=2, Lcap=4096, H=32, d=128, budget=1024,
             ws=P(0x100000000), wsb=1 << 30)
    a.update(kw)
    return lib.mustdrop_decode_evict(a["q"], a["k"], a["v"], a.get("acc", ACC), a.get("ids", IDS), PROT, LEN,
                                     a["B"], a["Lcap"], a["H"], a["d"],
                                     F(0.088), F(a.get("decay", 1.0)), a["budget"], None, None, a["ws"],
                                     C.c_size_t(a["wsb"]), None)


def test_decode_argument_errors(lib):
    assert decode(lib, q=None) == 1
    assert decode(lib, d=96) == 2
    assert decode(lib, H=2048) == 2
    assert decode(lib, budget=-5) == 1
    assert decode(lib, v=P(0x10000000)) == 4
    assert decode(lib, wsb=0) == 5
    assert decode(lib, k=P(0x10000008)) == 3
    assert decode(lib, decay=-0.5) == 1 and b"decay" in lib.mustdrop_last_error()
    assert decode(lib, acc=IDS) == 4                                        # acc and ids share memory
    assert decode(lib, ids=P(0x10000000 + 4096)) == 4                       # ids inside the K cache
    assert decode(lib, ws=P(0x80000000 + 4096)) == 4                        # workspace inside the V cache
    assert decode(lib, acc=P(0x100000000 + 1024)) == 4                      # acc inside the workspace
    rc = lib.mustdrop_decode_append(None, X, X, X, X, X, X, X, 2, 64, 32, 128, 5, 1, None)
    assert rc == 1
    rc = lib.mustdrop_decode_append(X, X, X, X, X, X, X, X, 2, 64, 32, 128, -1, 1, None)
    assert rc == 1


def test_decode_keep_argument_errors(lib):
    def keep(**kw):
        a = dict(k=P(0x10000000), v=P(0x80000000), keep=X, layers=4, B=2, Lcap=640, H=32, d=128, ws=P(0x100000000),
                 wsb=1 << 30)
        a.update(kw)
        return lib.mustdrop_decode_keep(a["k"], a["v"], a["keep"], None, X, X, X, a["layers"], a["B"], a["Lcap"], a["H"],
                                        a["d"], None, None, a["ws"], C.c_size_t(a["wsb"]), None)
    assert keep(keep=None) == 1
    assert keep(layers=0) == 1
    assert keep(d=96) == 2
    assert keep(v=P(0x10000000)) == 4
    assert keep(v=P(0x10000000 + 3 * 2 * 640 * 32 * 128 * 2)) == 4     # overlaps the fourth layer of k
    assert keep(wsb=0) == 5
    assert keep(k=P(0x10000008)) == 3


def test_encode_adaptive_argument_errors(lib):
    def enc(**kw):
        a = dict(x=P(0x1000000), q=P(0x2000000), k=P(0x3000000), out=P(0x8000000), cnt=X, kc=X, lam=F(1.0), cap=16,
                 ws=P(0x100000000), wsb=1 << 30)
        a.update(kw)
        return lib.mustdrop_encode_merge_adaptive(
            a["x"], 1, a["q"], a["k"], 1, None, None, 2, 1, 24, 24, 1024, 16, 64, 1, 2, 2, F(0.9), a["lam"], a["cap"],
            a["out"], X, X, X, None, a["cnt"], X, a["kc"], None, None, a["ws"], C.c_size_t(a["wsb"]), None)
    assert enc(kc=None) == 1                         # key_count is required
    assert enc(q=None) == 1                          # q_cls is always required
    assert enc(lam=F(float("nan"))) == 1
    assert enc(cap=-1) == 1
    assert enc(wsb=16) == 5


def test_layout_argument_errors(lib):
    """md_kv_layout is checked on the host: positive multiples of 8 elements, axes nested without overlap."""
    from paper_2411_10803_amd.binding import KvLayout

    def pre(q=None, kv=None, out=None, **kw):
        a = dict(k=P(0x2000000), ko=P(0x28000000), wsb=1 << 30)
        a.update(kw)
        ref = lambda l: C.byref(l) if l is not None else None
        return lib.mustdrop_prefill_filter_strided(
            P(0x1000000), a["k"], P(0x8000000), P(0x10000000), None, None, None, None, 1, 576, 64, 32, 128, 4096,
            F(0.088), 0, 192, F(1 / 576), F(2 / 640), 192, P(0x20000000), a["ko"], P(0x30000000), X, X, None, None, None,
            None, None, ref(q), ref(kv), ref(out), P(0x40000000), C.c_size_t(a["wsb"]), None)

    L, H, d = 640, 32, 128
    head_major = KvLayout(H * L * d, d, L * d)
    assert pre(kv=KvLayout(L * H * d, H * d, 0)) == 1 and b"strides" in lib.mustdrop_last_error()
    assert pre(kv=KvLayout(L * H * d, H * d, d + 4)) == 1                   # not a multiple of 8 elements
    assert pre(kv=KvLayout(L * H * d, H * d - 8, d)) == 2 and b"overlaps" in lib.mustdrop_last_error()
    assert pre(kv=KvLayout(L * H * d, d, (L - 1) * d)) == 2                 # head slices overlap in a head-major cache
    assert pre(q=KvLayout(64 * H * d, 64, d)) == 2
    assert pre(out=KvLayout(256 * H * d, H * d, 64)) == 2                   # head stride below d
    assert pre(kv=head_major, wsb=16) == 5                                  # a valid layout gets as far as the workspace check
    assert pre(kv=KvLayout(1 << 41, H * d, d)) == 1
    # a padded layout's extent counts for the alias check: 4 KiB beyond the dense extent of k
    padded = KvLayout(L * (H * d + 4096), H * d + 4096, d)
    dense_end = 0x2000000 + L * H * d * 2
    assert pre(kv=padded, ko=P(dense_end + 4096), wsb=16) == 4
    assert pre(ko=P(dense_end + 4096), wsb=16) == 5

    def dec(lay, fn="evict"):
        if fn == "evict":
            return lib.mustdrop_decode_evict_strided(P(0x1000), P(0x10000000), P(0x80000000), ACC, IDS, PROT, LEN, 2, 4096, 32, 128,
                                                     F(0.088), F(1.0), 1024, None, None, C.byref(lay), P(0x100000000),
                                                     C.c_size_t(16), None)
        return lib.mustdrop_decode_append_strided(None, X, X, X, X, X, X, X, 2, 4096, 32, 128, 5, 1, C.byref(lay), None)

    assert dec(KvLayout(32 * 4096 * 128, 128, 4096 * 128)) == 5             # head-major: valid, stops at the workspace
    assert dec(KvLayout(32 * 4096 * 128, 128, 4095 * 128)) == 2
    assert dec(KvLayout(32 * 4096 * 128, -128, 4096 * 128)) == 1
    assert dec(KvLayout(32 * 4096 * 128, 128, 4096 * 128), "append") == 1   # null k_new
    lay = KvLayout(32 * 640 * 128, 128, 640 * 128)

    def keep(layer_stride, layers=4):
        return lib.mustdrop_decode_keep_strided(P(0x10000000), P(0x80000000), X, None, X, X, X, layers, 2, 640, 32, 128,
                                                None, None, C.byref(lay), C.c_int64(layer_stride), P(0x100000000),
                                                C.c_size_t(16), None)
    assert keep(2 * 32 * 640 * 128) == 5
    assert keep(2 * 32 * 640 * 128 - 8) == 2 and b"layer_stride" in lib.mustdrop_last_error()
    assert keep(0) == 2
    assert keep(0, layers=1) == 5                                           # one layer: the stride is not used
