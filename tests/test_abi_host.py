"""Host-side checks of the C ABI: the library loads without a GPU, exports every symbol the
header declares, and rejects invalid arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2505_13204_amd import _lib, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3
FAKE = 0x10000  # a non-null, 16-byte aligned address that is never dereferenced on the host


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(_lib.LIB_PATH):
        build.build(verbose=False)
    return _lib.load()


def test_exports_every_declared_symbol(lib):
    names = set()
    inc = os.path.join(ROOT, "include")
    headers = sorted(f for f in os.listdir(inc) if f.endswith(".h"))
    assert "aasd.h" in headers and "aasd_hooks.h" in headers
    for h in headers:
        text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, h)).read(), flags=re.S)
        names |= set(re.findall(r"\b(aasd_[a-z_]+)\s*\(", text))
    assert {"aasd_hook_sweep_events", "aasd_hook_draw_events", "aasd_hook_sweep_plan"} <= names
    assert {"aasd_version", "aasd_last_error", "aasd_align_sample", "aasd_align_sample_workspace_bytes",
            "aasd_retrieve_drafts", "aasd_verify_workspace_bytes", "aasd_verify"} <= names
    for n in names:
        assert hasattr(lib, n), n
    assert b"gfx950" in lib.aasd_version()


def _align(lib, **kw):
    a = dict(logits=FAKE, dt=1, rows=4, V=100, row_stride=100, next_tok=FAKE, m=2, c=4, mode=0, seed=0, base=0,
             argmax=FAKE, mis=FAKE, ent=FAKE, pn=FAKE, pm=FAKE, rank=FAKE, extras=FAKE, nx=FAKE, near=None, ws=FAKE,
             wsb=1 << 20, stream=None)
    a.update(kw)
    return lib.aasd_align_sample(a["logits"], a["dt"], a["rows"], a["V"], a["row_stride"], a["next_tok"], a["m"], a["c"],
                                 a["mode"], a["seed"], a["base"], a["argmax"], a["mis"], a["ent"], a["pn"], a["pm"],
                                 a["rank"], a["extras"], a["nx"], a["near"], a["ws"], a["wsb"], a["stream"])


def test_align_sample_rejects_invalid_arguments(lib):
    for kw in [dict(dt=7), dict(rows=-1), dict(V=0), dict(row_stride=99), dict(m=5), dict(m=-1), dict(c=1), dict(c=9),
               dict(m=0, c=0), dict(mode=3), dict(mode=2, extras=None), dict(logits=None), dict(argmax=None), dict(ent=None), dict(extras=None),
               dict(nx=None)]:
        assert _align(lib, **kw) == INVALID, kw
        assert lib.aasd_last_error() != b""
    assert _align(lib, logits=FAKE + 1) == UNSUPPORTED
    assert _align(lib, ws=None) == WORKSPACE
    assert _align(lib, wsb=lib.aasd_align_sample_workspace_bytes(4, 100, 1) - 1) == WORKSPACE
    assert _align(lib, ws=FAKE + 8) == WORKSPACE
    assert _align(lib, rows=0, logits=None, ws=None) == 0  # empty call is a successful no-op


def _retrieve(lib, **kw):
    a = dict(tokens=FAKE, stride=64, len=FAKE, plen=FAKE, B=2, n_min=2, n_max=4, k=8, C=4, extras=None, nx=None, m=0,
             xs=0, drafts=FAKE, dl=FAKE, sp=FAKE, nc=FAKE, kl=FAKE, dx=None, strict=FAKE, stream=None)
    a.update(kw)
    return lib.aasd_retrieve_drafts(a["tokens"], a["stride"], a["len"], a["plen"], a["B"], a["n_min"], a["n_max"], a["k"],
                                    a["C"], a["extras"], a["nx"], a["m"], a["xs"], a["drafts"], a["dl"], a["sp"], a["nc"],
                                    a["kl"], a["dx"], a["strict"], a["stream"])


def test_retrieve_drafts_rejects_invalid_arguments(lib):
    for kw in [dict(B=-1), dict(stride=0), dict(n_min=0), dict(n_min=5), dict(n_max=9), dict(k=0), dict(k=17), dict(C=0),
               dict(C=33), dict(tokens=None), dict(len=None), dict(drafts=None), dict(strict=None),
               dict(extras=FAKE), dict(extras=FAKE, nx=FAKE, m=0), dict(extras=FAKE, nx=FAKE, m=5), dict(dx=FAKE)]:
        assert _retrieve(lib, **kw) == INVALID, kw
    assert _retrieve(lib, B=0, tokens=None) == 0


def _verify(lib, **kw):
    a = dict(logits=FAKE, dt=1, B=2, C=2, k=4, V=100, rs=100, ss=900, drafts=FAKE, dl=FAKE, strict=None, alpha=0.1,
             beta=0.1, flags=0, al=FAKE, bc=FAKE, nt=FAKE, re=None, rp=None, ra=None, tp=None, td=None, near=None,
             ws=FAKE, wsb=1 << 20, stream=None)
    a.update(kw)
    return lib.aasd_verify(a["logits"], a["dt"], a["B"], a["C"], a["k"], a["V"], a["rs"], a["ss"], a["drafts"], a["dl"],
                           a["strict"], a["alpha"], a["beta"], a["flags"], a["al"], a["bc"], a["nt"], a["re"], a["rp"],
                           a["ra"], a["tp"], a["td"], a["near"], a["ws"], a["wsb"], a["stream"])


def test_verify_rejects_invalid_arguments(lib):
    for kw in [dict(dt=-1), dict(B=-1), dict(C=0), dict(C=33), dict(k=0), dict(k=17), dict(V=0), dict(rs=99), dict(ss=899),
               dict(flags=4), dict(flags=8 | 1), dict(logits=None), dict(drafts=None), dict(dl=None), dict(al=None), dict(nt=None)]:
        assert _verify(lib, **kw) == INVALID, kw
    assert _verify(lib, logits=FAKE + 1) == UNSUPPORTED
    assert _verify(lib, ws=None) == WORKSPACE
    assert _verify(lib, wsb=lib.aasd_verify_workspace_bytes(2, 2, 4, 100, 1) - 1) == WORKSPACE
    assert _verify(lib, ws=FAKE + 4) == WORKSPACE and _verify(lib, ws=FAKE + 64) == WORKSPACE   # 128-byte alignment
    assert b"workspace" in lib.aasd_last_error()
    assert _verify(lib, flags=2, ws=None) == WORKSPACE   # the one-launch form needs the caller's workspace all the more
    assert _verify(lib, B=0) == 0 and _verify(lib, B=0, flags=3) == 0


def test_verify_static_checks_its_arguments_and_its_limit(lib):
    def call(**kw):
        a = dict(logits=FAKE, dt=1, B=2, C=2, k=4, V=100, rs=100, ss=900, drafts=FAKE, dl=FAKE, strict=None, alpha=0.1,
                 beta=0.1, flags=0, al=FAKE, bc=FAKE, nt=FAKE, stream=None)
        a.update(kw)
        return lib.aasd_verify_static(a["logits"], a["dt"], a["B"], a["C"], a["k"], a["V"], a["rs"], a["ss"], a["drafts"],
                                      a["dl"], a["strict"], a["alpha"], a["beta"], a["flags"], a["al"], a["bc"], a["nt"],
                                      None, None, None, None, None, None, a["stream"])
    for kw in [dict(dt=-1), dict(B=-1), dict(C=0), dict(k=17), dict(V=0), dict(rs=99), dict(ss=899), dict(flags=2),
               dict(flags=4), dict(logits=None), dict(al=None)]:
        assert call(**kw) == INVALID, kw
    assert call(logits=FAKE + 1) == UNSUPPORTED
    assert lib.aasd_verify_static_max_bytes() == 4 << 20
    # 300 sequences of 129 rows with 4 partials of 32 bytes each: beyond the built-in 4 MiB
    assert call(B=300, C=16, k=8, ss=12900) == UNSUPPORTED and b"built-in scratch" in lib.aasd_last_error()
    assert call(B=0) == 0


def test_sweep_plan_hook_accepts_compiled_shapes_only(lib):
    """The override is validated when it is set, so no call can fail on it after its first launch."""
    base = lib.aasd_verify_workspace_bytes(1, 1, 8, 128256, 1)
    try:
        for t, l, ok in [(256, 1, True), (256, 2, True), (256, 4, True), (512, 2, True), (512, 4, True), (1024, 1, True),
                         (1024, 2, True), (512, 1, False), (1024, 4, False), (128, 2, False), (0, 2, False), (256, 0, False),
                         (300, 2, False)]:
            assert (lib.aasd_hook_sweep_plan(t, l, 0) == 0) == ok, (t, l)
        assert lib.aasd_hook_sweep_plan(256, 2, 17) == INVALID and lib.aasd_hook_sweep_plan(256, 2, -1) == INVALID
        assert lib.aasd_hook_sweep_plan(0, 0, 17) == INVALID
        assert lib.aasd_hook_sweep_plan(1024, 1, 4) == 0
        assert lib.aasd_verify_workspace_bytes(1, 1, 8, 128256, 1) == 7 * 128 + 9 * 4 * 16 * 32   # 4 segments x 16 waves; 36 workgroups count in 6 groups
        assert lib.aasd_hook_sweep_plan(0, 0, 2) == 0                                        # segments only
        assert lib.aasd_verify_workspace_bytes(1, 1, 8, 128256, 1) == 128 + 9 * 2 * 4 * 32
    finally:
        assert lib.aasd_hook_sweep_plan(0, 0, 0) == 0
    assert lib.aasd_verify_workspace_bytes(1, 1, 8, 128256, 1) == base


def test_workspace_query(lib):
    """Arrival counters (a 128-byte line per sequence, plus one per group of workgroups in short launches), then one
    32-byte partial per wave of the sweep; alignment sampling adds a list of 48 chunk positions."""
    big = lib.aasd_verify_workspace_bytes(64, 16, 8, 152064, 1)      # 8256 rows, one workgroup of 4 waves per row
    assert big == 64 * 128 + 64 * 129 * 4 * 32
    small = lib.aasd_verify_workspace_bytes(1, 1, 8, 128256, 1)        # 9 rows: rows are cut into 16 segments, 144 workgroups in 12 groups
    assert small == 13 * 128 + 9 * 16 * 4 * 32
    assert lib.aasd_verify_workspace_bytes(1, 0, 4, 100, 1) == 0
    assert lib.aasd_verify_workspace_bytes(1, 4, 17, 100, 1) == 0
    assert lib.aasd_verify_workspace_bytes(1, 4, 8, 0, 1) == 0
    assert lib.aasd_verify_workspace_bytes(1, 4, 8, 100, 5) == 0
    assert lib.aasd_verify_workspace_bytes(0, 1, 1, 100, 1) == 0
    a = lib.aasd_align_sample_workspace_bytes(65536, 128256, 1)   # 4 waves per row
    assert a == 65536 * 4 * (32 + 48 * 4)
    assert lib.aasd_align_sample_workspace_bytes(10, 0, 1) == 0
    assert lib.aasd_align_sample_workspace_bytes(10, 128256, 3) == 0
    assert lib.aasd_align_sample_workspace_bytes(0, 128256, 1) == 0


def _build_tree(lib, **kw):
    a = dict(drafts=FAKE, dl=FAKE, strict=None, dx=None, m=0, root=None, B=2, C=4, k=8, N=64, tok=FAKE, par=FAKE,
             dep=FAKE, st=FAKE, nn=FAKE, mask=None, cn=None, stream=None)
    a.update(kw)
    return lib.aasd_build_tree(a["drafts"], a["dl"], a["strict"], a["dx"], a["m"], a["root"], a["B"], a["C"], a["k"],
                               a["N"], a["tok"], a["par"], a["dep"], a["st"], a["nn"], a["mask"], a["cn"], a["stream"])


def test_build_tree_rejects_invalid_arguments(lib):
    for kw in [dict(B=-1), dict(k=0), dict(k=17), dict(C=0), dict(C=33), dict(m=-1), dict(m=5), dict(dx=FAKE, m=0),
               dict(N=0), dict(N=513), dict(drafts=None), dict(dl=None), dict(tok=None), dict(par=None), dict(dep=None),
               dict(st=None), dict(nn=None)]:
        assert _build_tree(lib, **kw) == INVALID, kw
        assert b"build_tree" in lib.aasd_last_error()
    assert _build_tree(lib, B=0, drafts=None) == 0


def _verify_tree(lib, **kw):
    a = dict(logits=FAKE, dt=1, B=2, N=16, V=100, rs=100, ss=1600, tok=FAKE, par=FAKE, st=None, nn=FAKE, alpha=0.1,
             beta=0.1, flags=0, al=FAKE, bn=FAKE, path=None, nt=FAKE, re=None, rp=None, ra=None, np_=None, nd=None,
             near=None, ws=FAKE, wsb=1 << 20, stream=None)
    a.update(kw)
    return lib.aasd_verify_tree(a["logits"], a["dt"], a["B"], a["N"], a["V"], a["rs"], a["ss"], a["tok"], a["par"],
                                a["st"], a["nn"], a["alpha"], a["beta"], a["flags"], a["al"], a["bn"], a["path"], a["nt"],
                                a["re"], a["rp"], a["ra"], a["np_"], a["nd"], a["near"], a["ws"], a["wsb"], a["stream"])


def test_verify_tree_rejects_invalid_arguments(lib):
    for kw in [dict(dt=2), dict(B=-1), dict(N=0), dict(N=513), dict(V=0), dict(rs=99), dict(ss=1599), dict(flags=4),
               dict(logits=None), dict(tok=None), dict(par=None), dict(nn=None), dict(al=None), dict(bn=None),
               dict(nt=None)]:
        assert _verify_tree(lib, **kw) == INVALID, kw
    assert _verify_tree(lib, logits=FAKE + 1) == UNSUPPORTED
    assert _verify_tree(lib, ws=None) == WORKSPACE
    assert _verify_tree(lib, wsb=lib.aasd_verify_tree_workspace_bytes(2, 16, 100, 1) - 1) == WORKSPACE
    assert _verify_tree(lib, ws=FAKE + 4) == WORKSPACE
    assert _verify_tree(lib, B=0) == 0
    # the sweep is planned as if a quarter of the rows were in use: 8192 rows -> 4 segments of 4 waves per row
    assert lib.aasd_verify_tree_workspace_bytes(128, 64, 128256, 1) == 128 * 64 * 4 * 4 * 32
    assert lib.aasd_verify_tree_workspace_bytes(512, 64, 128256, 1) == 512 * 64 * 4 * 32      # 32768 rows: 4 waves per row
    assert lib.aasd_verify_tree_workspace_bytes(1, 0, 100, 1) == 0
    assert lib.aasd_verify_tree_workspace_bytes(1, 513, 100, 1) == 0


def _verify_topk(lib, **kw):
    a = dict(logits=FAKE, dt=1, B=2, C=2, k=4, V=100, rs=100, ss=900, drafts=FAKE, dl=FAKE, topk=5, al=FAKE, bc=FAKE,
             nt=FAKE, ra=None, tp=None, ws=FAKE, wsb=1 << 20, stream=None)
    a.update(kw)
    return lib.aasd_verify_topk(a["logits"], a["dt"], a["B"], a["C"], a["k"], a["V"], a["rs"], a["ss"], a["drafts"],
                                a["dl"], a["topk"], a["al"], a["bc"], a["nt"], a["ra"], a["tp"], a["ws"], a["wsb"],
                                a["stream"])


def test_verify_topk_rejects_invalid_arguments(lib):
    for kw in [dict(dt=3), dict(B=-1), dict(C=0), dict(C=33), dict(k=0), dict(k=17), dict(V=0), dict(rs=99), dict(ss=899),
               dict(topk=0), dict(topk=9), dict(logits=None), dict(drafts=None), dict(dl=None), dict(al=None),
               dict(bc=None), dict(nt=None)]:
        assert _verify_topk(lib, **kw) == INVALID, kw
        assert b"verify_topk" in lib.aasd_last_error()
    assert _verify_topk(lib, logits=FAKE + 1) == UNSUPPORTED
    assert _verify_topk(lib, ws=None) == WORKSPACE
    assert _verify_topk(lib, wsb=lib.aasd_verify_topk_workspace_bytes(2, 2, 4, 100, 1) - 1) == WORKSPACE
    assert _verify_topk(lib, B=0) == 0
    assert lib.aasd_verify_topk_workspace_bytes(2, 2, 4, 100, 1) > lib.aasd_verify_workspace_bytes(2, 2, 4, 100, 1)
    assert lib.aasd_verify_topk_workspace_bytes(2, 0, 4, 100, 1) == 0


def test_pool_rejects_invalid_arguments(lib):
    need = lib.aasd_pool_bytes(2, 1000, 2, 4)
    # counters, then per (sequence, key length) a table of 2048 heads (load factor <= 1/2) and 1001 links
    assert need == 32 + 2 * 3 * ((2048 + 1001) * 4 + 12)
    for args in [(-1, 10, 1, 1), (1, 0, 1, 1), (1, (1 << 24) + 1, 1, 1), (1, 10, 0, 1), (1, 10, 3, 2), (1, 10, 1, 9)]:
        assert lib.aasd_pool_bytes(*args) == 0
    def upd(**kw):
        a = dict(pool=FAKE, nb=need, B=2, cap=1000, n_min=2, n_max=4, tok=FAKE, stride=1000, len=FAKE, reset=1, stream=None)
        a.update(kw)
        return lib.aasd_pool_update(a["pool"], a["nb"], a["B"], a["cap"], a["n_min"], a["n_max"], a["tok"], a["stride"],
                                    a["len"], a["reset"], a["stream"])
    for kw in [dict(B=-1), dict(cap=0), dict(n_min=0), dict(n_max=9), dict(n_min=5), dict(stride=0), dict(tok=None), dict(len=None)]:
        assert upd(**kw) == INVALID, kw
    assert upd(pool=None) == WORKSPACE and upd(nb=need - 1) == WORKSPACE and upd(pool=FAKE + 8) == WORKSPACE
    assert upd(B=0) == 0
    def ret(**kw):
        a = dict(pool=FAKE, nb=need, B=2, cap=1000, n_min=2, n_max=4, tok=FAKE, stride=1000, len=FAKE, plen=FAKE, k=8, C=4,
                 extras=None, nx=None, m=0, xs=0, drafts=FAKE, dl=FAKE, sp=FAKE, nc=FAKE, kl=FAKE, dx=None, strict=FAKE,
                 stream=None)
        a.update(kw)
        return lib.aasd_pool_retrieve(a["pool"], a["nb"], a["B"], a["cap"], a["n_min"], a["n_max"], a["tok"], a["stride"],
                                      a["len"], a["plen"], a["k"], a["C"], a["extras"], a["nx"], a["m"], a["xs"], a["drafts"],
                                      a["dl"], a["sp"], a["nc"], a["kl"], a["dx"], a["strict"], a["stream"])
    for kw in [dict(B=-1), dict(cap=0), dict(k=0), dict(k=17), dict(C=0), dict(C=33), dict(tok=None), dict(plen=None),
               dict(drafts=None), dict(strict=None), dict(extras=FAKE), dict(extras=FAKE, nx=FAKE, m=5), dict(dx=FAKE)]:
        assert ret(**kw) == INVALID, kw
    assert ret(pool=None) == WORKSPACE and ret(nb=need - 1) == WORKSPACE
    assert ret(B=0) == 0


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 on its own (no C++ or HIP types in it)."""
    import subprocess
    src = tmp_path / "use.c"
    src.write_text('#include "aasd.h"\n#include "aasd_hooks.h"\nint main(void) { return (int)sizeof(aasd_status) + AASD_MAX_TREE_NODES > 0 ? 0 : 1; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only",
                           "-I", os.path.join(ROOT, "include"), str(src)])


def test_which_form_a_verification_takes(lib):
    """One launch only with a zeroed counter area and for a small call (measured: from about 128 rows on two are faster)."""
    lib.aasd_hook_verify_launches.restype = ctypes.c_int32
    lib.aasd_hook_verify_launches.argtypes = [ctypes.c_int32] * 5 + [ctypes.c_uint32]
    ZEROED = 2
    assert lib.aasd_hook_verify_launches(1, 1, 8, 128256, 1, ZEROED) == 1      # 9 rows
    assert lib.aasd_hook_verify_launches(14, 1, 8, 128256, 1, ZEROED) == 1     # 126 rows
    assert lib.aasd_hook_verify_launches(32, 1, 8, 128256, 1, ZEROED) == 2     # 288 rows
    assert lib.aasd_hook_verify_launches(1, 1, 8, 128256, 1, 0) == 2           # nobody vouches for the counters
    assert lib.aasd_hook_verify_launches(1, 16, 8, 152064, 1, ZEROED) == 2     # 129 rows
    assert lib.aasd_hook_verify_launches(0, 1, 8, 128256, 1, ZEROED) == 0 and lib.aasd_hook_verify_launches(1, 1, 8, 0, 1, 0) == 0

