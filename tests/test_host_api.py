"""Host logic of the C-ABI library, no GPU needed: the library loads, exports
every symbol the header declares, and rejects bad arguments before any HIP call."""
import ctypes
import os
import re

import pytest

from conftest import ROOT
from paper_2605_24584_amd import binding as B

FAKE = 0x10000          # a non-null, 256-byte aligned "device pointer" that must never be touched


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_2605_24584_amd import build
        build.build()
    return B.lib()


def test_every_declared_symbol_is_exported(L):
    for header_name, names in (("laplex.h", B.EXPORTS), ("laplex_diag.h", B.DIAG_EXPORTS)):
        header = open(os.path.join(ROOT, "include", header_name)).read()
        declared = set(re.findall(r"\b(laplex_[a-z0-9_]+)\s*\(", header))
        assert declared == set(names), header_name
        for name in declared:
            assert getattr(L, name) is not None


def test_status_strings(L):
    seen = {B.laplex_status_string(s) for s in range(0, -9, -1)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert B.laplex_status_string(-99) == "unknown status"
    assert B.laplex_last_hip_error() == ""


def ws_bytes(L, k, n, batch):
    out = ctypes.c_size_t(0)
    rc = L.laplex_workspace_bytes(k, n, batch, ctypes.byref(out))
    return rc, out.value


def test_workspace_bytes(L):
    assert L.laplex_workspace_bytes(1, 1, 1, None) == B.LAPLEX_ERR_NULL
    assert ws_bytes(L, -1, 1, 1)[0] == B.LAPLEX_ERR_SIZE
    assert ws_bytes(L, 1, -1, 1)[0] == B.LAPLEX_ERR_SIZE
    assert ws_bytes(L, 1, 1, -1)[0] == B.LAPLEX_ERR_SIZE
    assert ws_bytes(L, 1 << 31, 1 << 31, 1)[0] == B.LAPLEX_ERR_SIZE       # k + n = 2^32
    rc, top = ws_bytes(L, (1 << 31) - 1, (1 << 31) - 1, 1)                 # the largest merged length
    assert rc == 0 and top > 12 * ((1 << 32) - 2)
    sizes = [ws_bytes(L, 1024, n, 256)[1] for n in (1 << 10, 1 << 16, 1 << 20)]
    assert sizes == sorted(sizes) and sizes[0] > 0
    assert ws_bytes(L, 4096, 4096, 1)[1] % 256 == 0
    # plan (ids + decays) alone is 8 bytes per merged position
    assert ws_bytes(L, 1 << 20, 1 << 20, 1)[1] >= 8 * (1 << 21)
    assert ws_bytes(L, 0, 0, 0)[0] == 0


def apply_args(k=8, n=8, batch=4, a=FAKE, b=FAKE, x=FAKE, ldx=None, y=FAKE, ldy=None,
               ws=FAKE, wsb=1 << 40, flags=0):
    return (a, k, b, n, x, batch if ldx is None else ldx, batch, y, batch if ldy is None else ldy,
            ws, wsb, flags, None)


def test_apply_rejects_bad_arguments_before_touching_the_gpu(L):
    f = L.laplex_apply
    assert f(*apply_args(a=None)) == B.LAPLEX_ERR_NULL
    assert f(*apply_args(b=None)) == B.LAPLEX_ERR_NULL
    assert f(*apply_args(x=None)) == B.LAPLEX_ERR_NULL
    assert f(*apply_args(y=None)) == B.LAPLEX_ERR_NULL
    assert f(*apply_args(ws=None)) == B.LAPLEX_ERR_NULL
    assert f(*apply_args(k=-1)) == B.LAPLEX_ERR_SIZE
    assert f(*apply_args(n=-2)) == B.LAPLEX_ERR_SIZE
    assert f(*apply_args(batch=-1)) == B.LAPLEX_ERR_SIZE
    assert f(*apply_args(k=1 << 31, n=1 << 31)) == B.LAPLEX_ERR_SIZE
    assert f(*apply_args(ldx=3)) == B.LAPLEX_ERR_LD
    assert f(*apply_args(ldy=0)) == B.LAPLEX_ERR_LD
    assert f(*apply_args(flags=16)) == B.LAPLEX_ERR_FLAGS
    assert f(*apply_args(flags=1 << 31)) == B.LAPLEX_ERR_FLAGS
    assert f(*apply_args(a=FAKE + 2)) == B.LAPLEX_ERR_ALIGN
    assert f(*apply_args(ws=FAKE + 64)) == B.LAPLEX_ERR_ALIGN
    need = ws_bytes(L, 8, 8, 4)[1]
    assert f(*apply_args(wsb=need - 1)) == B.LAPLEX_ERR_WORKSPACE
    assert f(*apply_args(wsb=0)) == B.LAPLEX_ERR_WORKSPACE
    # nothing to do: success without any launch (pointers are never looked at)
    assert f(*apply_args(k=0, a=None, y=None, ws=None, wsb=0)) == B.LAPLEX_OK
    assert f(*apply_args(batch=0, x=None, y=None, ws=None, wsb=0)) == B.LAPLEX_OK


def bwd_args(k=8, n=8, batch=4, a=FAKE, b=FAKE, x=FAKE, gy=FAKE, gx=FAKE, ga=FAKE, gb=FAKE,
             ldx=None, ldgy=None, ldgx=None, ws=FAKE, wsb=1 << 40, flags=0):
    ld = lambda v: batch if v is None else v
    return (a, k, b, n, x, ld(ldx), gy, ld(ldgy), batch, gx, ld(ldgx), ga, gb, ws, wsb, flags, None)


def test_apply_backward_rejects_bad_arguments(L):
    f = L.laplex_apply_backward
    assert f(*bwd_args(gy=None)) == B.LAPLEX_ERR_NULL
    assert f(*bwd_args(x=None)) == B.LAPLEX_ERR_NULL              # ga / gb wanted: x is needed
    assert f(*bwd_args(x=None, ga=None, gb=None, ws=None)) == B.LAPLEX_ERR_NULL   # ... then only ws is missing
    assert f(*bwd_args(ldgy=1)) == B.LAPLEX_ERR_LD
    assert f(*bwd_args(ldgx=2)) == B.LAPLEX_ERR_LD
    assert f(*bwd_args(flags=32)) == B.LAPLEX_ERR_FLAGS
    assert f(*bwd_args(ga=FAKE + 1)) == B.LAPLEX_ERR_ALIGN
    assert f(*bwd_args(wsb=100)) == B.LAPLEX_ERR_WORKSPACE
    assert f(*bwd_args(n=-1)) == B.LAPLEX_ERR_SIZE


def test_gram_rejects_bad_arguments(L):
    g = L.laplex_gram
    ok = dict(a=FAKE, n=8, x=FAKE, ldx=4, batch=4, y=FAKE, ldy=4, ws=FAKE, wsb=1 << 40, flags=0)
    call = lambda **kw: g(*[{**ok, **kw}[key] for key in ("a", "n", "x", "ldx", "batch", "y", "ldy", "ws", "wsb", "flags")], None)
    assert call(a=None) == B.LAPLEX_ERR_NULL
    assert call(flags=B.LAPLEX_B_SORTED) == B.LAPLEX_ERR_FLAGS       # there is no b
    assert call(ldy=3) == B.LAPLEX_ERR_LD
    assert call(n=-1) == B.LAPLEX_ERR_SIZE
    assert call(wsb=8) == B.LAPLEX_ERR_WORKSPACE
    assert call(n=0, a=None, x=None, y=None, ws=None, wsb=0) == B.LAPLEX_OK
    gb = L.laplex_gram_backward
    assert gb(FAKE, 8, FAKE, 4, None, 4, 4, FAKE, 4, FAKE, FAKE, 1 << 40, 0, None) == B.LAPLEX_ERR_NULL
    assert gb(FAKE, 8, None, 4, FAKE, 4, 4, FAKE, 4, FAKE, FAKE, 1 << 40, 0, None) == B.LAPLEX_ERR_NULL
    assert gb(FAKE, 8, FAKE, 4, FAKE, 4, 4, FAKE, 4, FAKE, FAKE, 1 << 40, B.LAPLEX_B_SORTED, None) == B.LAPLEX_ERR_FLAGS


def test_get_perm_rejects_bad_arguments(L):
    f = L.laplex_get_perm
    assert f(None, 100, 4, FAKE, None) == B.LAPLEX_ERR_NULL
    assert f(FAKE, 100, 4, None, None) == B.LAPLEX_ERR_NULL
    assert f(FAKE, 100, -1, FAKE, None) == B.LAPLEX_ERR_SIZE
    assert f(FAKE, 15, 4, FAKE, None) == B.LAPLEX_ERR_WORKSPACE
    assert f(FAKE, 0, 0, None, None) == B.LAPLEX_OK


def test_get_plan_status_rejects_bad_arguments(L):
    f = L.laplex_get_plan_status
    assert f(FAKE, 1 << 40, -1, FAKE, None) == B.LAPLEX_ERR_SIZE
    assert f(FAKE, 1 << 40, 100000, None, None) == B.LAPLEX_ERR_NULL
    assert f(None, 1 << 40, 100000, FAKE, None) == B.LAPLEX_ERR_NULL
    assert f(FAKE, 1000, 100000, FAKE, None) == B.LAPLEX_ERR_WORKSPACE


def test_set_plan_status_rejects_bad_arguments(L):
    f = L.laplex_diag_set_plan_status
    assert f(FAKE, 1 << 40, 100, 1, None) == B.LAPLEX_ERR_SIZE            # plans sorted by counting have no status word
    assert f(None, 1 << 40, 100000, 1, None) == B.LAPLEX_ERR_NULL
    assert f(FAKE + 64, 1 << 40, 100000, 1, None) == B.LAPLEX_ERR_ALIGN
    assert f(FAKE, 1000, 100000, 1, None) == B.LAPLEX_ERR_WORKSPACE


def test_apply_static_rejects_bad_arguments_before_touching_the_gpu(L):
    """The entry point without a workspace argument: every argument error, and a problem larger than the
    library's own array, is reported on the host (no device is looked at)."""
    f = L.laplex_apply_static

    def args(k=8, n=8, batch=4, a=FAKE, b=FAKE, x=FAKE, y=FAKE, ldx=None, ldy=None, flags=0):
        return (a, k, b, n, x, batch if ldx is None else ldx, batch, y, batch if ldy is None else ldy, flags, None)

    assert f(*args(a=None)) == B.LAPLEX_ERR_NULL
    assert f(*args(x=None)) == B.LAPLEX_ERR_NULL
    assert f(*args(y=None)) == B.LAPLEX_ERR_NULL
    assert f(*args(k=-1)) == B.LAPLEX_ERR_SIZE
    assert f(*args(ldx=3)) == B.LAPLEX_ERR_LD
    assert f(*args(a=FAKE + 2)) == B.LAPLEX_ERR_ALIGN
    assert f(*args(flags=B.LAPLEX_REUSE_PLAN)) == B.LAPLEX_ERR_FLAGS     # no plan is handed from call to call
    assert f(*args(flags=B.LAPLEX_SAVE_SCANS)) == B.LAPLEX_ERR_FLAGS
    assert f(*args(flags=64)) == B.LAPLEX_ERR_FLAGS
    # the size limit follows laplex_workspace_bytes: the first problem that does not fit is rejected
    assert ws_bytes(L, 1000, 100000, 8)[1] <= B.LAPLEX_STATIC_WORKSPACE_BYTES
    assert ws_bytes(L, 1000, 4000000, 8)[1] > B.LAPLEX_STATIC_WORKSPACE_BYTES
    assert f(*args(k=1000, n=4000000, batch=8)) == B.LAPLEX_ERR_WORKSPACE
    assert f(*args(k=0, a=None, y=None)) == B.LAPLEX_OK
    assert f(*args(batch=0, x=None, y=None)) == B.LAPLEX_OK
    header = open(os.path.join(ROOT, "include", "laplex.h")).read()
    assert re.search(r"#define LAPLEX_STATIC_WORKSPACE_BYTES (\d+)ULL", header).group(1) == str(B.LAPLEX_STATIC_WORKSPACE_BYTES)


def test_diag_move_rows_rejects_bad_arguments(L):
    f = L.laplex_diag_move_rows
    assert f(FAKE, FAKE, FAKE, -1, 256, None) == B.LAPLEX_ERR_SIZE
    assert f(FAKE, FAKE, FAKE, 10, 255, None) == B.LAPLEX_ERR_SIZE
    assert f(None, FAKE, FAKE, 10, 256, None) == B.LAPLEX_ERR_NULL
    assert f(FAKE, FAKE, None, 10, 256, None) == B.LAPLEX_ERR_NULL
    assert f(FAKE + 4, FAKE, FAKE, 10, 256, None) == B.LAPLEX_ERR_ALIGN
    assert f(FAKE, FAKE, FAKE, 0, 256, None) == B.LAPLEX_OK


def test_binding_raises_with_status(L):
    with pytest.raises(B.LaplexError) as e:
        B.laplex_workspace_bytes(-1, 0, 0)
    assert e.value.status == B.LAPLEX_ERR_SIZE


def test_oracle_is_not_reachable_from_the_product():
    """The product package must not import, load or link the oracle."""
    pkg = os.path.join(ROOT, "paper_2605_24584_amd")
    pat = re.compile(r"import\s+oracle|from\s+oracle|laplex_oracle|oracle/")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                assert not pat.search(open(os.path.join(dirpath, fn)).read()), fn


# ------------------------------------------------------------------ phased entry points

def phased_ws(L, k, n, batch):
    out = ctypes.c_size_t(0)
    rc = L.laplex_phased_workspace_bytes(k, n, batch, ctypes.byref(out))
    return rc, out.value


def test_phased_workspace_and_argument_checks(L):
    assert L.laplex_phased_workspace_bytes(1, 1, 1, None) == B.LAPLEX_ERR_NULL
    assert phased_ws(L, 1, 1, -1)[0] == B.LAPLEX_ERR_SIZE
    rc, size = phased_ws(L, 64, 4096, 8)
    plain = ctypes.c_size_t(0)
    assert L.laplex_workspace_bytes(64, 4096, 16, ctypes.byref(plain)) == 0
    # the plain workspace of the doubled batch plus the halves of x, gx (n rows) and y, gy (k rows)
    assert rc == 0 and size % 256 == 0 and size >= plain.value + 4 * 16 * (2 * 4096 + 2 * 64)
    k, n, batch = 8, 8, 4
    good = [FAKE, FAKE, k, FAKE, FAKE, n, FAKE, batch, batch, FAKE, batch, FAKE, size, 0, None]
    def call(**kw):
        args = list(good)
        for i, v in kw.items():
            args[int(i[1:])] = v
        return L.laplex_phased_apply(*args)
    assert call(_1=None) == B.LAPLEX_ERR_NULL           # phi
    assert call(_4=None) == B.LAPLEX_ERR_NULL           # psi
    assert call(_6=None) == B.LAPLEX_ERR_NULL           # x
    assert call(_7=batch - 1) == B.LAPLEX_ERR_LD
    assert call(_11=None) == B.LAPLEX_ERR_NULL          # workspace
    assert call(_12=16) == B.LAPLEX_ERR_WORKSPACE
    assert call(_13=1 << 20) == B.LAPLEX_ERR_FLAGS
    assert call(_3=FAKE + 2) == B.LAPLEX_ERR_ALIGN
    assert call(_2=0) == B.LAPLEX_OK                     # k == 0: nothing to do, nothing touched
    # backward: x may be missing only if gx alone is wanted
    bgood = [FAKE, FAKE, k, FAKE, FAKE, n, None, batch, FAKE, batch, batch,
             FAKE, batch, None, None, None, FAKE, FAKE, size, 0, None]
    assert L.laplex_phased_apply_backward(*bgood) == B.LAPLEX_ERR_NULL      # gpsi wanted, x missing
    bgood[8] = None; bgood[6] = FAKE
    assert L.laplex_phased_apply_backward(*bgood) == B.LAPLEX_ERR_NULL      # gy missing


# ------------------------------------------------------------------ temperature entry points

def test_temperature_calls_reject_bad_tau_and_bad_arguments(L):
    F = ctypes.c_float
    k = n = 8; batch = 4
    fwd = lambda tau, **kw: L.laplex_apply_tau(*(lambda t: t[:4] + (F(tau),) + t[4:])(apply_args(**kw)))
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        assert fwd(bad) == B.LAPLEX_ERR_VALUE
    assert fwd(2.0, x=None) == B.LAPLEX_ERR_NULL
    assert fwd(2.0, ldx=3) == B.LAPLEX_ERR_LD
    assert fwd(2.0, wsb=0) == B.LAPLEX_ERR_WORKSPACE
    assert fwd(0.5, k=0, a=None, y=None, ws=None, wsb=0) == B.LAPLEX_OK
    bwd = L.laplex_apply_backward_tau
    args = lambda tau, ga=FAKE, gb=FAKE, gtau=FAKE: (FAKE, k, FAKE, n, F(tau), FAKE, batch, FAKE, batch, batch,
                                                     FAKE, batch, ga, gb, gtau, FAKE, 1 << 40, 0, None)
    assert bwd(*args(0.0)) == B.LAPLEX_ERR_VALUE
    assert bwd(*args(1.5, ga=None)) == B.LAPLEX_ERR_NULL          # gtau is formed from ga and gb
    assert bwd(*args(1.5, gb=None)) == B.LAPLEX_ERR_NULL
    assert bwd(*args(1.5, gtau=FAKE + 2)) == B.LAPLEX_ERR_ALIGN
    g = L.laplex_gram_tau
    assert g(FAKE, n, F(-2.0), FAKE, batch, batch, FAKE, batch, FAKE, 1 << 40, 0, None) == B.LAPLEX_ERR_VALUE
    assert g(None, n, F(2.0), FAKE, batch, batch, FAKE, batch, FAKE, 1 << 40, 0, None) == B.LAPLEX_ERR_NULL
    gb_ = L.laplex_gram_backward_tau
    assert gb_(FAKE, n, F(float("nan")), FAKE, batch, FAKE, batch, batch, FAKE, batch, FAKE, FAKE, FAKE, 1 << 40, 0, None) == B.LAPLEX_ERR_VALUE
    assert gb_(FAKE, n, F(2.0), FAKE, batch, FAKE, batch, batch, FAKE, batch, None, FAKE, FAKE, 1 << 40, 0, None) == B.LAPLEX_ERR_NULL


# ------------------------------------------------------------------ weighted Gram matrix

def test_weighted_gram_argument_checks(L):
    out = ctypes.c_size_t(0)
    assert L.laplex_wgram_workspace_bytes(8, 8, None) == B.LAPLEX_ERR_NULL
    assert L.laplex_wgram_workspace_bytes(-1, 8, ctypes.byref(out)) == B.LAPLEX_ERR_SIZE
    assert L.laplex_wgram_workspace_bytes((1 << 20) + 1, 8, ctypes.byref(out)) == B.LAPLEX_ERR_SIZE
    assert L.laplex_wgram_workspace_bytes(1024, 1 << 20, ctypes.byref(out)) == 0
    # at least the plan (12 B per merged position) and the sort's buffers (12 B more), + U, V, W (24 B) per anchor
    assert out.value % 256 == 0 and out.value >= 24 * ((1 << 20) + 1024) + 24 * 1024
    k, n = 8, 16
    good = dict(a=FAKE, k=k, b=FAKE, n=n, d=FAKE, m=FAKE, ldm=k, ws=FAKE, wsb=1 << 40, flags=0)
    call = lambda **kw: L.laplex_wgram(*[{**good, **kw}[key] for key in
                                         ("a", "k", "b", "n", "d", "m", "ldm", "ws", "wsb", "flags")], None)
    assert call(a=None) == B.LAPLEX_ERR_NULL
    assert call(b=None) == B.LAPLEX_ERR_NULL
    assert call(d=None) == B.LAPLEX_ERR_NULL
    assert call(m=None) == B.LAPLEX_ERR_NULL
    assert call(ws=None) == B.LAPLEX_ERR_NULL
    assert call(ldm=k - 1) == B.LAPLEX_ERR_LD
    assert call(k=-1) == B.LAPLEX_ERR_SIZE
    assert call(flags=B.LAPLEX_SAVE_SCANS) == B.LAPLEX_ERR_FLAGS
    assert call(wsb=64) == B.LAPLEX_ERR_WORKSPACE
    assert call(d=FAKE + 2) == B.LAPLEX_ERR_ALIGN
    assert call(k=0, a=None, m=None, ws=None, wsb=0) == B.LAPLEX_OK


# ------------------------------------------------------------------ LAPLEX^(r)

def test_mix_argument_checks(L):
    out = ctypes.c_size_t(0)
    assert L.laplex_mix_workspace_bytes(2, 8, 8, 4, None) == B.LAPLEX_ERR_NULL
    assert L.laplex_mix_workspace_bytes(-1, 8, 8, 4, ctypes.byref(out)) == B.LAPLEX_ERR_SIZE
    assert L.laplex_mix_workspace_bytes(4097, 8, 8, 4, ctypes.byref(out)) == B.LAPLEX_ERR_SIZE
    assert L.laplex_mix_workspace_bytes(3, 64, 4096, 8, ctypes.byref(out)) == 0
    plain = ctypes.c_size_t(0)
    assert L.laplex_workspace_bytes(64, 4096, 8, ctypes.byref(plain)) == 0
    assert out.value % 256 == 0 and out.value >= 3 * plain.value + 4 * 8 * (3 * 64 + 64 + 4096)
    r, k, n, batch = 2, 8, 8, 4
    good = [FAKE, FAKE, FAKE, r, k, n, FAKE, batch, batch, FAKE, batch, FAKE, 1 << 40, 0, None]
    def call(**kw):
        args = list(good)
        for i, v in kw.items():
            args[int(i[1:])] = v
        return L.laplex_mix_apply(*args)
    assert call(_0=None) == B.LAPLEX_ERR_NULL            # a
    assert call(_2=None) == B.LAPLEX_ERR_NULL            # w
    assert call(_6=None) == B.LAPLEX_ERR_NULL            # x
    assert call(_7=batch - 1) == B.LAPLEX_ERR_LD
    assert call(_11=None) == B.LAPLEX_ERR_NULL           # workspace
    assert call(_12=64) == B.LAPLEX_ERR_WORKSPACE
    assert call(_13=1 << 9) == B.LAPLEX_ERR_FLAGS
    assert call(_3=-1) == B.LAPLEX_ERR_SIZE
    assert call(_4=0, _9=None, _11=None, _12=0) == B.LAPLEX_OK        # k == 0: nothing to do
    bgood = [FAKE, FAKE, FAKE, r, k, n, None, batch, FAKE, batch, batch, FAKE, batch, None, None, FAKE,
             FAKE, 1 << 40, 0, None]
    assert L.laplex_mix_apply_backward(*bgood) == B.LAPLEX_ERR_NULL                 # gw wanted, x missing
    bgood[6] = FAKE; bgood[8] = None
    assert L.laplex_mix_apply_backward(*bgood) == B.LAPLEX_ERR_NULL                 # gy missing


def test_weighted_gram_fp64_argument_checks(L):
    out = ctypes.c_size_t(0)
    assert L.laplex_wgram_f64_workspace_bytes(8, 8, None) == B.LAPLEX_ERR_NULL
    assert L.laplex_wgram_f64_workspace_bytes(1024, 1 << 20, ctypes.byref(out)) == 0 and out.value % 256 == 0
    k, n = 8, 16
    good = dict(a=FAKE, k=k, b=FAKE, n=n, d=FAKE, m=FAKE, ldm=k, ws=FAKE, wsb=1 << 40, flags=0)
    call = lambda **kw: L.laplex_wgram_f64(*[{**good, **kw}[key] for key in
                                             ("a", "k", "b", "n", "d", "m", "ldm", "ws", "wsb", "flags")], None)
    assert call(d=None) == B.LAPLEX_ERR_NULL
    assert call(m=None) == B.LAPLEX_ERR_NULL
    assert call(d=FAKE + 4) == B.LAPLEX_ERR_ALIGN          # doubles: 8-byte alignment
    assert call(m=FAKE + 4) == B.LAPLEX_ERR_ALIGN
    assert call(ldm=k - 1) == B.LAPLEX_ERR_LD
    assert call(flags=B.LAPLEX_SAVE_SCANS) == B.LAPLEX_ERR_FLAGS
    assert call(wsb=64) == B.LAPLEX_ERR_WORKSPACE
    assert call(k=0, a=None, m=None, ws=None, wsb=0) == B.LAPLEX_OK
