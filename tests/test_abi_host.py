"""Host-only checks of the C ABI: the library loads, exports every symbol include/sa.h declares, and
reports argument errors before anything is launched (no GPU needed, no kernel is run)."""
import ctypes as C
import os
import re

import pytest

from paper_2604_00754_amd import binding as sa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = C.c_void_p(4096)  # never dereferenced: every call below must fail validation first


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:sa|swa|gated)_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert set(names) == set(sa.EXPORTS), names
    lib = sa.raw()
    for name in names:
        assert getattr(lib, name) is not None


def test_status_strings():
    for code in range(8):
        assert sa.status_string(code) and sa.status_string(code) != "unknown status"
    assert sa.status_string(99) == "unknown status"


def good():
    return sa.make_desc(2, 8, 2, 1000, 128, 256, sa.SA_WIN_SYM_CIRCULAR, 1, sa.SA_BF16, 0.0, 1, 1)


def fwd(desc, q=FAKE, k=FAKE, v=FAKE, y=FAKE):
    d = C.byref(desc) if desc is not None else None
    return sa.raw().sa_fwd(d, q, k, v, None, y, None, None, 0, None)


def test_null_arguments():
    assert fwd(None) == sa.SA_ERR_NULL
    for kw in ("q", "k", "v", "y"):
        assert fwd(good(), **{kw: None}) == sa.SA_ERR_NULL
    d = good()
    assert sa.raw().sa_check_perm(C.byref(d), None, FAKE, 1 << 30, None) == sa.SA_ERR_NULL


@pytest.mark.parametrize("field,value,status", [
    ("B", 0, sa.SA_ERR_SHAPE), ("n", 0, sa.SA_ERR_SHAPE), ("w", 0, sa.SA_ERR_SHAPE),
    ("Hkv", 3, sa.SA_ERR_SHAPE), ("window", 3, sa.SA_ERR_SHAPE), ("window", -1, sa.SA_ERR_SHAPE),
    ("perm_B", 3, sa.SA_ERR_SHAPE), ("perm_H", 2, sa.SA_ERR_SHAPE), ("causal_orig", 2, sa.SA_ERR_SHAPE),
    ("gate_per_dim", 2, sa.SA_ERR_SHAPE), ("scale", float("nan"), sa.SA_ERR_SHAPE),
    ("d", 96, sa.SA_ERR_UNSUPPORTED), ("d", 256, sa.SA_ERR_UNSUPPORTED), ("dtype", 2, sa.SA_ERR_UNSUPPORTED),
    ("gate_dtype", 5, sa.SA_ERR_UNSUPPORTED),
])
def test_bad_descriptors(field, value, status):
    d = good()
    setattr(d, field, value)
    assert fwd(d) == status
    assert sa.sa_workspace_bytes(d, sa.SA_OP_BWD) == 0


def test_workspace_sizes_and_checks():
    d = good()
    rows = d.B * d.Hq * d.n
    assert sa.sa_workspace_bytes(d, sa.SA_OP_FWD) == 0
    assert sa.sa_workspace_bytes(d, sa.SA_OP_GATED_FWD) >= rows * d.d * 2   # the first branch as a bf16 tensor
    f32 = good()
    f32.dtype = sa.SA_F32
    assert sa.sa_workspace_bytes(f32, sa.SA_OP_GATED_FWD) == 0
    ws_bwd = sa.sa_workspace_bytes(d, sa.SA_OP_BWD)
    ws_gated = sa.sa_workspace_bytes(d, sa.SA_OP_GATED_BWD)
    assert ws_bwd >= rows * 4 and ws_bwd % 256 == 0
    assert ws_gated >= 2 * rows * 4 + 2 * rows * d.d * 2
    assert sa.sa_workspace_bytes(d, sa.SA_OP_CHECK_PERM) >= d.n * 4 + 4
    lib = sa.raw()
    args = [C.byref(d), None] + [FAKE] * 17
    # ungated backward: workspace too small / missing
    assert lib.sa_bwd(*args, ws_bwd - 1, None) == sa.SA_ERR_WORKSPACE
    args_nows = list(args)
    args_nows[18] = None
    assert lib.sa_bwd(*args_nows, ws_bwd, None) == sa.SA_ERR_WORKSPACE
    # gated backward needs the larger workspace and all gate pointers
    swa = good()
    swa.window = sa.SA_WIN_ONE_SIDED
    gargs = [C.byref(d), C.byref(swa)] + [FAKE] * 17
    assert lib.sa_bwd(*gargs, ws_bwd, None) == sa.SA_ERR_WORKSPACE
    gargs_null = list(gargs)
    gargs_null[6] = None  # gate_sa
    assert lib.sa_bwd(*gargs_null, ws_gated, None) == sa.SA_ERR_NULL
    assert lib.sa_check_perm(C.byref(d), FAKE, FAKE, 16, None) == sa.SA_ERR_WORKSPACE


def test_gated_descriptors_must_agree():
    a, b = good(), good()
    b.window = sa.SA_WIN_ONE_SIDED
    lib = sa.raw()
    call = lambda x, y: lib.gated_sa_swa_fwd(C.byref(x), C.byref(y), FAKE, FAKE, FAKE, None, FAKE, FAKE,
                                             FAKE, None, None, None, None, None, 0, None)
    b.n = 999
    assert call(a, b) == sa.SA_ERR_SHAPE
    b.n = a.n
    b.dtype = sa.SA_F32
    assert call(a, b) == sa.SA_ERR_SHAPE
    b.dtype = a.dtype
    assert call(a, b) == sa.SA_ERR_WORKSPACE
    assert lib.gated_sa_swa_fwd(C.byref(a), C.byref(b), FAKE, FAKE, FAKE, None, None, FAKE, FAKE, None,
                                None, None, None, None, 0, None) == sa.SA_ERR_NULL


def test_binding_raises_with_status():
    d = good()
    d.d = 96
    with pytest.raises(sa.SaError) as e:
        sa._check(fwd(d), "sa_fwd")
    assert e.value.status == sa.SA_ERR_UNSUPPORTED


def test_decode_step_arguments():
    """sa_decode_fwd reports bad lengths, missing pointers and a short workspace before any launch."""
    d = good()
    lib = sa.raw()
    need = sa.sa_workspace_bytes(d, sa.SA_OP_DECODE)
    # one partial result of d + 2 floats per (b, hq) and chunk of the cache; chunks hold at most 1024 rows
    assert need >= 2 * 8 * (128 + 2) * 4 and need % 256 == 0

    def call(length=1000, q=FAKE, k=FAKE, v=FAKE, y=FAKE, ws=FAKE, ws_bytes=need):
        return lib.sa_decode_fwd(C.byref(d), q, k, v, length, y, None, ws, ws_bytes, None)

    for bad in (0, -1, 1001):
        assert call(length=bad) == sa.SA_ERR_SHAPE
    for kw in ("q", "k", "v", "y"):
        assert call(**{kw: None}) == sa.SA_ERR_NULL
    assert call(ws=None) == sa.SA_ERR_WORKSPACE
    assert call(ws_bytes=need - 1) == sa.SA_ERR_WORKSPACE
    assert lib.sa_decode_fwd(None, FAKE, FAKE, FAKE, 1, FAKE, None, FAKE, need, None) == sa.SA_ERR_NULL
    # the per-sequence form takes the same checks, and needs its length array
    assert lib.sa_decode_fwd_varlen(C.byref(d), FAKE, FAKE, FAKE, None, 1000, FAKE, None, FAKE, need, None) == sa.SA_ERR_NULL
    assert lib.sa_decode_fwd_varlen(C.byref(d), FAKE, FAKE, FAKE, FAKE, 1001, FAKE, None, FAKE, need, None) == sa.SA_ERR_SHAPE
    assert lib.sa_decode_fwd_varlen(C.byref(d), FAKE, FAKE, FAKE, FAKE, 1000, FAKE, None, FAKE, need - 1, None) == sa.SA_ERR_WORKSPACE
    # more (b, hq) pairs than one launch dimension holds
    wide = sa.make_desc(2048, 64, 64, 16, 64, 2)
    assert lib.sa_decode_fwd(C.byref(wide), FAKE, FAKE, FAKE, 16, FAKE, None, FAKE, 1 << 40, None) == sa.SA_ERR_UNSUPPORTED
    # the workspace is sized by the capacity: it never grows when the descriptor's n shrinks
    small = sa.make_desc(2, 8, 2, 500, 128, 256)
    assert sa.sa_workspace_bytes(small, sa.SA_OP_DECODE) <= need


def test_misaligned_pointers_are_refused_before_any_launch():
    """Tensors are accessed 16 bytes at a time: an address off that grid is reported, not launched."""
    d = good()
    lib = sa.raw()
    odd = C.c_void_p(4096 + 8)     # 8-byte aligned only
    for kw in ("q", "k", "v", "y"):
        assert fwd(d, **{kw: odd}) == sa.SA_ERR_UNSUPPORTED
    # perm and LSE need their element's alignment
    assert lib.sa_fwd(C.byref(d), FAKE, FAKE, FAKE, C.c_void_p(4098), FAKE, None, None, 0, None) == sa.SA_ERR_UNSUPPORTED
    assert lib.sa_fwd(C.byref(d), FAKE, FAKE, FAKE, None, FAKE, C.c_void_p(4098), None, 0, None) == sa.SA_ERR_UNSUPPORTED
    need = sa.sa_workspace_bytes(d, sa.SA_OP_DECODE)
    assert lib.sa_decode_fwd(C.byref(d), FAKE, odd, FAKE, 10, FAKE, None, FAKE, need, None) == sa.SA_ERR_UNSUPPORTED
    assert lib.sa_decode_fwd(C.byref(d), FAKE, FAKE, FAKE, 10, FAKE, None, odd, need, None) == sa.SA_ERR_UNSUPPORTED
    nb = sa.sa_workspace_bytes(d, sa.SA_OP_BWD)
    args = [FAKE] * 17
    args[13] = odd                 # dV
    assert lib.sa_bwd(C.byref(d), None, *args, nb, None) == sa.SA_ERR_UNSUPPORTED


def test_row_count_must_fit_32_bits():
    """B * Hq * n rows are counted in 32-bit integers inside the library: more is a shape error, not a launch."""
    ok = sa.make_desc(16, 64, 8, 1 << 20, 128, 512)          # 2^30 rows
    assert sa.sa_workspace_bytes(ok, sa.SA_OP_BWD) > 0
    big = sa.make_desc(64, 64, 8, 1 << 20, 128, 512)         # 2^32 rows
    assert fwd(big) == sa.SA_ERR_SHAPE
    assert sa.sa_workspace_bytes(big, sa.SA_OP_BWD) == 0


def test_one_head_must_span_less_than_2_gib_in_bf16():
    """The bf16 kernels form 32-bit byte offsets inside a head: n * d * 2 >= 2^31 is refused on the host, by the
    forward and by the backward alike (the fp32 path has no such limit)."""
    lib = sa.raw()
    big = sa.make_desc(1, 1, 1, 1 << 23, 128, 512)           # 2^23 rows of 256 bytes = 2 GiB
    assert fwd(big) == sa.SA_ERR_UNSUPPORTED
    nb = sa.sa_workspace_bytes(big, sa.SA_OP_BWD)
    assert nb > 0
    assert lib.sa_bwd(C.byref(big), None, *([FAKE] * 17), nb, None) == sa.SA_ERR_UNSUPPORTED
    ok = sa.make_desc(1, 1, 1, (1 << 23) - 1, 128, 512)
    assert lib.sa_bwd(C.byref(ok), None, *([FAKE] * 17), nb - 1024, None) == sa.SA_ERR_WORKSPACE   # passes the size check


def test_static_decode_refuses_what_its_buffer_cannot_hold():
    """sa_decode_fwd_static judges the size on the host, before it touches the device."""
    lib = sa.raw()
    fits = sa.make_desc(1, 32, 4, 131072, 128, 1024)
    assert 0 < sa.sa_workspace_bytes(fits, sa.SA_OP_DECODE) <= sa.SA_STATIC_SCRATCH_BYTES
    big = sa.make_desc(16, 32, 8, 131072, 128, 1024)
    assert sa.sa_workspace_bytes(big, sa.SA_OP_DECODE) > sa.SA_STATIC_SCRATCH_BYTES
    assert lib.sa_decode_fwd_static(C.byref(big), FAKE, FAKE, FAKE, 16, FAKE, None, None) == sa.SA_ERR_STATIC_LIMIT
    assert sa.status_string(sa.SA_ERR_STATIC_LIMIT).startswith("request needs more scratch")
    assert lib.sa_decode_fwd_static(C.byref(fits), None, FAKE, FAKE, 16, FAKE, None, None) == sa.SA_ERR_NULL
    assert lib.sa_decode_fwd_static(C.byref(fits), FAKE, FAKE, FAKE, 0, FAKE, None, None) == sa.SA_ERR_SHAPE
    assert lib.sa_decode_fwd_static(None, FAKE, FAKE, FAKE, 1, FAKE, None, None) == sa.SA_ERR_NULL


def test_bwd_rope_arguments():
    """sa_bwd_rope validates on the host: nulls, flags, dtype, alignment, the 2 GiB head limit, the workspace
    (the plain backward's plus the rotated query rows)."""
    lib = sa.raw()
    d = good()
    need = sa.sa_workspace_bytes(d, sa.SA_OP_BWD_ROPE)
    assert need >= sa.sa_workspace_bytes(d, sa.SA_OP_BWD) + d.B * d.Hq * d.n * d.d * 2

    def call(desc=d, table=FAKE, inter=0, dku=0, dv=FAKE, ws=FAKE, nb=need):
        return lib.sa_bwd_rope(C.byref(desc), FAKE, FAKE, FAKE, None, table, inter, dku, FAKE, FAKE, FAKE, FAKE, FAKE,
                               dv, ws, nb, None)

    assert call(table=None) == sa.SA_ERR_NULL
    assert call(dv=None) == sa.SA_ERR_NULL
    assert call(inter=2) == sa.SA_ERR_SHAPE
    assert call(dku=-1) == sa.SA_ERR_SHAPE
    assert call(dv=C.c_void_p(4096 + 8)) == sa.SA_ERR_UNSUPPORTED
    assert call(table=C.c_void_p(4096 + 4)) == sa.SA_ERR_UNSUPPORTED
    assert call(ws=None) == sa.SA_ERR_WORKSPACE
    assert call(nb=need - 1) == sa.SA_ERR_WORKSPACE
    f32 = sa.make_desc(2, 8, 2, 1000, 128, 256, dtype=sa.SA_F32)
    assert call(desc=f32) == sa.SA_ERR_UNSUPPORTED
    big = sa.make_desc(1, 1, 1, 1 << 23, 128, 512)
    assert call(desc=big, nb=1 << 40) == sa.SA_ERR_UNSUPPORTED
