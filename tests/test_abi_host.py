"""Host-only checks of the C ABI: the library loads, exports every symbol that
include/ist.h declares, and rejects bad model descriptions without a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_1910_02120_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_1910_02120_amd import build
        build.build(verbose=False)
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "ist.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ist_[a-z_]+)\s*\(", hdr))
    assert {"ist_partition", "ist_subnet_steps", "ist_merge"} <= declared
    for name in declared:
        assert hasattr(lib, name), name
    from paper_1910_02120_amd import EXPORTS
    assert declared == set(EXPORTS)
    assert lib.ist_version().startswith(b"ist-gfx950")


def _create(lib, dims, S, dtype=0, inp=0, bias=1, max_B=8, t=None):
    from paper_1910_02120_amd.binding import _ModelDesc
    arr = (C.c_int64 * len(dims))(*dims)
    d = _ModelDesc(len(dims) - 1 if t is None else t, arr, S, dtype, inp, bias)
    ctx = C.c_void_p()
    st = lib.ist_create(C.byref(d), max_B, C.byref(ctx))
    return st, ctx


def test_create_validates_the_description(lib):
    st, ctx = _create(lib, [8, 16, 16, 4], 4)
    assert st == 0 and ctx.value
    n = C.c_size_t()
    assert lib.ist_subnets_bytes(ctx, C.byref(n)) == 0 and n.value > 0
    # weights of all subnets: 8*16 + 16*16/4 + 16*4 values of 4 bytes, plus tables and biases
    assert n.value >= 4 * (8 * 16 + 16 * 16 // 4 + 16 * 4)
    assert lib.ist_workspace_bytes(ctx, C.byref(n)) == 0 and n.value > 0
    r, c = C.c_int64(), C.c_int64()
    assert lib.ist_subnet_shape(ctx, 2, C.byref(r), C.byref(c)) == 0 and (r.value, c.value) == (4, 4)
    assert lib.ist_subnet_shape(ctx, 1, C.byref(r), C.byref(c)) == 0 and (r.value, c.value) == (4, 8)
    assert lib.ist_subnet_shape(ctx, 3, C.byref(r), C.byref(c)) == 0 and (r.value, c.value) == (4, 4)
    assert lib.ist_subnet_shape(ctx, 4, C.byref(r), C.byref(c)) == -1
    # state machine: nothing bound yet
    assert lib.ist_merge(ctx, None, None) == -6
    assert lib.ist_subnet_steps(ctx, None, C.c_float(0.1), 1, None, None) == -6
    assert b"partition" in lib.ist_last_error(ctx)
    assert lib.ist_destroy(ctx) == 0
    assert _create(lib, [8, 3, 4], 4)[0] == -2           # fewer hidden neurons than subnets
    st, ctx = _create(lib, [8, 10, 7, 4], 4)             # blocks of unequal width: 10 = 3 + 3 + 2 + 2, 7 = 2 + 2 + 2 + 1
    assert st == 0
    got = []
    for s_ in range(4):
        assert lib.ist_subnet_shape_of(ctx, s_, 2, C.byref(r), C.byref(c)) == 0
        got.append((r.value, c.value))
    assert got == [(2, 3), (2, 3), (2, 2), (1, 2)]
    assert lib.ist_subnet_shape(ctx, 2, C.byref(r), C.byref(c)) == 0 and (r.value, c.value) == (2, 3)
    assert lib.ist_subnet_shape_of(ctx, 4, 2, C.byref(r), C.byref(c)) == -1
    assert lib.ist_destroy(ctx) == 0
    assert _create(lib, [8, 16, 4], 0)[0] == -1          # S < 1
    assert _create(lib, [8, 4], 1)[0] == -1              # no hidden layer
    assert _create(lib, [8, 16, 4], 2, dtype=7)[0] == -1
    assert _create(lib, [8, 16, 4], 2, max_B=0)[0] == -2
    assert _create(lib, [8, 0, 4], 1)[0] == -2
    assert lib.ist_create(None, 1, None) == -1


def test_create_validates_the_normalisation_fields(lib):
    from paper_1910_02120_amd.binding import _ModelDesc
    dims = [8, 16, 16, 4]
    arr = (C.c_int64 * len(dims))(*dims)
    sizes = []
    for norm in (0, 1):
        ctx = C.c_void_p()
        d = _ModelDesc(3, arr, 4, 0, 0, 1, norm, 0.0)
        assert lib.ist_create(C.byref(d), 8, C.byref(ctx)) == 0
        n = C.c_size_t()
        assert lib.ist_workspace_bytes(ctx, C.byref(n)) == 0
        sizes.append(n.value)
        assert lib.ist_destroy(ctx) == 0
    assert sizes[1] > sizes[0]            # pre-activations, standardised values, 1/sigma per hidden layer
    ctx = C.c_void_p()
    assert lib.ist_create(C.byref(_ModelDesc(3, arr, 4, 0, 0, 1, 2, 0.0)), 8, C.byref(ctx)) == -1
    assert lib.ist_create(C.byref(_ModelDesc(3, arr, 4, 0, 0, 1, 1, float("nan"))), 8, C.byref(ctx)) == -1


def test_create_validates_the_layer_factors(lib):
    from paper_1910_02120_amd.binding import _ModelDesc
    dims = [8, 16, 16, 4]
    arr = (C.c_int64 * len(dims))(*dims)
    for vals, want in (((1.0, 16.0, 1.0), 0), ((1.0, 0.0, 1.0), -1), ((1.0, -4.0, 1.0), -1),
                       ((float("nan"), 1.0, 1.0), -1), ((1.0, 1.0, float("inf")), -1)):
        sc = (C.c_float * 3)(*vals)
        d = _ModelDesc(3, arr, 4, 0, 0, 1, 0, 0.0, sc)
        ctx = C.c_void_p()
        assert lib.ist_create(C.byref(d), 8, C.byref(ctx)) == want, vals
        if want == 0:
            assert lib.ist_destroy(ctx) == 0
