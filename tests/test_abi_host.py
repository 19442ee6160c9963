"""Host-side checks that need no GPU: the library loads, exports every symbol declared in
include/aser.h, and rejects bad arguments before any HIP call is made."""
import ctypes
import os
import re

import pytest

import paper_2411_07762_amd as aser

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 0x7F0000001000  # a fake, aligned "device address": validation must fail before it is touched


@pytest.fixture(scope="module")
def ctx():
    lib = aser.load_library()
    h = ctypes.c_void_p()
    assert lib.aser_create(ctypes.byref(h), 0, None) == aser.ASER_OK
    c = aser.Context.__new__(aser.Context)
    c._lib, c.handle, c.device, c._ws, c._ws_bytes = lib, h, 0, None, 0
    yield c
    c.close()


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "aser.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(aser_[a-z0-9_]+)\s*\(", text))
    assert {"aser_gram_accumulate", "aser_smooth_outliers", "aser_quantize_rtn", "aser_whiten",
            "aser_error_reconstruct"} <= declared
    lib = aser.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(aser.EXPORTS)


def test_status_strings():
    assert aser.status_string(aser.ASER_OK) == "ok"
    assert "positive definite" in aser.status_string(aser.ASER_ERR_NOT_SPD)
    assert aser.status_string(99) == "unknown status"


def test_create_rejects_bad_arguments():
    lib = aser.load_library()
    assert lib.aser_create(None, 0, None) == aser.ASER_ERR_INVALID_ARG
    h = ctypes.c_void_p()
    assert lib.aser_create(ctypes.byref(h), -1, None) == aser.ASER_ERR_INVALID_ARG
    assert lib.aser_destroy(None) == aser.ASER_ERR_INVALID_ARG


def test_workspace_rules(ctx):
    assert aser.aser_set_workspace(ctx, P + 8, 1024) == aser.ASER_ERR_INVALID_ARG      # not 256-byte aligned
    assert aser.aser_set_workspace(ctx, None, 0) == aser.ASER_OK
    need = aser.aser_workspace_bytes(4096, 4096, 64)
    assert need >= 2 * 4096 * 4096 * 4
    assert aser.aser_workspace_bytes(0, 16, 4) == 0
    # a call that needs scratch fails cleanly without one
    st = aser.aser_smooth_outliers(ctx, P, P, P, 4, P, P, m=16, n=16, ldw=16)
    assert st == aser.ASER_ERR_WORKSPACE
    st, _ = aser.aser_whiten(ctx, P, None, 0.0, P, n=64, ldg=64, lds=64)
    assert st == aser.ASER_ERR_WORKSPACE
    st, _, _ = aser.aser_error_reconstruct(ctx, P, P, 4, P, P, P, m=64, n=64, ldt=64, lds=64)
    assert st == aser.ASER_ERR_WORKSPACE
    assert "workspace" in ctx._lib.aser_last_error(ctx.handle).decode()


def test_precision_modes(ctx):
    lib = ctx._lib
    for mode in (aser.ASER_PRECISION_FAST, aser.ASER_PRECISION_EXACT, aser.ASER_PRECISION_AUTO):
        assert lib.aser_set_precision(ctx.handle, mode) == aser.ASER_OK
    assert lib.aser_set_precision(ctx.handle, 7) == aser.ASER_ERR_INVALID_ARG
    assert lib.aser_set_precision(None, 0) == aser.ASER_ERR_INVALID_ARG


def test_gram_validation(ctx):
    g = aser.aser_gram_accumulate
    assert g(ctx, None, P, rows=8, n=8, ldx=8, ldg=8, x_dtype=0) == aser.ASER_ERR_INVALID_ARG
    assert g(ctx, P, P, rows=8, n=8, ldx=4, ldg=8, x_dtype=0) == aser.ASER_ERR_SHAPE
    assert g(ctx, P, P, rows=8, n=8, ldx=8, ldg=7, x_dtype=0) == aser.ASER_ERR_SHAPE
    assert g(ctx, P, P, rows=-1, n=8, ldx=8, ldg=8, x_dtype=0) == aser.ASER_ERR_SHAPE
    assert g(ctx, P, P, rows=8, n=8, ldx=8, ldg=8, x_dtype=5) == aser.ASER_ERR_DTYPE
    assert g(ctx, P + 1, P, rows=8, n=8, ldx=8, ldg=8, x_dtype=0) == aser.ASER_ERR_INVALID_ARG
    assert g(ctx, P, P, P + 4, None, rows=8, n=8, ldx=8, ldg=8, x_dtype=0) == aser.ASER_ERR_INVALID_ARG
    assert g(ctx, P, P, rows=0, n=8, ldx=8, ldg=8, x_dtype=0) == aser.ASER_OK           # empty chunk: no-op


def test_smooth_validation(ctx):
    s = aser.aser_smooth_outliers
    assert s(ctx, P, P, P, 9, P, P, m=4, n=8, ldw=8) == aser.ASER_ERR_SHAPE              # f > n
    assert s(ctx, P, P, P, -1, P, P, m=4, n=8, ldw=8) == aser.ASER_ERR_SHAPE
    assert s(ctx, P, P, P, 2, None, P, m=4, n=8, ldw=8) == aser.ASER_ERR_INVALID_ARG     # idx missing
    assert s(ctx, P, P, P, 2, P, P, m=4, n=8, ldw=4) == aser.ASER_ERR_SHAPE
    assert s(ctx, P, None, P, 2, P, P, m=4, n=8, ldw=8) == aser.ASER_ERR_INVALID_ARG


def test_rtn_validation(ctx):
    q = aser.aser_quantize_rtn
    assert q(ctx, P, P, P, 2, 3, 0, P, P, P, m=4, n=8) == aser.ASER_ERR_DTYPE            # bits
    assert q(ctx, P, P, P, 2, 8, 1, P, P, P, m=4, n=8) == aser.ASER_ERR_SHAPE            # packed needs 4 bits
    assert q(ctx, P, P, P, 2, 4, 1, P, P, P, m=4, n=7) == aser.ASER_ERR_SHAPE            # packed needs even n
    assert q(ctx, P, P, P, 2, 4, 7, P, P, P, m=4, n=8) == aser.ASER_ERR_INVALID_ARG      # layout
    assert q(ctx, P, None, None, 2, 4, 0, P, P, P, m=4, n=8) == aser.ASER_ERR_INVALID_ARG
    assert q(ctx, P, P, P, 2, 4, 0, P, P, P, m=4, n=8, ldt=4) == aser.ASER_ERR_SHAPE
    assert q(ctx, P, P, P, 2, 4, 0, None, P, P, m=4, n=8) == aser.ASER_ERR_INVALID_ARG
    assert q(ctx, P, P, P, 2, 4, 0, P, P, P, m=4, n=40000) == aser.ASER_ERR_SHAPE


def test_passes_around_another_quantizer_validation(ctx):
    sw, qt = aser.aser_smoothed_weight, aser.aser_quant_target
    assert sw(ctx, None, P, 2, P, m=4, n=8) == aser.ASER_ERR_INVALID_ARG
    assert sw(ctx, P, None, 2, P, m=4, n=8) == aser.ASER_ERR_INVALID_ARG                # idx needed when f > 0
    assert sw(ctx, P, P, 9, P, m=4, n=8) == aser.ASER_ERR_SHAPE                          # f > n
    assert sw(ctx, P, P, 2, P, m=4, n=8, ldws=7) == aser.ASER_ERR_SHAPE
    assert sw(ctx, P + 2, P, 2, P, m=4, n=8) == aser.ASER_ERR_INVALID_ARG               # misaligned
    assert qt(ctx, P, P, None, P, m=4, n=8) == aser.ASER_ERR_INVALID_ARG
    assert qt(ctx, P, P, P, P, m=0, n=8) == aser.ASER_ERR_SHAPE
    assert qt(ctx, P, P, P, P, m=4, n=8, ldq=4) == aser.ASER_ERR_SHAPE
    assert qt(ctx, P, P, P, P, m=4, n=8, ldq=8, ldt=12) == aser.ASER_ERR_SHAPE          # in place with another leading dimension
    assert "in place" in ctx.last_error()


def test_whiten_and_reconstruct_validation(ctx):
    st, _ = aser.aser_whiten(ctx, P, None, -1.0, P, n=8, ldg=8, lds=8)
    assert st == aser.ASER_ERR_INVALID_ARG
    st, _ = aser.aser_whiten(ctx, P, None, 0.0, P, n=8, ldg=4, lds=8)
    assert st == aser.ASER_ERR_SHAPE
    st, _ = aser.aser_whiten(ctx, None, None, 0.0, P, n=8, ldg=8, lds=8)
    assert st == aser.ASER_ERR_INVALID_ARG
    r = aser.aser_error_reconstruct
    assert r(ctx, P, P, 0, P, P, P, m=64, n=64)[0] == aser.ASER_ERR_SHAPE
    assert r(ctx, P, P, 65, P, P, P, m=64, n=256)[0] == aser.ASER_ERR_SHAPE             # r > min(m, n)
    assert r(ctx, P, P, 257, P, P, P, m=512, n=512)[0] == aser.ASER_ERR_SHAPE            # the dense solver's limit
    assert r(ctx, P, P, 129, P, P, P, m=512, n=512)[0] == aser.ASER_ERR_WORKSPACE        # accepted: dense solver, no workspace bound
    assert r(ctx, P, P, 129, P, P, P, m=20000, n=20000)[0] == aser.ASER_ERR_SHAPE        # dense solver: shorter side <= 16384
    assert r(ctx, P, P, 8, None, P, P, m=64, n=64)[0] == aser.ASER_ERR_INVALID_ARG
    assert r(ctx, P, P, 8, P, P, P, idx=None, f=3, m=64, n=64)[0] == aser.ASER_ERR_INVALID_ARG   # f > 0 needs idx
    assert r(ctx, P, P, 8, P, P, P, idx=P, f=65, m=64, n=64)[0] == aser.ASER_ERR_SHAPE            # f > n
    o = aser.aser_svd_opts(block=48, max_iter=0, seed=0)
    assert r(ctx, P, P, 8, P, P, P, o, m=64, n=64)[0] == aser.ASER_ERR_SHAPE             # block not multiple of 32
    it = aser.aser_svd_opts(block=0, max_iter=5, seed=0)                                 # asks for the subspace iteration
    assert r(ctx, P, P, 40, P, P, P, it, m=695, n=44)[0] == aser.ASER_ERR_SHAPE          # no multiple of 32 in [40, 44]
    assert "block width" in ctx._lib.aser_last_error(ctx.handle).decode()
    assert r(ctx, P, P, 40, P, P, P, m=695, n=44)[0] == aser.ASER_ERR_WORKSPACE          # the dense solver takes any r <= min(m, n)
    assert r(ctx, P, P, 45, P, P, P, m=695, n=44)[0] == aser.ASER_ERR_SHAPE


def test_layers_in_flight_validation(ctx):
    lib = aser.load_library()
    # nothing enqueued: nothing to finish
    st, _, _ = aser.aser_finish(ctx)
    assert st == aser.ASER_ERR_INVALID_ARG and "pending" in ctx.last_error()
    assert lib.aser_calibrate_layers(None, 1, None, 0) == aser.ASER_ERR_INVALID_ARG
    handles = (ctypes.c_void_p * 1)(ctx.handle)
    assert lib.aser_calibrate_layers(handles, 0, None, 0) == aser.ASER_ERR_INVALID_ARG
    assert lib.aser_calibrate_layers(handles, 1, None, 0) == aser.ASER_OK                # no layers: nothing to do
    assert lib.aser_calibrate_layers(handles, 1, None, 2) == aser.ASER_ERR_INVALID_ARG
    # a layer whose arguments a stage refuses is reported in its descriptor and the others are still visited
    bad = aser.aser_layer_desc()                                                       # no shape at all
    nostats = aser.aser_layer_desc()
    nostats.m, nostats.n = 8, 16                                                       # neither activations nor statistics
    worse = aser.aser_layer_desc()
    worse.X, worse.x_dtype, worse.rows, worse.ldx, worse.G, worse.ldg = P, 7, 4, 16, P, 16       # unknown dtype
    worse.m, worse.n, worse.T, worse.S = 8, 16, P, P
    small = aser.aser_layer_desc()                                                     # T and S left to a workspace that is not bound
    small.X, small.rows, small.ldx, small.G, small.ldg, small.m, small.n, small.r = P, 4, 16, P, 16, 8, 16, 4
    st = aser.aser_calibrate_layers([ctx], [bad, nostats, worse, small])
    assert st == aser.ASER_ERR_SHAPE                                                   # the first one that failed
    assert [d.status for d in (bad, nostats, worse, small)] == [aser.ASER_ERR_SHAPE, aser.ASER_ERR_INVALID_ARG,
                                                                aser.ASER_ERR_DTYPE, aser.ASER_ERR_WORKSPACE]
    assert aser.aser_layer_workspace_bytes(small) == aser.aser_workspace_bytes(8, 16, 4) + 8 * 16 * 4 + 16 * 16 * 4
    # statistics taken over from an earlier layer of the call: the reference must point backwards, and at a layer that started
    fwd = aser.aser_layer_desc()
    fwd.m, fwd.n, fwd.stats_from = 8, 16, 2                                            # 1-based: layer 1, which is itself
    back = aser.aser_layer_desc()
    back.m, back.n, back.stats_from = 8, 16, 1                                         # layer 0, which was refused
    st = aser.aser_calibrate_layers([ctx], [bad, fwd, back])
    assert st == aser.ASER_ERR_SHAPE
    assert [d.status for d in (fwd, back)] == [aser.ASER_ERR_INVALID_ARG, aser.ASER_ERR_INVALID_ARG]
    assert "was not started" in ctx.last_error()
    assert aser.aser_layer_workspace_bytes(worse) == aser.aser_workspace_bytes(8, 16, 0)
    cnt, chosen = ctypes.c_int32(0), (ctypes.c_int32 * 2)()
    assert lib.aser_pick_concurrent_streams(0, None, 2, 1, chosen, ctypes.byref(cnt)) == aser.ASER_ERR_INVALID_ARG
    assert lib.aser_pick_concurrent_streams(0, handles, 1, 0, chosen, ctypes.byref(cnt)) == aser.ASER_ERR_INVALID_ARG
    assert lib.aser_pick_concurrent_streams(-1, handles, 1, 1, chosen, ctypes.byref(cnt)) == aser.ASER_ERR_INVALID_ARG
    # the struct the binding marshals has the layout the header declares (sizes of the C compiler's struct)
    assert ctypes.sizeof(aser.aser_layer_desc) == 232


def test_svd_plan_reports_what_the_iteration_will_use():
    assert aser.aser_svd_plan(4096, 4096, 64) == (aser.ASER_OK, 128, 9)
    assert aser.aser_svd_plan(4096, 11008, 64) == (aser.ASER_OK, 128, 12)
    assert aser.aser_svd_plan(8192, 28672, 128) == (aser.ASER_OK, 128, 30)       # no oversampling columns
    # ranks beyond the widest subspace block go to the dense solver: no block, no iterations
    assert aser.aser_svd_plan(4096, 4096, 200) == (aser.ASER_OK, 0, 0)
    assert aser.aser_svd_plan(4096, 4096, 257)[0] == aser.ASER_ERR_SHAPE
    assert aser.aser_svd_plan(20000, 28672, 200)[0] == aser.ASER_ERR_SHAPE       # dense solver: shorter side <= 16384
    assert aser.aser_workspace_bytes(2048, 2048, 192) > 3 * 2048 * 2048 * 8      # fp64 product, Gram matrix, reflectors
    assert aser.aser_svd_plan(256, 256, 16) == (aser.ASER_OK, 32, 9)
    assert aser.aser_svd_plan(322, 74, 23) == (aser.ASER_OK, 64, 9)              # 2 r = 46 -> 64 fits in n = 74
    assert aser.aser_svd_plan(300, 40, 23)[:2] == (aser.ASER_OK, 32)             # shrunk to fit the matrix
    assert aser.aser_svd_plan(695, 44, 40)[0] == aser.ASER_ERR_SHAPE
    o = aser.aser_svd_opts(block=96, max_iter=5, seed=0)
    assert aser.aser_svd_plan(4096, 4096, 64, o) == (aser.ASER_OK, 96, 5)


def test_act_rtn_validation(ctx):
    a = aser.aser_quantize_act_rtn
    assert a(ctx, P, None, 9, P, P, rows=4, n=8, ldx=8, x_dtype=0) == aser.ASER_ERR_DTYPE
    assert a(ctx, P, None, 8, P, P, rows=4, n=8, ldx=8, x_dtype=3) == aser.ASER_ERR_DTYPE
    assert a(ctx, P, None, 8, P, P, rows=4, n=8, ldx=4, x_dtype=0) == aser.ASER_ERR_SHAPE
    assert a(ctx, P, None, 8, P, P, rows=0, n=8, ldx=8, x_dtype=0) == aser.ASER_OK


def test_spectrum_validation(ctx):
    sv = aser.aser_singular_values
    assert sv(ctx, P, None, None, m=8, n=8) == aser.ASER_ERR_INVALID_ARG                 # sigma missing
    assert sv(ctx, P, None, P, m=8, n=8, ldt=4) == aser.ASER_ERR_SHAPE
    assert sv(ctx, P, None, P, m=20000, n=20000) == aser.ASER_ERR_SHAPE                  # min(m, n) > 16384
    assert sv(ctx, P, P, P, m=64, n=64) == aser.ASER_ERR_WORKSPACE
    assert aser.aser_spectrum_workspace_bytes(4096, 4096, True) >= 3 * 4096 * 4096 * 4 + 4096 * 4096 * 8
    assert aser.aser_spectrum_workspace_bytes(4096, 1024, False) < aser.aser_spectrum_workspace_bytes(4096, 1024, True)
    assert aser.aser_select_rank(ctx, P, 0.0, k=8)[0] == aser.ASER_ERR_INVALID_ARG       # alpha outside (0, 1)
    assert aser.aser_select_rank(ctx, P, 1.0, k=8)[0] == aser.ASER_ERR_INVALID_ARG
    assert aser.aser_select_rank(ctx, P, 0.5, k=0)[0] == aser.ASER_ERR_SHAPE
    assert aser.aser_select_rank(ctx, P, 0.5, k=8)[0] == aser.ASER_ERR_WORKSPACE
    assert aser.aser_effective_rank(ctx, P, -1.0, k=8)[0] == aser.ASER_ERR_INVALID_ARG
    assert aser.aser_effective_rank(ctx, P + 4, 0.0, k=8)[0] == aser.ASER_ERR_INVALID_ARG


def test_output_error_validation(ctx):
    e = aser.aser_layer_output_error
    kw = dict(m=8, n=16, ldw=16, rows=4, ldx=16, x_dtype=0)
    assert e(ctx, P, P, None, P, 0, P, None, None, 0, 8, **kw)[0] == aser.ASER_ERR_WORKSPACE
    assert e(ctx, P, P, None, P, 0, P, None, None, 3, 8, **kw)[0] == aser.ASER_ERR_INVALID_ARG     # r > 0 without factors
    assert e(ctx, P, P, None, P, 0, P, None, None, 0, 9, **kw)[0] == aser.ASER_ERR_DTYPE
    assert e(ctx, P, P, None, P, 0, P, None, None, 0, 1, **kw)[0] == aser.ASER_ERR_DTYPE
    assert e(ctx, P, P, None, P, 5, P, None, None, 0, 8, **kw)[0] == aser.ASER_ERR_INVALID_ARG     # layout
    assert e(ctx, P, P, None, P, 1, P, None, None, 0, 8, m=8, n=15, ldw=15, rows=4, ldx=15, x_dtype=0)[0] == aser.ASER_ERR_SHAPE
    assert e(ctx, P, P, None, None, 0, P, None, None, 0, 8, **kw)[0] == aser.ASER_ERR_INVALID_ARG
    assert e(ctx, P, P, None, P, 0, P, None, None, 0, 8, m=8, n=16, ldw=8, rows=4, ldx=16, x_dtype=0)[0] == aser.ASER_ERR_SHAPE
    assert aser.aser_output_error_workspace_bytes(4096, 4096, 4096, 64) >= 5 * 4096 * 4096 * 4


def test_forward_validation(ctx):
    f = aser.aser_compensated_forward
    kw = dict(rows=4, n=64, m=8, ldy=8)
    assert f(ctx, P, P, P, 0, P, None, None, 0, False, None, **kw) == aser.ASER_ERR_INVALID_ARG      # Y missing
    assert f(ctx, P, P, P, 0, P, None, None, 0, False, P, rows=4, n=48, m=8, ldy=8) == aser.ASER_ERR_SHAPE   # n % 32
    assert f(ctx, P, P, P, 0, P, None, None, 0, False, P, rows=4, n=64, m=8, ldy=4) == aser.ASER_ERR_SHAPE
    assert f(ctx, P, P, P, 3, P, None, None, 0, False, P, **kw) == aser.ASER_ERR_INVALID_ARG         # layout
    assert f(ctx, P, P, P, 0, P, None, None, 8, False, P, **kw) == aser.ASER_ERR_INVALID_ARG         # r > 0 without factors
    assert f(ctx, P, P, P, 0, P, P, P, 129, False, P, **kw) == aser.ASER_ERR_SHAPE
    assert f(ctx, P + 8, P, P, 0, P, None, None, 0, False, P, **kw) == aser.ASER_ERR_INVALID_ARG     # codes not 16-byte aligned
    assert f(ctx, P, P, P, 0, P, P, P, 8, False, P, **kw) == aser.ASER_ERR_WORKSPACE
    assert f(ctx, P, P, P, 0, P, None, None, 0, False, P, rows=0, n=64, m=8, ldy=8) == aser.ASER_OK  # no tokens: no-op
    assert aser.aser_forward_workspace_bytes(32768, 4096, 4096, 0) == 256


def test_mfma_rate_probe_validation(ctx):
    assert aser.aser_mfma_rate_probe(ctx, 4, 1, 100)[0] == aser.ASER_ERR_INVALID_ARG       # unknown kind
    assert aser.aser_mfma_rate_probe(ctx, -1, 1, 100)[0] == aser.ASER_ERR_INVALID_ARG
    assert aser.aser_mfma_rate_probe(ctx, 2, 2, 100)[0] == aser.ASER_ERR_SHAPE             # with operand traffic: one per compute unit
    assert aser.aser_mfma_rate_probe(ctx, 0, 0, 100)[0] == aser.ASER_ERR_SHAPE             # workgroups per compute unit
    assert aser.aser_mfma_rate_probe(ctx, 0, 5, 100)[0] == aser.ASER_ERR_SHAPE
    assert aser.aser_mfma_rate_probe(ctx, 1, 1, 0)[0] == aser.ASER_ERR_SHAPE               # iterations
    assert aser.aser_mfma_rate_probe(ctx, 1, 1, 100)[0] == aser.ASER_ERR_WORKSPACE         # nothing bound
    assert aser.aser_mfma_rate_probe(ctx, 3, 1, 100)[0] == aser.ASER_ERR_WORKSPACE


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2411_07762_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                assert "oracle" not in open(os.path.join(dirpath, fn)).read().lower().replace("no cpu fallback", ""), fn
