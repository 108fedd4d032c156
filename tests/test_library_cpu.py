"""CPU-side checks of liblutkan: it loads, exports every symbol the header declares, its host LUT compiler
produces bit-identical artifacts to the oracle, the device-table layout matches its documentation, and bad
arguments come back as error codes.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2601_03332_amd as lk
from paper_2601_03332_amd import binding
from lutkan_inputs import (ASYM_UINT8, CLIP_X, CLOSED, HALF_OPEN, SYM_INT8, ZERO_SPLINE, cfg1, cfg2, cfg5,
                           random_layer, uniform_ext_knots)
from lutkan_inputs import draw_edge_scales, per_input_layer

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "lutkan.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:lutkan|bspline)_[a-z0-9_]+)\s*\(", header))
    assert {"lutkan_compile", "lutkan_forward", "bspline_kan_forward", "lutkan_model_forward",
            "lutkan_forward_trace"} <= declared
    lib = lk.load_library()
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in lutkan.h but not exported"
    assert declared == set(binding.EXPORTS)
    assert lk.lutkan_version().startswith("lutkan-gfx950")


def _both(s):
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob)
    ora = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme)
    return art, ora


def _specs():
    yield cfg1().layers[0]
    yield from cfg2(B=4).layers
    yield from cfg5(B=4).layers
    for seed, (d, m, G, L, scheme, uni) in enumerate([(3, 5, 4, 2, SYM_INT8, False), (2, 130, 7, 33, ASYM_UINT8, False),
                                                      (4, 70, 64, 8, SYM_INT8, True), (2, 129, 8, 128, ASYM_UINT8, False),
                                                      (1, 1, 1, 16, ASYM_UINT8, True)]):
        yield random_layer(50 + seed, d, m, G, L, scheme, CLOSED, CLIP_X, 4, uniform=uni).layers[0]


@pytest.mark.parametrize("s", list(_specs()), ids=lambda s: f"{s.d}x{s.m}_G{s.G}_L{s.L}_s{s.scheme}")
def test_host_compile_is_bit_identical_to_the_oracle_and_tables_follow_the_documented_layout(s):
    art, ora = _both(s)
    np.testing.assert_array_equal(art.q, ora.q)
    np.testing.assert_array_equal(art.scale.view(np.uint32), ora.scale.view(np.uint32))
    np.testing.assert_array_equal(art.y_min, ora.y_min)
    np.testing.assert_array_equal(art.knots, ora.knots)
    I = art.info
    K, L, jt, nt = I.K, I.L, I.jt, I.n_tiles
    assert nt == -(-s.m // jt) and (jt & (jt - 1)) == 0 and 4 <= jt <= 64
    cjt, cnt = I.coef_jt, I.coef_n_tiles                   # the B-spline table has its own tile width, up to 128 columns
    assert cnt == -(-s.m // cjt) and (cjt & (cjt - 1)) == 0 and jt <= cjt <= 128 and I.coef_blob_bytes == (s.G + 3) * cjt * 4
    asym = s.scheme == ASYM_UINT8
    codes_off = (K + 1) * jt * 4 * (2 if asym else 1)
    assert I.blob_bytes == (codes_off + (K * L + 2) * jt + 15) // 16 * 16
    assert I.table_bytes == nt * s.d * I.blob_bytes and I.coef_table_bytes == cnt * s.d * (s.G + 3) * cjt * 4
    assert I.artifact_bytes == oracle.artifact_bytes(s.d * s.m, K, L, 8)
    tab = art.table.reshape(nt, s.d, I.blob_bytes)
    ctab = art.coef_table.reshape(cnt, s.d, s.G + 3, cjt)
    for t in range(cnt):
        cols = np.arange(t * cjt, min(s.m, (t + 1) * cjt))
        for i in range(s.d):
            np.testing.assert_array_equal(ctab[t, i, :, :cols.size], s.coef[i, cols].T)
            assert np.all(ctab[t, i, :, cols.size:] == 0)
    qdt = np.uint8 if asym else np.int8
    for t in range(nt):
        cols = np.arange(t * jt, min(s.m, (t + 1) * jt))
        n = cols.size
        for i in range(s.d):
            e = i * s.m + cols
            blob = tab[t, i]
            prm = blob[:codes_off].view(np.float32).reshape(K + 1, 2 if asym else 1, jt)   # row = alpha plane, y_min plane
            np.testing.assert_array_equal(prm[:K, 0, :n], art.scale[e].T)
            if asym:
                np.testing.assert_array_equal(prm[:K, 1, :n], art.y_min[e].T)
            assert np.all(prm[:, :, n:] == 0) and np.all(prm[K] == 0)
            codes = blob[codes_off:codes_off + K * L * jt].reshape(K, L, jt)
            want = np.transpose(art.q[e], (1, 2, 0))
            want = want.view(np.uint8) if asym else (want.astype(np.int16) + 128).astype(np.uint8)   # int8: excess-128
            np.testing.assert_array_equal(codes[:, :, :n], want)
            assert np.all(codes[:, :, n:] == 0) and np.all(blob[codes_off + K * L * jt:] == 0)


def test_device_struct_initialisers():
    s = cfg2(B=4).layers[0]
    art, _ = _both(s)
    lib = lk.load_library()
    dl = binding._DevLayer()
    assert lib.lutkan_dev_layer_init(art._h, C.byref(dl)) == 0
    assert (dl.d, dl.m, dl.K, dl.L, dl.scheme, dl.boundary, dl.oob) == (78, 16, 5, 64, ASYM_UINT8, CLOSED, CLIP_X)
    assert dl.table is None and list(dl.knots)[:6] == list(art.knots)
    bl = binding._SplineDevLayer()
    assert lib.bspline_dev_layer_init(art._h, C.byref(bl)) == 0
    assert (bl.d, bl.m, bl.G, bl.degree) == (78, 16, 5, 3) and list(bl.ext_knots)[:12] == list(art.ext_knots)
    need = lib.lutkan_forward_workspace_bytes(C.byref(dl), 1000)      # records (8 B per input and padded row) + partial sums
    assert 78 * 1024 * 8 <= need <= 78 * 1024 * 8 + 32 * 1000 * 16 * 4
    dl.value_repr = 1                                                 # spline_component: 16-byte records (with SiLU(x))
    assert lib.lutkan_forward_workspace_bytes(C.byref(dl), 1000) == need + 78 * 1024 * 8
    # a shape whose base branch can run as a matrix product (d a multiple of 32, m >= 64) also needs room for the three
    # bf16 pieces of s_out * s_base, columns padded to 128
    wide = random_layer(7, 64, 200, 5, 16, SYM_INT8, CLOSED, CLIP_X, 4, with_base=True).layers[0]
    wide_art = lk.lutkan_compile(wide.d, wide.m, wide.G, wide.p, wide.ext_knots, wide.coef, wide.L, wide.scheme, wide.boundary,
                                 wide.oob, edge_scales=wide.edge_scales)
    wl = binding._DevLayer()
    assert lib.lutkan_dev_layer_init(wide_art._h, C.byref(wl)) == 0
    with_pieces = lib.lutkan_forward_workspace_bytes(C.byref(wl), 1000)
    wl.value_repr = 0
    assert with_pieces - lib.lutkan_forward_workspace_bytes(C.byref(wl), 1000) == 64 * 1024 * 8 + 6 * 256 * 64
    dl.value_repr = 0
    assert lib.lutkan_forward_workspace_bytes(C.byref(dl), 0) == 0
    assert I_tK_star(art, CLOSED) == art.knots[-1]


def I_tK_star(art, boundary):
    return art.info.tK_star


def test_tK_star_is_nextafter_in_half_open_mode():
    s = cfg1().layers[0]
    a = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, HALF_OPEN, ZERO_SPLINE)
    assert a.info.tK_star == np.nextafter(np.float32(1.0), np.float32(-np.inf)) and a.info.tK == 1.0 and a.info.t0 == -1.0


def test_compile_rejects_bad_arguments_with_error_codes():
    s = cfg1().layers[0]
    lib = lk.load_library()

    def rc(**kw):
        a = dict(d=s.d, m=s.m, G=s.G, degree=3, ext_knots=s.ext_knots, coef=s.coef, L=s.L, scheme=s.scheme,
                 boundary=s.boundary, oob=s.oob)
        a.update(kw)
        tau = np.ascontiguousarray(a["ext_knots"], dtype=np.float32)
        cf = np.ascontiguousarray(a["coef"], dtype=np.float32)
        desc = binding._LayerDesc(a["d"], a["m"], a["G"], a["degree"], tau.ctypes.data, cf.ctypes.data, a["L"],
                                  a["scheme"], a["boundary"], a["oob"], a.get("value_repr", 0), None, None, None)
        out = C.c_void_p()
        code = lib.lutkan_compile(C.byref(desc), 1, C.byref(out))
        if code == 0:
            lib.lutkan_artifact_free(out)
        return code, lk.lutkan_last_error()

    assert rc()[0] == 0
    assert rc(L=1) == (-1, "lutkan_compile: L must be >= 2 (got 1)")
    assert rc(degree=2)[0] == -5
    assert rc(scheme=2)[0] == -1 and rc(boundary=-1)[0] == -1 and rc(oob=9)[0] == -1
    assert rc(value_repr=2)[0] == -1
    code, msg = rc(value_repr=1)                       # spline_component without its three per-edge arrays
    assert code == -1 and "edge_base_scale" in msg
    bad = s.ext_knots.copy()
    bad[4] = bad[3]
    code, msg = rc(ext_knots=bad)
    assert code == -1 and "strictly increasing" in msg
    nanc = s.coef.copy()
    nanc[1, 2, 3] = np.nan
    assert rc(coef=nanc)[0] == -1
    assert lib.lutkan_compile(None, 1, None) == -1
    big = uniform_ext_knots(-1, 1, 65)
    assert rc(G=65, ext_knots=big, coef=np.zeros((s.d, s.m, 68), np.float32))[0] == -5
    assert lib.lutkan_artifact_info(None, None) == -1


def test_forward_argument_validation_happens_before_any_launch():
    # None of these reaches a kernel launch: every call must be rejected on the host, GPU or not.
    s = cfg1().layers[0]
    art, _ = _both(s)
    lib = lk.load_library()
    dl = binding._DevLayer()
    lib.lutkan_dev_layer_init(art._h, C.byref(dl))
    assert lib.lutkan_forward(C.byref(dl), 16, 4, 32, None, 256, 1 << 20, None) == -1      # table is NULL
    assert "table" in lk.lutkan_last_error()
    assert lk.lutkan_last_plan() == ""                                                       # nothing was launched
    dl.table = 4096
    assert lib.lutkan_forward(C.byref(dl), 16, 0, 32, None, None, 0, None) == 0            # B == 0: no-op
    assert lib.lutkan_forward(C.byref(dl), 16, -1, 32, None, 256, 1 << 20, None) == -1
    assert lib.lutkan_forward(C.byref(dl), None, 4, 32, None, 256, 1 << 20, None) == -1
    assert lib.lutkan_forward(C.byref(dl), 16, 4, 32, None, 256, 8, None) == -2            # workspace too small
    assert lib.lutkan_forward(C.byref(dl), 16, 4, 32, None, 257, 1 << 20, None) == -1      # misaligned workspace
    dl.L = 1
    assert lib.lutkan_forward(C.byref(dl), 16, 4, 32, None, 256, 1 << 20, None) == -1
    dl.L = s.L
    dl.knots[2] = dl.knots[1]
    assert lib.lutkan_forward(C.byref(dl), 16, 4, 32, None, 256, 1 << 20, None) == -1
    two = (binding._DevLayer * 2)(dl, dl)
    assert lib.lutkan_model_forward(two, 2, 16, 4, 32, None, 256, 1 << 20, None) == -1     # every layer is validated first
    # the fused chain: same checks, plus the shapes it cannot hold
    assert lib.lutkan_chain_forward(two, 2, 16, 4, 32, None, None, None) == -1             # the knots are still broken
    dl.knots[2] = np.float32(0.5 * (dl.knots[1] + dl.knots[3]))
    two, one = (binding._DevLayer * 2)(dl, dl), (binding._DevLayer * 1)(dl)
    assert lib.lutkan_chain_forward(two, 2, 16, 4, 32, None, None, None) == -2
    assert lib.lutkan_model_forward(two, 2, 16, 4, 32, None, 256, 1 << 20, None) == -2     # m of layer 0 != d of layer 1
    assert lib.lutkan_chain_forward(one, 1, 16, 0, 32, None, None, None) == 0               # B == 0: no-op
    assert lib.lutkan_chain_forward(one, 1, None, 4, 32, None, None, None) == -1
    assert lib.lutkan_chain_forward(one, 1, 16, 4, 16, None, None, None) == -1              # x and y alias
    assert lib.lutkan_chain_forward(one, 0, 16, 4, 32, None, None, None) == -1
    nine = (binding._DevLayer * 9)(*([dl] * 9))
    assert lib.lutkan_chain_forward(nine, 9, 16, 4, 32, None, None, None) == -5             # more than eight layers
    # the entry point with the built-in scratch array: the same checks, and sizes beyond the array are refused
    assert lib.lutkan_forward_static_scratch(C.byref(dl), 16, 0, 32, None, None) == 0       # B == 0: no-op
    assert lib.lutkan_forward_static_scratch(C.byref(dl), 16, -1, 32, None, None) == -1
    too_many = binding.STATIC_SCRATCH_BYTES // (8 * s.d) + 1024
    assert lib.lutkan_forward_workspace_bytes(C.byref(dl), too_many) > binding.STATIC_SCRATCH_BYTES
    assert lib.lutkan_forward_static_scratch(C.byref(dl), 16, too_many, 32, None, None) == -2
    assert "built-in array holds 67108864" in lk.lutkan_last_error()
    header = open(os.path.join(ROOT, "include", "lutkan.h")).read()
    assert re.search(r"#define LUTKAN_STATIC_SCRATCH_BYTES \(64u << 20\)", header) and binding.STATIC_SCRATCH_BYTES == 64 << 20
    nul = binding._DevLayer.from_buffer_copy(dl)
    nul.table = None
    assert lib.lutkan_forward_static_scratch(C.byref(nul), 16, 4, 32, None, None) == -1
    wide = cfg5().layers[1]                                                                  # 128 -> 128
    wl = binding._DevLayer()
    wide_art = _both(wide)[0]                                                               # stays alive across the call
    lib.lutkan_dev_layer_init(wide_art._h, C.byref(wl))
    wl.table = 4096
    assert lib.lutkan_chain_forward((binding._DevLayer * 1)(wl), 1, 16, 4, 32, None, None, None) == -5
    assert "at most 64 columns" in lk.lutkan_last_error()


def test_binding_refuses_tensors_of_the_wrong_shape_dtype_or_device():
    """The kernels index x as [B, d] and y as [B, m] on trust, so the binding checks every tensor before a pointer
    reaches the library.  No GPU is needed to see the refusals: the layer below is a host-side stand-in."""
    import torch
    s = cfg2(B=4).layers[0]                                     # 78 -> 16
    art, _ = _both(s)
    layer = object.__new__(lk.LutLayer)
    layer.c = binding._DevLayer()
    lk.load_library().lutkan_dev_layer_init(art._h, C.byref(layer.c))
    layer.d, layer.m, layer.device = s.d, s.m, torch.device("cpu")
    spline = object.__new__(lk.BsplineLayer)
    spline.c = binding._SplineDevLayer()
    lk.load_library().bspline_dev_layer_init(art._h, C.byref(spline.c))
    spline.d, spline.m, spline.device = s.d, s.m, torch.device("cpu")
    x = torch.zeros((8, s.d))
    y = torch.zeros((8, s.m))
    ws = torch.zeros(1 << 16, dtype=torch.uint8)
    bad_calls = [
        lambda: lk.lutkan_forward(layer, torch.zeros((8, s.d + 1))),                       # wrong width
        lambda: lk.lutkan_forward(layer, torch.zeros(8 * s.d)),                            # not two-dimensional
        lambda: lk.lutkan_forward(layer, x.double()),                                       # wrong dtype
        lambda: lk.lutkan_forward(layer, x, torch.zeros((7, s.m))),                        # y too short
        lambda: lk.lutkan_forward(layer, x, torch.zeros((8, s.m - 1))),
        lambda: lk.lutkan_forward(layer, x, y, stats=torch.zeros(3, dtype=torch.int64)),
        lambda: lk.lutkan_forward(layer, x, y, workspace=ws.float()),
        lambda: lk.lutkan_forward(layer, x, y),                                             # right shapes, but not on a GPU
        lambda: lk.lutkan_forward_static_scratch(layer, x, None),
        lambda: lk.lutkan_forward_static_scratch(layer, x, torch.zeros((9, s.m))),
        lambda: lk.lutkan_forward_trace(layer, torch.zeros((8, 3))),
        lambda: lk.lutkan_forward_locate(layer, torch.zeros((8, s.m)), ws),
        lambda: lk.lutkan_forward_edges(layer, 9, y, ws),                                  # B does not match y
        lambda: lk.lutkan_forward_edges(layer, 8, torch.zeros((8, s.d)), ws),
        lambda: lk.bspline_kan_forward(spline, torch.zeros((8, s.d - 1))),
        lambda: lk.bspline_kan_forward(spline, x, torch.zeros((8, s.m + 1))),
        lambda: lk.bspline_forward_locate(spline, torch.zeros((s.d, 8)), ws),
        lambda: lk.bspline_forward_edges(spline, 4, y, ws),
        lambda: lk.lutkan_model_forward([layer, layer], x),                                # 16 outputs feed 78 inputs
        lambda: lk.lutkan_model_forward([], x),
        lambda: lk.lutkan_model_forward([layer], torch.zeros((8, 5))),
        lambda: lk.lutkan_model_forward([layer], x, torch.zeros((8, s.m)), stats=torch.zeros(4, dtype=torch.int64)),
        lambda: lk.lutkan_chain_forward([layer], torch.zeros((8, s.d, 1))),
        lambda: lk.lutkan_chain_forward([layer, layer], x),
        lambda: lk.lutkan_error_stats(y, torch.zeros((8, s.m + 1)), x, -1.0, 1.0, CLOSED),
        lambda: lk.lutkan_error_stats(y, y, torch.zeros((7, s.d)), -1.0, 1.0, CLOSED),
    ]
    for n, call in enumerate(bad_calls):
        with pytest.raises(lk.LutKanError):
            call()
            pytest.fail(f"call {n} was not refused")
    assert lk.lutkan_last_plan() == ""                          # nothing reached a launch


def test_stored_symmetric_artifact_with_an_offset_is_refused():
    """Eq. 11 fixes y_min = 0 for symmetric int8 and the device table of that scheme carries no y_min plane: stored
    arrays that say otherwise are refused instead of silently losing the offset."""
    s = cfg1().layers[0]
    art, _ = _both(s)
    ok = lk.lutkan_artifact_from_arrays(s.d, s.m, art.knots, art.q, art.scale, art.y_min, s.boundary, s.oob)
    assert np.array_equal(ok.table, art.table)
    shifted = art.y_min.copy()
    shifted[5, 2] = np.float32(1e-3)
    with pytest.raises(lk.LutKanError) as e:
        lk.lutkan_artifact_from_arrays(s.d, s.m, art.knots, art.q, art.scale, shifted, s.boundary, s.oob)
    assert str(e.value).startswith("[-1]") and "Eq. 11" in str(e.value)
    minus_zero = np.full_like(art.y_min, -0.0)                  # -0 is still zero
    lk.lutkan_artifact_from_arrays(s.d, s.m, art.knots, art.q, art.scale, minus_zero, s.boundary, s.oob)


def test_workspace_queries_return_zero_for_tile_widths_no_kernel_has():
    """The size queries run on structs nobody has validated yet: a tile width outside what the kernels exist for gives
    0 (and the forward call then refuses the layer), never a division by zero in the launch planning."""
    s = cfg1().layers[0]
    art, _ = _both(s)
    lib = lk.load_library()
    dl = binding._DevLayer()
    lib.lutkan_dev_layer_init(art._h, C.byref(dl))
    bl = binding._SplineDevLayer()
    lib.bspline_dev_layer_init(art._h, C.byref(bl))
    assert lib.lutkan_forward_workspace_bytes(C.byref(dl), 100) > 0 and lib.bspline_forward_workspace_bytes(C.byref(bl), 100) > 0
    for jt in (0, 3, 6, 128, 256, 260, 1024, 1 << 20):
        dl.jt = jt
        assert lib.lutkan_forward_workspace_bytes(C.byref(dl), 100) == 0, jt
        assert lib.lutkan_model_workspace_bytes((binding._DevLayer * 1)(dl), 1, 100) == 0
        dl.table = 4096
        assert lib.lutkan_model_forward((binding._DevLayer * 1)(dl), 1, 16, 100, 32, None, 256, 1 << 30, None) == -1
        assert "jt" in lk.lutkan_last_error()
    for jt in (0, 3, 12, 256, 512, 1 << 20):
        bl.jt = jt
        assert lib.bspline_forward_workspace_bytes(C.byref(bl), 100) == 0, jt


def test_wide_table_form_sizes_and_refusals():
    """The second form of the device table (two bytes per code): which layers have one, how large it is, and what the
    build call and the forward calls refuse before anything reaches the GPU (the pointers below are stand-ins)."""
    lib = lk.load_library()
    rng = np.random.Generator(np.random.PCG64(12))

    def dev_layer(m, G, L, scheme, scales=False):
        tau = np.linspace(-1.0, 1.0, G + 7).astype(np.float32)
        art = lk.lutkan_compile(3, m, G, 3, tau, rng.normal(size=(3, m, G + 3)).astype(np.float32), L, scheme, CLOSED, CLIP_X,
                                edge_scales=draw_edge_scales(rng, 3, m) if scales else None)
        dl = binding._DevLayer()
        assert lib.lutkan_dev_layer_init(art._h, C.byref(dl)) == 0
        assert not dl.wide_table and dl.wide_blob_bytes == 0
        return art, dl

    for m, G, L, scheme, scales in ((130, 8, 64, SYM_INT8, False), (64, 5, 32, ASYM_UINT8, False), (300, 8, 64, ASYM_UINT8, True)):
        art, dl = dev_layer(m, G, L, scheme, scales)
        I = art.info
        assert I.jt == 64
        wide_blob = I.blob_bytes + (I.K * L + 2) * 64               # every code one byte longer, the rest of the slice as it is
        assert wide_blob % 16 == 0 and 2 * wide_blob + 16 * 2 * 64 * 8 <= 160 * 1024
        assert lib.lutkan_wide_table_bytes(C.byref(dl), 2) == I.n_tiles * 3 * wide_blob
        # fp32 values: the base row (with edge scales), then one 256-byte row per code row and no parameter rows
        values_blob = (256 if scales else 0) + (I.K * L + 2) * 256
        fits = 2 * values_blob + 16 * 2 * 64 * 8 <= 160 * 1024
        assert fits == (L == 32)
        assert lib.lutkan_wide_table_bytes(C.byref(dl), 4) == (I.n_tiles * 3 * values_blob if fits else 0)
        for cb in (0, 1, 3, 8):
            assert lib.lutkan_wide_table_bytes(C.byref(dl), cb) == 0
    # no wide form: tiles narrower than 64 columns; slices that do not fit the LDS twice (642 and 1026 code rows)
    for m, G, L in ((32, 5, 16), (16, 8, 64), (128, 10, 64), (128, 8, 128)):
        art, dl = dev_layer(m, G, L, SYM_INT8)
        dl.table = 4096
        for cb in (2, 4):
            assert lib.lutkan_wide_table_bytes(C.byref(dl), cb) == 0
            assert lib.lutkan_wide_table_build(C.byref(dl), cb, 8192, 1 << 30, None) == -5 and "no wide form" in lk.lutkan_last_error()
    assert lib.lutkan_wide_table_bytes(None, 2) == 0

    art, dl = dev_layer(130, 8, 64, SYM_INT8)
    need = lib.lutkan_wide_table_bytes(C.byref(dl), 2)
    assert lib.lutkan_wide_table_build(C.byref(dl), 2, 8192, need, None) == -1 and "table is null" in lk.lutkan_last_error()
    dl.table = 4096
    assert lib.lutkan_wide_table_build(C.byref(dl), 2, None, need, None) == -1
    assert lib.lutkan_wide_table_build(C.byref(dl), 2, 8192 + 8, need, None) == -1 and "aligned" in lk.lutkan_last_error()
    assert lib.lutkan_wide_table_build(C.byref(dl), 2, 8192, need - 1, None) == -2 and str(need) in lk.lutkan_last_error()
    assert lib.lutkan_wide_table_build(C.byref(dl), 3, 8192, need, None) == -1 and "code_bytes" in lk.lutkan_last_error()
    assert lib.lutkan_wide_table_build(C.byref(dl), 4, 8192, 1 << 30, None) == -5       # 514 rows of 256 bytes do not fit twice
    assert lib.lutkan_wide_table_build(None, 2, 8192, need, None) == -1
    assert not dl.wide_table and dl.wide_blob_bytes == 0 and dl.wide_code_bytes == 0      # a refused build leaves the layer without
    # a layer whose wide fields do not fit its shape is refused by every forward call
    ws_bytes = lib.lutkan_forward_workspace_bytes(C.byref(dl), 64)
    dl.wide_table, dl.wide_blob_bytes, dl.wide_code_bytes = 8192, art.info.blob_bytes, 2
    assert lib.lutkan_forward(C.byref(dl), 16, 64, 32, None, 256, 1 << 30, None) == -2 and "wide_blob_bytes" in lk.lutkan_last_error()
    dl.wide_table, dl.wide_blob_bytes = 8192 + 4, art.info.blob_bytes + (art.info.K * 64 + 2) * 64
    assert lib.lutkan_forward(C.byref(dl), 16, 64, 32, None, 256, 1 << 30, None) == -1 and "wide_table" in lk.lutkan_last_error()
    dl.wide_table = 8192
    assert lib.lutkan_forward_workspace_bytes(C.byref(dl), 64) >= ws_bytes
    for cb in (0, 1, 4):                                             # no such form, or none of this layer
        dl.wide_code_bytes = cb
        assert lib.lutkan_forward(C.byref(dl), 16, 64, 32, None, 256, 1 << 30, None) == -1 and "no wide form" in lk.lutkan_last_error()
    _, narrow = dev_layer(32, 5, 16, SYM_INT8)
    narrow.table, narrow.wide_table, narrow.wide_blob_bytes, narrow.wide_code_bytes = 4096, 8192, 4096, 2
    assert lib.lutkan_forward(C.byref(narrow), 16, 64, 32, None, 256, 1 << 30, None) == -1 and "no wide form" in lk.lutkan_last_error()
    # the fp32 form of a small asymmetric layer: its size is checked the same way
    art, small = dev_layer(64, 5, 32, ASYM_UINT8)
    small.table, small.wide_table, small.wide_code_bytes = 4096, 8192, 4
    small.wide_blob_bytes = (art.info.K * 32 + 2) * 256
    assert lib.lutkan_forward(C.byref(small), 16, 0, 32, None, 256, 1 << 30, None) == 0   # B = 0: validated, nothing launched
    small.wide_blob_bytes += 16
    assert lib.lutkan_forward(C.byref(small), 16, 0, 32, None, 256, 1 << 30, None) == -2 and "wide_blob_bytes" in lk.lutkan_last_error()


def test_spline_component_tables_carry_the_base_row_and_folded_gains():
    w = random_layer(77, 3, 70, 5, 16, ASYM_UINT8, CLOSED, ZERO_SPLINE, 4, with_base=True)
    s = w.layers[0]
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob, edge_scales=s.edge_scales)
    ora = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme)
    np.testing.assert_array_equal(art.q, ora.q)                        # the table still stores the spline branch
    np.testing.assert_array_equal(art.scale, ora.scale)
    sb, ss, so = (a.reshape(-1) for a in s.edge_scales)
    for got, want in zip(art.edge_scales, (sb, ss, so)):
        np.testing.assert_array_equal(got, want)
    I = art.info
    assert I.value_repr == lk.REPR_SPLINE_COMPONENT
    K, L, jt, nt = I.K, I.L, I.jt, I.n_tiles
    params_off = jt * 4
    codes_off = params_off + (K + 1) * jt * 8
    assert I.blob_bytes == (codes_off + (K * L + 2) * jt + 15) // 16 * 16
    assert I.artifact_bytes == oracle.artifact_bytes(s.d * s.m, K, L, 8) + 12 * s.d * s.m
    tab = art.table.reshape(nt, s.d, I.blob_bytes)
    cjt, cnt = I.coef_jt, I.coef_n_tiles
    ctab = art.coef_table.reshape(cnt, s.d, s.G + 4, cjt)
    for t in range(cnt):
        cols = np.arange(t * cjt, min(s.m, (t + 1) * cjt))
        for i in range(s.d):
            e = i * s.m + cols
            np.testing.assert_array_equal(ctab[t, i, 0, :cols.size], so[e] * sb[e])
            gain = (so[e] * ss[e]).astype(np.float32)
            np.testing.assert_array_equal(ctab[t, i, 1:, :cols.size], (gain[None, :] * s.coef[i, cols].T).astype(np.float32))
    for t in range(nt):
        cols = np.arange(t * jt, min(s.m, (t + 1) * jt))
        n = cols.size
        for i in range(s.d):
            e = i * s.m + cols
            base = tab[t, i, :params_off].view(np.float32)
            np.testing.assert_array_equal(base[:n], so[e] * sb[e])
            prm = tab[t, i, params_off:codes_off].view(np.float32).reshape(K + 1, 2, jt)
            gain = (so[e] * ss[e]).astype(np.float32)
            np.testing.assert_array_equal(prm[:K, 0, :n], (gain[None, :] * art.scale[e].T).astype(np.float32))
            np.testing.assert_array_equal(prm[:K, 1, :n], (gain[None, :] * art.y_min[e].T).astype(np.float32))


@pytest.mark.parametrize("m", [30, 70])
@pytest.mark.parametrize("scheme", [SYM_INT8, ASYM_UINT8])
def test_fp16_parameter_tables(scheme, m):
    """Sec. 4.6 float16 scale / y_min: codes as with fp32 parameters, parameters bit-identical to the oracle's
    rounding, the byte accounting halves the parameter bytes; device rows hold the binary16 bit patterns on tiles of
    up to 32 columns and the same rounded values as fp32 on wider ones."""
    w = random_layer(91, 3, m, 6, 16, scheme, CLOSED, CLIP_X, 4)
    s = w.layers[0]
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, s.boundary, s.oob, param_dtype=lk.PARAM_FP16)
    a32 = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, s.boundary, s.oob)
    ora = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, param_fp16=True)
    np.testing.assert_array_equal(art.q, a32.q)
    np.testing.assert_array_equal(art.q, ora.q)
    np.testing.assert_array_equal(art.scale.view(np.uint32), ora.scale.view(np.uint32))
    np.testing.assert_array_equal(art.y_min.view(np.uint32), ora.y_min.view(np.uint32))
    I = art.info
    assert I.param_dtype == lk.PARAM_FP16 and a32.info.param_dtype == lk.PARAM_FP32
    K, L, jt, nt = I.K, I.L, I.jt, I.n_tiles
    per = 2 if scheme == ASYM_UINT8 else 1
    assert jt == (32 if m == 30 else 64)
    pdt = np.float16 if jt <= 32 else np.float32
    codes_off = (K + 1) * jt * np.dtype(pdt).itemsize * per
    assert I.blob_bytes == (codes_off + (K * L + 2) * jt + 15) // 16 * 16
    assert I.params_canonical_bytes == s.d * s.m * K * 2
    assert I.artifact_bytes == oracle.artifact_bytes(s.d * s.m, K, L, 4)
    tab = art.table.reshape(nt, s.d, I.blob_bytes)
    for t in range(nt):
        cols = np.arange(t * jt, min(s.m, (t + 1) * jt))
        n = cols.size
        for i in range(s.d):
            e = i * s.m + cols
            prm = tab[t, i, :codes_off].view(pdt).reshape(K + 1, per, jt)
            np.testing.assert_array_equal(prm[:K, 0, :n].astype(np.float32), art.scale[e].T)
            if scheme == ASYM_UINT8:
                np.testing.assert_array_equal(prm[:K, 1, :n].astype(np.float32), art.y_min[e].T)
            assert np.all(prm[:, :, n:] == 0) and np.all(prm[K] == 0)
            codes = tab[t, i, codes_off:codes_off + K * L * jt].reshape(K, L, jt)
            want = np.transpose(art.q[e], (1, 2, 0))
            want = want.view(np.uint8) if scheme == ASYM_UINT8 else (want.astype(np.int16) + 128).astype(np.uint8)
            np.testing.assert_array_equal(codes[:, :, :n], want)


@pytest.mark.parametrize("scheme", [SYM_INT8, ASYM_UINT8])
def test_fp16_parameters_with_spline_component(scheme):
    """Sec. 4.6 float16 parameters together with Eq. 2's per-edge scalars: the canonical parameters are the rounded
    values (what Eq. 10 dequantises with); the device table holds their fp32 products with s_out*s_spline, in the
    layout of a float32 spline_component layer."""
    w = random_layer(97, 3, 70, 6, 16, scheme, CLOSED, CLIP_X, 4, with_base=True)
    s = w.layers[0]
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, s.boundary, s.oob,
                            edge_scales=s.edge_scales, param_dtype=lk.PARAM_FP16)
    ora = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, param_fp16=True)
    np.testing.assert_array_equal(art.q, ora.q)
    np.testing.assert_array_equal(art.scale.view(np.uint32), ora.scale.view(np.uint32))
    np.testing.assert_array_equal(art.y_min.view(np.uint32), ora.y_min.view(np.uint32))
    I = art.info
    K, L, jt, nt = I.K, I.L, I.jt, I.n_tiles
    per = 2 if scheme == ASYM_UINT8 else 1
    params_off = jt * 4
    codes_off = params_off + (K + 1) * jt * 4 * per
    assert I.blob_bytes == (codes_off + (K * L + 2) * jt + 15) // 16 * 16
    a32 = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, s.boundary, s.oob, edge_scales=s.edge_scales)
    assert (a32.info.jt, a32.info.blob_bytes) == (jt, I.blob_bytes)
    sb, ss, so = (np.asarray(v, np.float32).reshape(-1) for v in s.edge_scales)
    tab = art.table.reshape(nt, s.d, I.blob_bytes)
    for t in range(nt):
        cols = np.arange(t * jt, min(s.m, (t + 1) * jt))
        n = cols.size
        for i in range(s.d):
            e = i * s.m + cols
            head = tab[t, i, :params_off].view(np.float32)
            np.testing.assert_array_equal(head[:n], so[e] * sb[e])
            assert np.all(head[n:] == 0)
            gain = (so[e] * ss[e]).astype(np.float32)
            prm = tab[t, i, params_off:codes_off].view(np.float32).reshape(K + 1, per, jt)
            np.testing.assert_array_equal(prm[:K, 0, :n], (gain[None, :] * art.scale[e].T).astype(np.float32))
            if scheme == ASYM_UINT8:
                np.testing.assert_array_equal(prm[:K, 1, :n], (gain[None, :] * art.y_min[e].T).astype(np.float32))
            assert np.all(prm[K] == 0)


def test_fp16_parameters_are_refused_where_they_cannot_hold():
    w = random_layer(92, 2, 3, 5, 8, SYM_INT8, CLOSED, CLIP_X, 4)
    s = w.layers[0]
    with pytest.raises(lk.LutKanError) as e:                      # alpha beyond the largest binary16
        lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef * np.float32(1e8), s.L, s.scheme, s.boundary, s.oob,
                          param_dtype=lk.PARAM_FP16)
    assert str(e.value).startswith("[-5]")
    with pytest.raises(lk.LutKanError) as e:
        lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob, param_dtype=7)
    assert str(e.value).startswith("[-1]")


@pytest.mark.parametrize("with_base,param_dtype,scheme", [(False, 0, SYM_INT8), (False, 1, ASYM_UINT8), (True, 0, ASYM_UINT8), (True, 1, ASYM_UINT8)])
def test_artifact_round_trip_through_npz_and_manifest(tmp_path, with_base, param_dtype, scheme):
    """Sec. 4.6 serialisation: the NPZ holds the paper's keys, the manifest its metadata fields, and loading it gives
    back the same canonical arrays and a byte-identical device table."""
    import json
    w = random_layer(93, 3, 70, 6, 16, scheme, HALF_OPEN, ZERO_SPLINE, 4, with_base=with_base)
    s = w.layers[0]
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, s.boundary, s.oob,
                            edge_scales=s.edge_scales, param_dtype=param_dtype)
    path = str(tmp_path / "layer0.npz")
    art.save(path)
    with np.load(path, allow_pickle=False) as z:
        keys = set(z.files)
        man = json.loads(bytes(z["manifest"]).decode())
        assert z["q_table"].shape == (s.d * s.m, s.G, s.L) and z["knots"].shape == (s.G + 1,)
        assert z["scale"].dtype == (np.float16 if param_dtype else np.float32) and z["scale"].shape == (s.d * s.m, s.G)
        payload = sum(z[k].nbytes for k in keys - {"manifest"})
    want_keys = {"manifest", "knots", "q_table", "scale", "y_min"}
    if with_base:
        want_keys |= {"edge_base_scale", "edge_spline_scale", "edge_out_scale"}
        assert man["base_kind"] == "silu"
    assert keys == want_keys
    assert payload == art.info.artifact_bytes                       # "LUT artifact bytes = sum of NPZ payload fields" (Sec. 6.6)
    assert (man["format_version"], man["interp"], man["boundary_mode"], man["oob_policy"], man["L"]) == (1, "linear", "half_open", "zero_spline", s.L)
    assert man["value_repr"] == ("spline_component" if with_base else "phi")
    back = lk.lutkan_artifact_load(path)
    for name in ("q", "scale", "y_min", "knots", "table"):
        np.testing.assert_array_equal(getattr(back, name), getattr(art, name), err_msg=name)
    if with_base:
        for a, b in zip(back.edge_scales, art.edge_scales):
            np.testing.assert_array_equal(a, b)
    for f in ("d", "m", "K", "L", "scheme", "boundary", "oob", "value_repr", "param_dtype", "jt", "n_tiles", "blob_bytes",
              "table_bytes", "artifact_bytes", "tK_star"):
        assert getattr(back.info, f) == getattr(art.info, f), f
    assert back.info.G == 0 and back.coef_table is None and back.ext_knots is None
    bl = binding._SplineDevLayer()
    assert lk.load_library().bspline_dev_layer_init(back._h, C.byref(bl)) == -5     # no spline coefficients in a LUT artifact


def test_artifact_from_arrays_validates_its_input():
    s = random_layer(94, 2, 3, 5, 8, ASYM_UINT8, CLOSED, CLIP_X, 4).layers[0]
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob)
    ok = lambda **kw: lk.lutkan_artifact_from_arrays(**{**dict(d=s.d, m=s.m, knots=art.knots, q_table=art.q, scale=art.scale,
                                                                  y_min=art.y_min, boundary=CLOSED, oob=CLIP_X), **kw})
    np.testing.assert_array_equal(ok().table, art.table)
    bad_knots = art.knots.copy(); bad_knots[2] = bad_knots[1]
    nan_scale = art.scale.copy(); nan_scale[0, 0] = np.nan
    for kw, code in ((dict(knots=bad_knots), "[-1]"), (dict(scale=nan_scale), "[-1]"), (dict(boundary=5), "[-1]"),
                     (dict(param_dtype=lk.PARAM_FP16), "[-1]"),            # fp32 values that are not binary16 values
                     (dict(q_table=art.q.astype(np.int16)), "q_table must be"), (dict(knots=art.knots[:-1]), "do not match")):
        with pytest.raises(lk.LutKanError) as e:
            ok(**kw)
        assert code in str(e.value), (kw.keys(), str(e.value))


@pytest.mark.parametrize("scheme,uniform", [(SYM_INT8, True), (ASYM_UINT8, False)])
def test_extended_knot_span_compiles_like_the_oracle(scheme, uniform):
    s = random_layer(95, 3, 5, 6, 16, scheme, CLOSED, CLIP_X, 4, uniform=uniform).layers[0]
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, s.boundary, s.oob, knot_span=lk.SPAN_EXTENDED)
    ora = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, extended=True)
    assert (art.info.K, art.info.G, art.info.knot_span) == (s.G + 6, s.G, lk.SPAN_EXTENDED)
    np.testing.assert_array_equal(art.knots, s.ext_knots)
    np.testing.assert_array_equal(art.q, ora.q)
    np.testing.assert_array_equal(art.scale.view(np.uint32), ora.scale.view(np.uint32))
    np.testing.assert_array_equal(art.y_min.view(np.uint32), ora.y_min.view(np.uint32))
    assert art.info.t0 == s.ext_knots[0] and art.info.tK == s.ext_knots[-1]
    with pytest.raises(lk.LutKanError) as e:                      # G + 2p segments must fit the kernels' knot table
        big = random_layer(96, 1, 1, 60, 2, scheme, CLOSED, CLIP_X, 4).layers[0]
        lk.lutkan_compile(1, 1, 60, 3, big.ext_knots, big.coef, 2, scheme, CLOSED, CLIP_X, knot_span=lk.SPAN_EXTENDED)
    assert str(e.value).startswith("[-5]")


@pytest.mark.parametrize("scheme,extended,half,base", [(SYM_INT8, False, False, False), (ASYM_UINT8, True, True, True)])
def test_knots_per_input_compile_like_the_oracle(scheme, extended, half, base, tmp_path):
    """One knot vector per input dimension (Sec. 6.2): codes, parameters and knot rows bit-identical to the oracle's,
    the byte accounting counts d knot vectors, and the NPZ round trip keeps the [d, K+1] knots."""
    s = per_input_layer(98, 5, 70, 6, 16, scheme, HALF_OPEN, ZERO_SPLINE, 4, with_base=base).layers[0]
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, s.boundary, s.oob, edge_scales=s.edge_scales,
                            param_dtype=int(half), knot_span=int(extended), knots_per_input=True, n_threads=3)
    ora = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, param_fp16=half, extended=extended,
                               per_input=True)
    I = art.info
    K = s.G + 6 if extended else s.G
    assert (I.knots_per_input, I.K) == (1, K) and art.knots.shape == (s.d, K + 1) and art.ext_knots.shape == (s.d, s.G + 7)
    np.testing.assert_array_equal(art.knots, ora.knots)
    np.testing.assert_array_equal(art.ext_knots, s.ext_knots)
    np.testing.assert_array_equal(art.q, ora.q)
    np.testing.assert_array_equal(art.scale.view(np.uint32), ora.scale.view(np.uint32))
    np.testing.assert_array_equal(art.y_min.view(np.uint32), ora.y_min.view(np.uint32))
    E = s.d * s.m
    assert I.artifact_bytes == E * K * s.L + 2 * E * K * (2 if half else 4) + 4 * s.d * (K + 1) + (12 * E if base else 0)
    assert (I.t0, I.tK) == (art.knots[0, 0], art.knots[0, -1])
    # the tables of input i are those of a single-input layer on knot vector i
    one = lk.lutkan_compile(1, s.m, s.G, s.p, s.ext_knots[2], s.coef[2], s.L, scheme, s.boundary, s.oob,
                            edge_scales=None if not base else tuple(a[2] for a in s.edge_scales),
                            param_dtype=int(half), knot_span=int(extended))
    np.testing.assert_array_equal(art.table.reshape(I.n_tiles, s.d, I.blob_bytes)[:, 2], one.table.reshape(I.n_tiles, 1, I.blob_bytes)[:, 0])
    path = str(tmp_path / "per_input.npz")
    art.save(path)
    back = lk.lutkan_artifact_load(path)
    assert back.info.knots_per_input == 1
    for name in ("q", "scale", "y_min", "knots", "table"):
        np.testing.assert_array_equal(getattr(back, name), getattr(art, name), err_msg=name)
    bad = s.ext_knots.copy()
    bad[3, 4] = bad[3, 3]
    with pytest.raises(lk.LutKanError) as e:
        lk.lutkan_compile(s.d, s.m, s.G, s.p, bad, s.coef, s.L, scheme, s.boundary, s.oob, knots_per_input=True)
    assert str(e.value).startswith("[-1]") and "vector 3" in str(e.value)
    bad_rows = art.knots.copy()
    bad_rows[4, 1] = np.nan
    with pytest.raises(lk.LutKanError) as e:
        lk.lutkan_artifact_from_arrays(s.d, s.m, bad_rows, art.q, art.scale, art.y_min, s.boundary, s.oob,
                                       edge_scales=art.edge_scales, param_dtype=int(half), knots_per_input=True)
    assert str(e.value).startswith("[-1]") and "vector 4" in str(e.value)
    dl = binding._DevLayer()
    assert lk.load_library().lutkan_dev_layer_init(art._h, C.byref(dl)) == 0
    assert dl.knots_per_input == 1 and not dl.input_knots and not dl.table


def test_tile_width_follows_the_table_size():
    """The widest power of two in 4..64 whose slice fits 72 KiB of LDS (two slices and the record buffers in the 160 KiB
    of a compute unit; 64 KiB with the base branch, whose records are twice as large); 32 (gather kernel) if not even
    4 columns fit.  The B-spline table's tiles go up to 128 columns."""
    rng = np.random.Generator(np.random.PCG64(3))
    for G, L, m, want in ((8, 64, 300, 64), (8, 128, 300, 64), (9, 128, 300, 32), (16, 128, 300, 32), (32, 128, 300, 16), (64, 200, 300, 4),
                          (64, 512, 300, 32), (64, 512, 10, 16), (8, 16, 300, 64), (8, 16, 5, 8), (32, 128, 3, 4)):
        tau = np.linspace(-1.0, 1.0, G + 7).astype(np.float32)
        art = lk.lutkan_compile(1, m, G, 3, tau, rng.normal(size=(1, m, G + 3)).astype(np.float32), L, SYM_INT8, CLOSED, CLIP_X)
        I = art.info
        assert I.jt == want, (G, L, m, I.jt, want)
        assert I.n_tiles == -(-m // I.jt) and I.table_bytes == I.n_tiles * I.blob_bytes
        assert I.coef_jt == min(128, max(4, 1 << (m - 1).bit_length())) and I.coef_n_tiles == -(-m // I.coef_jt)
        assert (I.blob_bytes <= 72 * 1024) == (not (G == 64 and L == 512))
    # with the base branch the records are 16 bytes: 64 KiB per slice, so the 1026-row table takes 32-column tiles
    tau = np.linspace(-1.0, 1.0, 8 + 7).astype(np.float32)
    coef = rng.normal(size=(1, 300, 8 + 3)).astype(np.float32)
    based = lk.lutkan_compile(1, 300, 8, 3, tau, coef, 128, SYM_INT8, CLOSED, CLIP_X, edge_scales=draw_edge_scales(rng, 1, 300))
    assert based.info.jt == 32 and 2 * based.info.blob_bytes > 64 * 1024


def test_table9_artifact_bytes_from_the_compiler():
    """Table 9 (Sec. 8.6): LUT artifact bytes of the case study's layers [78,32,16,1], grid 5, cubic, L = 64.  The
    compiler reproduces every row with the LUT over the extended knot vector and float16 scale / y_min."""
    gold = os.path.join(ROOT, "tests", "golden", "table9_artifact_bytes.txt")
    rows = [[int(v) for v in l.split()] for l in open(gold) if l[0] != "#"]
    widths = [78, 32, 16, 1]
    rng = np.random.Generator(np.random.PCG64(9))
    total = 0
    for (d, m), (E, K, L, nbytes) in zip(zip(widths[:-1], widths[1:]), rows):
        assert d * m == E
        s = random_layer(int(rng.integers(1 << 30)), d, m, 5, L, ASYM_UINT8, CLOSED, CLIP_X, 2).layers[0]
        art = lk.lutkan_compile(d, m, 5, 3, s.ext_knots, s.coef, L, ASYM_UINT8, CLOSED, CLIP_X,
                                param_dtype=lk.PARAM_FP16, knot_span=lk.SPAN_EXTENDED)
        assert art.info.K == K and art.info.artifact_bytes == nbytes
        total += art.info.artifact_bytes
    assert total == 2262096                                          # the table's "LUT Total"


def test_m0_is_only_touched_by_the_lds_dma_helper(tmp_path):
    """The LDS-DMA copy helper writes M0 inside an inline-asm block and declares it clobbered.  That is only sound
    while the compiler itself keeps nothing in M0 in the kernels that use the helper: check the generated gfx950
    assembly (every mention of m0 in a tiled kernel lies inside an inline-asm block)."""
    import subprocess
    from paper_2601_03332_amd import build as lib_build
    lines = []
    for name in ("lutkan_kernels", "bspline_kernels"):
        out = tmp_path / (name + ".s")
        src = os.path.join(ROOT, "paper_2601_03332_amd", "csrc", name + ".hip")
        cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + lib_build.HIPCC_FLAGS + \
              ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2601_03332_amd", "csrc"),
               "-x", "hip", "--cuda-device-only", "-S", src, "-o", str(out)]
        subprocess.run(cmd, check=True, capture_output=True)
        lines += open(out).readlines()
    kernels, inside_asm, current = 0, False, None
    for line in lines:
        text = line.strip()
        if re.match(r"_Z\S*tiled_kernel\S*:", text):
            current, kernels = text.split(":")[0], kernels + 1
        elif text.startswith(".Lfunc_end"):
            current = None
        elif text.startswith(";;#ASMSTART"):
            inside_asm = True
        elif text.startswith(";;#ASMEND"):
            inside_asm = False
        elif current and not text.startswith(";") and re.search(r"\bm0\b", text.split(";")[0]):
            assert inside_asm, f"compiler-generated use of m0 in {current}: {text}"
    assert kernels > 50                                              # every LUT and B-spline tiled variant was seen


def test_host_compile_matches_the_oracle_on_random_shapes():
    """Forty layers with random shapes, grids, table sizes and options: codes, parameters and knots bit-identical to
    the oracle's, rebuilt artifacts byte-identical to compiled ones."""
    rng = np.random.Generator(np.random.PCG64(77))
    for it in range(40):
        G = int(rng.choice([1, 2, 3, 5, 8, 13, 31, 58]))
        L = int(rng.choice([2, 3, 7, 16, 33, 64, 200]))
        d, m = int(rng.integers(1, 9)), int(rng.choice([1, 2, 3, 5, 8, 15, 16, 17, 40, 70, 130]))
        scheme = int(rng.integers(0, 2))
        half, extended, base = bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        s = random_layer(3000 + it, d, m, G, L, scheme, CLOSED, CLIP_X, 2, uniform=bool(rng.integers(0, 2)), with_base=base).layers[0]
        art = lk.lutkan_compile(d, m, G, 3, s.ext_knots, s.coef, L, scheme, CLOSED, CLIP_X, edge_scales=s.edge_scales,
                                param_dtype=int(half), knot_span=int(extended), n_threads=int(rng.integers(1, 5)))
        ora = oracle.compile_layer(d, m, G, 3, s.ext_knots, s.coef, L, scheme, param_fp16=half, extended=extended)
        what = f"case {it}: d={d} m={m} G={G} L={L} scheme={scheme} half={half} extended={extended} base={base}"
        np.testing.assert_array_equal(art.q, ora.q, err_msg=what)
        np.testing.assert_array_equal(art.scale.view(np.uint32), ora.scale.view(np.uint32), err_msg=what)
        np.testing.assert_array_equal(art.y_min.view(np.uint32), ora.y_min.view(np.uint32), err_msg=what)
        np.testing.assert_array_equal(art.knots, ora.knots, err_msg=what)
        back = lk.lutkan_artifact_from_arrays(d, m, art.knots, art.q, art.scale, art.y_min, CLOSED, CLIP_X,
                                              edge_scales=art.edge_scales, param_dtype=int(half))
        np.testing.assert_array_equal(back.table, art.table, err_msg=what)
        assert back.info.blob_bytes == art.info.blob_bytes and back.info.jt == art.info.jt


def test_bench_refuses_more_than_one_gpu():
    """The measurement script is single-GPU by design and says so (no GPU is touched before the check)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "single-GPU" in (r.stderr + r.stdout)


def test_product_package_does_not_touch_the_oracle():
    """Nothing under the product package, the input generators or the build script may import or run the oracle."""
    import glob
    files = glob.glob(os.path.join(ROOT, "paper_2601_03332_amd", "**", "*"), recursive=True) + \
        glob.glob(os.path.join(ROOT, "lutkan_inputs", "*.py")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    checked = 0
    for path in files:
        if not path.endswith((".py", ".hip", ".cpp", ".h")):
            continue
        text = open(path).read()
        checked += 1
        assert "import oracle" not in text and "from oracle" not in text and "lutkan_oracle" not in text and "lko_" not in text, path
    assert checked >= 10
