"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bar (stated by the benchmark spec): segment index k, LUT index l0, the domain predicate In(x) and the integer
codes bit-exact; outputs within |dy| <= 1e-5 * sum_i |phi_ij(x_i)| + 1e-6 (fp32).  The interpolation weight w is
produced by the same IEEE fp32 operations on both sides and is compared bit-exactly as well.
"""
from types import SimpleNamespace

import numpy as np
import pytest

import oracle
from lutkan_inputs import (ASYM_UINT8, CLIP_X, CLOSED, HALF_OPEN, SYM_INT8, ZERO_SPLINE, case_a, cfg1, cfg2, cfg3, cfg4,
                           cfg5, random_layer)
from lutkan_inputs import per_input_layer

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2601_03332_amd as lk  # noqa: E402

DEV = "cuda:0"
RTOL, ATOL = 1e-5, 1e-6


def _say(msg):
    print(msg, flush=True)


_COMPILED = {}


def _compile_both(s, param_fp16=False):
    """Library artifact + oracle artifact for a layer spec; the codes must already agree bit for bit.
    Cached per table content (the contract fields do not change the tables)."""
    key = (s.d, s.m, s.G, s.L, s.scheme, hash(s.coef.tobytes()), hash(s.ext_knots.tobytes()), param_fp16, s.per_input,
           None if s.edge_scales is None else hash(b"".join(a.tobytes() for a in s.edge_scales)))
    if key not in _COMPILED:
        if len(_COMPILED) > 4:
            _COMPILED.clear()
        art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob,
                                edge_scales=s.edge_scales, param_dtype=lk.PARAM_FP16 if param_fp16 else lk.PARAM_FP32,
                                knots_per_input=s.per_input)
        ora = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, param_fp16=param_fp16,
                                   per_input=s.per_input)
        assert np.array_equal(art.q, ora.q) and np.array_equal(art.scale, ora.scale) and np.array_equal(art.y_min, ora.y_min)
        _COMPILED[key] = (art, ora)
    return _COMPILED[key]


def _device_layer(art, s, algo=lk.ALGO_AUTO, wide=None):
    return art.to_device(DEV, algo, wide=wide).with_contract(s.boundary, s.oob)


def _assert_close(y_gpu, ref, what):
    err = np.abs(y_gpu.astype(np.float64) - ref.y.astype(np.float64))
    tol = RTOL * ref.A + ATOL
    nan_ok = np.isnan(y_gpu) == np.isnan(ref.y)
    assert nan_ok.all(), f"{what}: NaN pattern differs"
    bad = np.nan_to_num(err, nan=0.0) > np.nan_to_num(tol, nan=np.inf)
    assert not bad.any(), f"{what}: {bad.sum()} outputs out of tolerance, worst ratio {np.nanmax(err / tol):.3g}"
    return float(np.nanmax(err / tol))


def _check_layer(s, x, algo, codes=False, what="", param_fp16=False, wide=None):
    art, ora = _compile_both(s, param_fp16)
    layer = _device_layer(art, s, algo, wide)
    xg = torch.from_numpy(x).to(DEV)
    _say(f"case {what} d={s.d} m={s.m} K={s.G} L={s.L} scheme={s.scheme} boundary={s.boundary} oob={s.oob} "
         f"B={x.shape[0]} algo={algo} jt={art.info.jt} param_fp16={param_fp16} wide={wide}")
    y, k, l0, inside, w, q01 = lk.lutkan_forward_trace(layer, xg, codes=codes)
    stats = torch.zeros(2, dtype=torch.int64, device=DEV)
    y2 = lk.lutkan_forward(layer, xg, stats=stats)
    torch.cuda.synchronize()
    ref = oracle.lut_forward(ora, s.boundary, s.oob, x, trace=True, codes=codes, edge_scalars=s.edge_scales)
    np.testing.assert_array_equal(k.cpu().numpy(), ref.k)
    np.testing.assert_array_equal(l0.cpu().numpy(), ref.l0)
    np.testing.assert_array_equal(inside.cpu().numpy(), ref.inside)
    np.testing.assert_array_equal(w.cpu().numpy().view(np.uint32), ref.w.view(np.uint32))
    if codes:
        np.testing.assert_array_equal(q01.cpu().numpy(), ref.q01)
    worst = _assert_close(y.cpu().numpy(), ref, what)
    worst = max(worst, _assert_close(y2.cpu().numpy(), ref, what + " (plain launch)"))
    if not codes and algo != lk.ALGO_AUTO:              # a named kernel: trace and plain launch are the same arithmetic
        assert torch.equal(y, y2) or np.array_equal(np.isnan(y.cpu().numpy()), np.isnan(y2.cpu().numpy()))
    st = stats.cpu().numpy()
    assert (int(st[0]), int(st[1])) == (ref.oob_count, ref.oob_any_rows)
    return worst


def test_cfg1_tiny_layer_with_codes():
    w = cfg1()
    _check_layer(w.layers[0], w.x, lk.ALGO_GATHER, codes=True, what=w.name)


PROPERTY_CASES = [
    # seed, d, m, G, L, scheme, boundary, oob, B, uniform
    (101, 1, 1, 3, 2, SYM_INT8, CLOSED, CLIP_X, 1, True),
    (102, 1, 5, 5, 16, ASYM_UINT8, HALF_OPEN, CLIP_X, 33, False),
    (103, 7, 1, 4, 32, SYM_INT8, HALF_OPEN, ZERO_SPLINE, 257, True),
    (104, 5, 3, 6, 33, ASYM_UINT8, CLOSED, ZERO_SPLINE, 100, False),
    (105, 13, 17, 11, 64, SYM_INT8, CLOSED, CLIP_X, 513, False),
    (106, 9, 70, 5, 128, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 65, True),
    (107, 3, 130, 8, 16, SYM_INT8, HALF_OPEN, CLIP_X, 31, False),
    (108, 20, 64, 5, 64, ASYM_UINT8, CLOSED, CLIP_X, 300, True),
    (109, 6, 200, 64, 8, SYM_INT8, CLOSED, ZERO_SPLINE, 129, False),
    (110, 70, 2, 5, 64, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 5000, True),     # inputs split into chunks, 4-column tile
    (111, 130, 9, 7, 32, SYM_INT8, CLOSED, CLIP_X, 3001, False),            # 16-column tile, 8 chunks
    (112, 33, 30, 9, 16, SYM_INT8, HALF_OPEN, CLIP_X, 40000, True),         # 32-column tile, many row tiles
]


@pytest.mark.parametrize("case", PROPERTY_CASES, ids=lambda c: f"seed{c[0]}")
def test_property_layers_gather_with_codes(case):
    seed, d, m, G, L, scheme, boundary, oob, B, uniform = case
    w = random_layer(seed, d, m, G, L, scheme, boundary, oob, B, uniform=uniform)
    _check_layer(w.layers[0], w.x, lk.ALGO_GATHER, codes=(B * d * m <= 2_000_000), what=w.name)
    _check_layer(w.layers[0], w.x, lk.ALGO_TILED, what=w.name)          # narrow column tiles: 4..64 columns


TILED_CASES = [
    # seed, d, m, G, L, scheme, boundary, oob, B
    (201, 17, 128, 5, 32, SYM_INT8, CLOSED, CLIP_X, 700),
    (202, 33, 130, 8, 64, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 1025),
    (203, 5, 70, 10, 64, SYM_INT8, HALF_OPEN, ZERO_SPLINE, 64),
    (204, 40, 300, 6, 16, ASYM_UINT8, CLOSED, CLIP_X, 4099),
    (205, 64, 256, 8, 128, SYM_INT8, CLOSED, ZERO_SPLINE, 2500),     # slice too big for 128-wide tiles -> 64-wide
    (206, 64, 256, 8, 128, ASYM_UINT8, HALF_OPEN, CLIP_X, 9000),
    (207, 3, 1000, 10, 64, SYM_INT8, CLOSED, CLIP_X, 20000),         # enough rows for the 32-rows-per-wave variant
    (208, 1, 128, 2, 2, ASYM_UINT8, CLOSED, CLIP_X, 1),
    (209, 7, 70, 16, 128, SYM_INT8, CLOSED, CLIP_X, 1500),           # 2048 table rows: 16-column tiles of a wide layer
    (210, 5, 50, 32, 128, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 2100), # 4096 table rows: 8-column tiles, ragged last tile
    (211, 3, 21, 64, 200, SYM_INT8, HALF_OPEN, CLIP_X, 300),         # 12800 table rows: 4-column tiles
    (213, 5000, 4, 3, 8, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 50),    # very many inputs: 79 locate tiles, many chunks
    (214, 2, 5000, 3, 8, SYM_INT8, CLOSED, CLIP_X, 33),              # very many outputs: 40 column tiles
]


@pytest.mark.parametrize("case", TILED_CASES, ids=lambda c: f"seed{c[0]}")
def test_property_layers_tiled(case):
    seed, d, m, G, L, scheme, boundary, oob, B = case
    w = random_layer(seed, d, m, G, L, scheme, boundary, oob, B, uniform=(seed % 2 == 0))
    _check_layer(w.layers[0], w.x, lk.ALGO_TILED, what=w.name)
    _check_layer(w.layers[0], w.x, lk.ALGO_GATHER, what=w.name)


WIDE_CASES = [
    # seed, d, m, G, L, scheme, boundary, oob, B, with_base     64-column tiles whose wide slice (2 bytes per code) fits the LDS twice
    (701, 17, 128, 5, 32, SYM_INT8, CLOSED, CLIP_X, 700, False),
    (702, 33, 130, 8, 64, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 1025, False),     # 514 code rows: the largest wide slices; ragged last tile
    (703, 64, 256, 8, 64, SYM_INT8, CLOSED, ZERO_SPLINE, 2500, False),
    (704, 40, 300, 6, 16, ASYM_UINT8, CLOSED, CLIP_X, 4099, False),
    (705, 1, 64, 2, 2, ASYM_UINT8, CLOSED, CLIP_X, 1, False),
    (706, 300, 64, 5, 32, SYM_INT8, HALF_OPEN, CLIP_X, 9000, False),            # many inputs: chunks and the summing pass
    (707, 3, 1000, 10, 50, SYM_INT8, HALF_OPEN, ZERO_SPLINE, 20000, False),     # 16 column tiles, three slice buffers
    (708, 64, 128, 5, 32, ASYM_UINT8, CLOSED, CLIP_X, 70000, True),             # spline_component: base branch as a product, 8-byte records
    (709, 24, 70, 6, 16, SYM_INT8, CLOSED, ZERO_SPLINE, 3000, True),            # spline_component with 16-byte records: byte form or fp32 values
    (713, 40, 128, 5, 32, ASYM_UINT8, HALF_OPEN, CLIP_X, 20000, True),          # the same at 16 row steps per wave
    (710, 64, 256, 8, 32, SYM_INT8, HALF_OPEN, CLIP_X, 16384 + 3, False),       # large enough for the launch planning to pick the wide form
    (711, 20, 192, 5, 32, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 5001, False),     # masked inputs on a layer that has both wide forms
    (712, 96, 64, 3, 90, SYM_INT8, HALF_OPEN, ZERO_SPLINE, 33000, False),       # 272 value rows: the largest fp32 slices (two buffers)
]


@pytest.mark.parametrize("cb", [2, 4], ids=["binary16_codes", "fp32_values"])
@pytest.mark.parametrize("case", WIDE_CASES, ids=lambda c: f"seed{c[0]}")
def test_wide_table_form(case, cb):
    """The wide forms of the device table against the oracle, to the bar of every other path.  16-bit codes (no byte
    unpacking in the tiled kernel): the arithmetic after the unpacking is that of the byte form, so with the same launch
    plan the outputs agree bit for bit.  fp32 values (Eq. 10 applied when the table is built, the kernel interpolates
    the values): a different rounding order, so only the oracle is the measure."""
    seed, d, m, G, L, scheme, boundary, oob, B, with_base = case
    w = random_layer(seed, d, m, G, L, scheme, boundary, oob, B, uniform=(seed % 2 == 0), oob_frac=0.3, with_base=with_base)
    s = w.layers[0]
    x = w.x.copy()
    if B > 1:
        x[B // 2, d // 3] = np.nan
    art, ora = _compile_both(s)
    assert art.info.jt == 64
    value_rows_fit = (art.info.K * L + 2 + with_base) * 256 <= 72 * 1024
    if cb == 4 and not value_rows_fit:
        with pytest.raises(lk.LutKanError) as e:
            art.to_device(DEV, wide=4)
        assert "no wide table form of 4 bytes" in str(e.value)
        assert art.to_device(DEV, wide=True).c.wide_code_bytes == 2           # "any": the form the layer has
        return
    wide, byte = _device_layer(art, s, lk.ALGO_TILED_WIDE, wide=cb), _device_layer(art, s, lk.ALGO_TILED, wide=False)
    assert wide.wide_table is not None and byte.wide_table is None and wide.c.wide_code_bytes == cb
    if cb == 2:
        assert wide.wide_table.numel() == art.info.table_bytes + art.info.n_tiles * d * (art.info.K * L + 2) * 64
    else:
        assert wide.wide_table.numel() == art.info.n_tiles * d * (art.info.K * L + 2 + with_base) * 256
        assert art.to_device(DEV, wide=True).c.wide_code_bytes == 4
    xg = torch.from_numpy(x).to(DEV)
    if with_base and B * d * m < 5e8 and cb == 2:
        # 16-byte records (the base branch inside the edge kernel) go with the byte form or with fp32 values
        with pytest.raises(lk.LutKanError) as e:
            lk.lutkan_forward(wide, xg)
        assert str(e.value).startswith("[-5]") and "16-byte records" in str(e.value)
        _check_layer(s, x, lk.ALGO_TILED, what=w.name + " (wide table present, byte form runs)", wide=cb)
        assert "tiled np=" in lk.lutkan_last_plan()
        return
    tag = "tiled wide np=" if cb == 2 else "tiled wide32 np="
    worst = _check_layer(s, x, lk.ALGO_TILED_WIDE, what=w.name + f" (wide form, {cb} bytes per code)", wide=cb)
    y_wide = lk.lutkan_forward(wide, xg)
    plan_wide = lk.lutkan_last_plan()
    y_byte = lk.lutkan_forward(byte, xg)
    plan_byte = lk.lutkan_last_plan()
    _say(f"wide: {plan_wide!r}  byte: {plan_byte!r}  worst error / tolerance {worst:.3g}")
    assert tag in plan_wide and " wide" not in plan_byte
    if cb == 2 and plan_wide.replace("tiled wide", "tiled") == plan_byte:
        assert bool(((y_wide == y_byte) | (torch.isnan(y_wide) & torch.isnan(y_byte))).all())
    # the two phases apart, and the entry point with the built-in scratch, take the same form
    ws = torch.empty(lk.lutkan_forward_workspace_bytes(wide, B), dtype=torch.uint8, device=DEV)
    lk.lutkan_forward_locate(wide, xg, ws)
    y_two = lk.lutkan_forward_edges(wide, B, torch.full((B, m), 3.0, dtype=torch.float32, device=DEV), ws)
    assert bool(((y_two == y_wide) | (torch.isnan(y_two) & torch.isnan(y_wide))).all())
    if lk.lutkan_forward_workspace_bytes(wide, B) <= lk.STATIC_SCRATCH_BYTES:
        y_static = lk.lutkan_forward_static_scratch(wide, xg, torch.full((B, m), -3.0, dtype=torch.float32, device=DEV))
        assert bool(((y_static == y_wide) | (torch.isnan(y_static) & torch.isnan(y_wide))).all())
    # left to the launch planning: 16-bit codes run on large batches of symmetric layers, fp32 values with both schemes
    auto = _device_layer(art, s, lk.ALGO_AUTO, wide=cb)
    lk.lutkan_forward(auto, xg)
    if cb == 2 and scheme == ASYM_UINT8:
        assert " wide" not in lk.lutkan_last_plan(), lk.lutkan_last_plan()
    elif B * d * m >= 2e8:
        assert tag in lk.lutkan_last_plan(), lk.lutkan_last_plan()
    # the default upload: fp32 values where they fit, else 16-bit codes for symmetric layers; layers of some size only
    default = art.to_device(DEV).c.wide_code_bytes
    assert default == (0 if d * m < 4096 else 4 if value_rows_fit else 2 if scheme == SYM_INT8 else 0)


def test_wide_table_form_exists_only_where_it_pays():
    """No wide form on tiles narrower than 64 columns or when two wide slices do not fit the LDS (the widest layer:
    642 code rows); asking for one is an error, the default upload simply goes without."""
    for d, m, G, L in ((8, 32, 5, 16), (4, 1024, 10, 64), (4, 256, 8, 128)):
        w = random_layer(720, d, m, G, L, SYM_INT8, CLOSED, CLIP_X, 8)
        art, _ = _compile_both(w.layers[0])
        assert art.to_device(DEV).wide_table is None
        with pytest.raises(lk.LutKanError):
            art.to_device(DEV, wide=True)


@pytest.mark.parametrize("case", [(731, 5, 130, 6, 16, SYM_INT8, False), (732, 3, 64, 5, 32, ASYM_UINT8, False),
                                  (733, 4, 200, 8, 8, ASYM_UINT8, True), (734, 2, 70, 4, 64, SYM_INT8, True)],
                         ids=lambda c: f"seed{c[0]}")
def test_wide_tables_hold_exactly_what_the_codes_stand_for(case):
    """The two wide forms as built on the device, read back and compared bit for bit with what the oracle's artifact
    arrays say they must hold: the binary16 pattern of q * 2^-24 (sign and magnitude) resp. the fp32 value of Eq. 10,
    fl(y_min + fl(alpha * q)), for every (tile, input, code row, column); the two rows after the last code row and
    the columns past m are zero."""
    seed, d, m, G, L, scheme, half = case
    w = random_layer(seed, d, m, G, L, scheme, CLOSED, CLIP_X, 4)
    s = w.layers[0]
    art, ora = _compile_both(s, param_fp16=half)
    K, jt, n_tiles = art.info.K, art.info.jt, art.info.n_tiles
    assert jt == 64 and K == ora.K
    rows = K * L + 2
    q = ora.q.reshape(d, m, K * L).astype(np.int32)                  # [i][j][row]
    alpha = np.repeat(ora.scale.reshape(d, m, K), L, axis=2)         # the parameters of each row's segment
    y_min = np.repeat(ora.y_min.reshape(d, m, K), L, axis=2)
    values = (y_min + (alpha * q.astype(np.float32)).astype(np.float32)).astype(np.float32)        # two fp32 roundings
    bits16 = np.where(q < 0, 0x8000 | -q, q).astype(np.uint16)
    _say(f"case {w.name} wide table contents, param_fp16={half}")
    for cb, want, dtype in ((2, bits16, np.uint16), (4, values, np.float32)):
        layer = art.to_device(DEV, wide=cb)
        blob = layer.c.wide_blob_bytes
        host = layer.wide_table.cpu().numpy().reshape(n_tiles, d, blob)
        codes_off = blob - (-(-rows * jt * cb // 16) * 16)             # the code rows end the slice (padded to 16 bytes)
        if cb == 4:
            assert codes_off == 0                                    # phi layer: no base row, no parameter rows
        got = np.ascontiguousarray(host[:, :, codes_off:codes_off + rows * jt * cb]).view(dtype).reshape(n_tiles, d, rows, jt)
        full = np.zeros((n_tiles * jt, d, rows), dtype=dtype)
        full[:m, :, :K * L] = np.transpose(want, (1, 0, 2))          # [j][i][row]
        expect = np.transpose(full.reshape(n_tiles, jt, d, rows), (0, 2, 3, 1))                   # [t][i][row][column]
        if cb == 4:
            assert np.array_equal(got, expect)                       # (padding: 0 * -128 under y_min = 0 is +0)
        else:
            pad = np.zeros(expect.shape, dtype=bool)
            pad[:, :, K * L:, :] = True
            pad |= (np.arange(n_tiles * jt).reshape(n_tiles, jt) >= m)[:, None, None, :]
            assert np.array_equal(got[~pad], expect[~pad])
            # padding holds a code byte of 0 or the code 0 (excess-128: byte 0 reads as -128, under alpha = 0)
            assert np.isin(got[pad], (0, 0x8080)).all()
        if cb == 2:                                                  # everything before the code rows is the byte table's
            byte = np.asarray(art.table).reshape(n_tiles, d, art.info.blob_bytes)
            assert np.array_equal(host[:, :, :codes_off], byte[:, :, :codes_off])


@pytest.mark.parametrize("base", [False, True], ids=["phi", "spline_component"])
def test_largest_slices_with_the_largest_record_buffers_fill_the_lds(base):
    """The LDS budget at its edge: 64-column slices of 72 KiB (64 KiB with the base branch, whose records are 16 bytes)
    at a batch large enough for 16 row steps per wave, so that two slice buffers and the record buffers take all but
    a few hundred bytes of the 160 KiB of a compute unit.  Sampled rows against the oracle."""
    L = 122 if base else 139         # 8 L + 2 code rows of 64 bytes + parameters: just under the budget
    B = 262144 + 3
    w = random_layer(230 + base, 4, 64, 8, L, SYM_INT8, HALF_OPEN, ZERO_SPLINE, B, with_base=base)
    s = w.layers[0]
    art, ora = _compile_both(s)
    budget = (64 if base else 72) * 1024
    assert art.info.jt == 64 and budget - 1024 < art.info.blob_bytes <= budget
    layer = _device_layer(art, s)
    xg = torch.from_numpy(w.x).to(DEV)
    _say(f"case {w.name} B={B} slice of {art.info.blob_bytes} bytes")
    y = lk.lutkan_forward(layer, xg)
    assert lk.lutkan_last_plan().startswith("locate; tiled np=16 "), lk.lutkan_last_plan()
    lds = 2 * art.info.blob_bytes + 16 * 2 * 64 * (16 if base else 8)
    assert 160 * 1024 - 1024 < lds <= 160 * 1024
    rows = np.unique(np.concatenate([np.random.Generator(np.random.PCG64(5)).integers(0, B, size=1500), [0, B - 1]]))
    ref = oracle.lut_forward(ora, s.boundary, s.oob, w.x[rows], edge_scalars=s.edge_scales)
    _assert_close(y[torch.from_numpy(rows).to(DEV)].cpu().numpy(), ref, w.name)


def test_table_too_large_for_any_tile_runs_on_the_gather_kernel():
    """32768 table rows: not even a 4-column slice fits the LDS budget; AUTO takes the gather kernel on 32-column
    tiles, and asking for the tiled kernel is an error, not a silent fallback."""
    w = random_layer(212, 2, 40, 64, 512, ASYM_UINT8, CLOSED, ZERO_SPLINE, 257)
    s = w.layers[0]
    _check_layer(s, w.x, lk.ALGO_AUTO, what=w.name)
    art = _compile_both(s)[0]
    assert art.info.jt == 32 and art.info.blob_bytes > 72 * 1024
    with pytest.raises(lk.LutKanError) as e:
        lk.lutkan_forward(_device_layer(art, s, lk.ALGO_TILED), torch.from_numpy(w.x).to(DEV))
    assert str(e.value).startswith("[-5]")


FP16_PARAM_CASES = [
    # seed, d, m, G, L, scheme, boundary, oob, B          float16 scale / y_min (Sec. 4.6)
    (601, 4, 3, 5, 16, SYM_INT8, CLOSED, CLIP_X, 200),                # 4-column tile
    (602, 78, 16, 5, 64, ASYM_UINT8, CLOSED, CLIP_X, 3000),           # 16-column tile, inputs split
    (603, 33, 130, 8, 64, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 1025),  # 128-column tiles, ragged last tile
    (604, 64, 256, 8, 128, SYM_INT8, CLOSED, ZERO_SPLINE, 2500),      # 64-column tiles
    (605, 40, 300, 6, 16, SYM_INT8, HALF_OPEN, CLIP_X, 4099),
    (606, 20, 64, 10, 64, ASYM_UINT8, CLOSED, CLIP_X, 17000),         # 16 row steps per wave
]


@pytest.mark.parametrize("case", FP16_PARAM_CASES, ids=lambda c: f"seed{c[0]}")
def test_fp16_parameters(case):
    seed, d, m, G, L, scheme, boundary, oob, B = case
    w = random_layer(seed, d, m, G, L, scheme, boundary, oob, B, uniform=(seed % 2 == 0))
    _check_layer(w.layers[0], w.x, lk.ALGO_TILED, what=w.name, param_fp16=True)
    _check_layer(w.layers[0], w.x, lk.ALGO_GATHER, codes=(B * d * m <= 2_000_000), what=w.name, param_fp16=True)


@pytest.mark.parametrize("case", FP16_PARAM_CASES, ids=lambda c: f"seed{c[0]}")
def test_fp16_parameters_with_spline_component(case):
    """The deployment combination of Sec. 8: asymmetric or symmetric codes, float16 scale / y_min, Eq. 2's base branch
    and per-edge scalars; the scalars multiply the dequantised value, the parameters stay the rounded ones."""
    seed, d, m, G, L, scheme, boundary, oob, B = case
    w = random_layer(seed + 50, d, m, G, L, scheme, boundary, oob, B, uniform=(seed % 2 == 1), with_base=True)
    _check_layer(w.layers[0], w.x, lk.ALGO_TILED, what=w.name, param_fp16=True)
    _check_layer(w.layers[0], w.x, lk.ALGO_GATHER, codes=(B * d * m <= 2_000_000), what=w.name, param_fp16=True)


PER_INPUT_CASES = [
    # seed, d, m, G, L, scheme, boundary, oob, B, with_base, param_fp16
    (801, 1, 1, 3, 2, SYM_INT8, CLOSED, CLIP_X, 1, False, False),
    (802, 3, 5, 5, 16, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 300, False, False),      # 16 inputs per locate block
    (803, 20, 16, 8, 64, SYM_INT8, HALF_OPEN, CLIP_X, 1025, True, False),           # 32 inputs per locate block
    (804, 70, 130, 10, 32, ASYM_UINT8, CLOSED, ZERO_SPLINE, 2100, False, True),     # two blocks of 64 inputs, ragged
    (805, 33, 64, 64, 8, SYM_INT8, CLOSED, CLIP_X, 700, True, True),                # the longest knot vectors
    (806, 129, 40, 6, 128, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 4099, True, False),
]


@pytest.mark.parametrize("case", PER_INPUT_CASES, ids=lambda c: f"seed{c[0]}")
def test_one_knot_vector_per_input(case):
    """Sec. 6.2's knot grid "shared per input dimension": every input is located, clipped and masked on its own knot
    vector (different domains, uniform and non-uniform); LUT layer (both kernels, counters) and B-spline layer."""
    seed, d, m, G, L, scheme, boundary, oob, B, with_base, half = case
    w = per_input_layer(seed, d, m, G, L, scheme, boundary, oob, B, with_base=with_base)
    s = w.layers[0]
    _check_layer(s, w.x, lk.ALGO_AUTO, what=w.name, param_fp16=half)
    _check_layer(s, w.x, lk.ALGO_GATHER, codes=(B * d * m <= 2_000_000), what=w.name, param_fp16=half)
    art = _compile_both(s, half)[0]
    xg = torch.from_numpy(w.x).to(DEV)
    refb = oracle.bspline_forward(d, m, G, s.p, s.ext_knots, s.coef, boundary, oob, w.x, edge_scalars=s.edge_scales, per_input=True)
    for algo in (lk.ALGO_AUTO, lk.ALGO_GATHER):
        yb = lk.bspline_kan_forward(art.bspline_to_device(DEV, algo), xg)
        torch.cuda.synchronize()
        _assert_close(yb.cpu().numpy(), refb, f"{w.name} bspline algo={algo}")
    # the error statistics with every input's own domain
    y_lut = lk.lutkan_forward(_device_layer(art, s), xg)
    dom = torch.from_numpy(np.ascontiguousarray(art.knots[:, [0, -1]])).to(DEV)
    got = lk.lutkan_error_stats(y_lut, yb, xg, 0.0, 0.0, boundary, input_domain=dom)
    want = oracle.error_stats(y_lut.cpu().numpy(), yb.cpu().numpy(), w.x, art.knots[:, 0], art.knots[:, -1], boundary)
    _same_error_summary(got, want)


def test_per_input_layer_without_its_knot_table_is_refused():
    w = per_input_layer(810, 4, 4, 5, 8, SYM_INT8, CLOSED, CLIP_X, 16)
    s = w.layers[0]
    art = _compile_both(s)[0]
    layer, bl = art.to_device(DEV), art.bspline_to_device(DEV)
    layer.c.input_knots = None
    bl.c.input_ext_knots = None
    xg = torch.from_numpy(w.x).to(DEV)
    for call in (lambda: lk.lutkan_forward(layer, xg), lambda: lk.bspline_kan_forward(bl, xg)):
        with pytest.raises(lk.LutKanError) as e:
            call()
        assert str(e.value).startswith("[-1]")


def test_loaded_artifact_runs_like_the_compiled_one(tmp_path):
    """An artifact written to NPZ + manifest and read back (Sec. 4.6) gives bit-identical outputs and counters."""
    w = random_layer(611, 20, 150, 6, 32, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 3000)
    s = w.layers[0]
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob)
    path = str(tmp_path / "layer.npz")
    art.save(path)
    back = lk.lutkan_artifact_load(path)
    xg = torch.from_numpy(w.x).to(DEV)
    _say(f"case {w.name} loaded artifact jt={back.info.jt}")
    st1, st2 = torch.zeros(2, dtype=torch.int64, device=DEV), torch.zeros(2, dtype=torch.int64, device=DEV)
    y1 = lk.lutkan_forward(art.to_device(DEV), xg, stats=st1)
    y2 = lk.lutkan_forward(back.to_device(DEV), xg, stats=st2)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2) and torch.equal(st1, st2)
    ora = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme)
    _assert_close(y2.cpu().numpy(), oracle.lut_forward(ora, s.boundary, s.oob, w.x), w.name)


EXTENDED_CASES = [
    # seed, d, m, G, L, scheme, boundary, oob, B, uniform          LUT and B-spline layer over the extended knot vector
    (801, 3, 5, 5, 16, SYM_INT8, CLOSED, CLIP_X, 300, True),
    (802, 10, 130, 4, 32, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 1500, False),
    (803, 20, 64, 8, 64, SYM_INT8, CLOSED, ZERO_SPLINE, 2000, False),
    (804, 7, 9, 1, 8, ASYM_UINT8, HALF_OPEN, CLIP_X, 500, True),       # one grid interval: R = 4 coefficients
    (805, 5, 40, 58, 4, SYM_INT8, CLOSED, CLIP_X, 700, True),         # K = 64 segments
]


@pytest.mark.parametrize("case", EXTENDED_CASES, ids=lambda c: f"seed{c[0]}")
def test_extended_knot_span(case):
    seed, d, m, G, L, scheme, boundary, oob, B, uniform = case
    w = random_layer(seed, d, m, G, L, scheme, boundary, oob, B, uniform=uniform)
    s = w.layers[0]
    tau = s.ext_knots
    rng = np.random.Generator(np.random.PCG64(seed))
    span = float(tau[-1] - tau[0])
    x = rng.uniform(tau[0] - 0.1 * span, tau[-1] + 0.1 * span, size=(B, d)).astype(np.float32)
    pick = rng.integers(0, B * d, size=B * d // 8)                    # exact extended knots and their neighbours
    vals = tau[rng.integers(0, tau.size, size=pick.size)]
    nudge = rng.integers(-1, 2, size=pick.size)
    x.reshape(-1)[pick] = np.where(nudge < 0, np.nextafter(vals, np.float32(-np.inf)),
                                   np.where(nudge > 0, np.nextafter(vals, np.float32(np.inf)), vals)).astype(np.float32)
    art = lk.lutkan_compile(d, m, G, 3, tau, s.coef, L, scheme, boundary, oob, knot_span=lk.SPAN_EXTENDED)
    ora = oracle.compile_layer(d, m, G, 3, tau, s.coef, L, scheme, extended=True)
    assert np.array_equal(art.q, ora.q) and np.array_equal(art.scale, ora.scale) and np.array_equal(art.y_min, ora.y_min)
    xg = torch.from_numpy(x).to(DEV)
    _say(f"case extended {w.name} K={art.info.K} jt={art.info.jt}")
    y, k, l0, inside, wgt, _ = lk.lutkan_forward_trace(art.to_device(DEV), xg)
    yb = lk.bspline_kan_forward(art.bspline_to_device(DEV), xg)
    yb_g = lk.bspline_kan_forward(art.bspline_to_device(DEV, lk.ALGO_GATHER), xg)
    torch.cuda.synchronize()
    ref = oracle.lut_forward(ora, boundary, oob, x, trace=True)
    np.testing.assert_array_equal(k.cpu().numpy(), ref.k)
    np.testing.assert_array_equal(l0.cpu().numpy(), ref.l0)
    np.testing.assert_array_equal(inside.cpu().numpy(), ref.inside)
    np.testing.assert_array_equal(wgt.cpu().numpy().view(np.uint32), ref.w.view(np.uint32))
    _assert_close(y.cpu().numpy(), ref, w.name)
    refb = oracle.bspline_forward(d, m, G, 3, tau, s.coef, boundary, oob, x, extended=True)
    _assert_close(yb.cpu().numpy(), refb, w.name + " bspline")
    _assert_close(yb_g.cpu().numpy(), refb, w.name + " bspline gather")


def test_special_inputs_nan_inf_all_oob():
    w = random_layer(301, 6, 140, 5, 32, ASYM_UINT8, CLOSED, ZERO_SPLINE, 40)
    x = w.x.copy()
    x[3, 2] = np.nan
    x[5, :] = np.inf
    x[6, :] = -np.inf
    x[7, :] = 1e30
    x[8, 0] = -0.0
    for algo in (lk.ALGO_GATHER, lk.ALGO_TILED):
        for boundary in (HALF_OPEN, CLOSED):
            for oob in (CLIP_X, ZERO_SPLINE):
                s = w.layers[0]
                s.boundary, s.oob = boundary, oob
                _check_layer(s, x, algo, what="special")


def test_domain_ends_at_zero_and_below_and_subnormal_inputs():
    """The safe upper clip value of Eq. 13 in half-open mode is nextafter(t_K, -inf): below t_K = 0 that is the
    smallest negative subnormal, below a negative t_K the next float of larger magnitude.  Shared knots (clip value
    from the host) and one vector per input (clip value computed in the kernel), inputs on and around those values."""
    from lutkan_inputs import LayerSpec, uniform_ext_knots
    rng = np.random.Generator(np.random.PCG64(31))
    G, L, m = 4, 16, 5
    tiny = np.float32(1e-45)                                            # the smallest positive subnormal
    ends = [(-2.0, 0.0), (-3.0, -1.0), (0.0, 2.0), (-1.0, 1.0)]
    specials = []
    for lo, hi in ends:
        for v in (lo, hi):
            v = np.float32(v)
            specials += [v, np.nextafter(v, np.float32(-np.inf)), np.nextafter(v, np.float32(np.inf))]
    specials += [np.float32(0.0), np.float32(-0.0), tiny, -tiny, np.float32(1e-39), np.float32(-1e-39)]
    specials = np.array(specials, dtype=np.float32)
    for boundary in (HALF_OPEN, CLOSED):
        for oob in (CLIP_X, ZERO_SPLINE):
            # one vector per input: the four domains side by side, every special value in every column
            tau = np.stack([uniform_ext_knots(lo, hi, G, 3) for lo, hi in ends])
            coef = rng.normal(size=(4, m, G + 3)).astype(np.float32)
            x = np.tile(specials[:, None], (1, 4))
            _check_layer(LayerSpec(4, m, G, 3, tau, coef, L, SYM_INT8, boundary, oob, per_input=True), x, lk.ALGO_AUTO,
                         what=f"zero-ended domains, per input, b{boundary} o{oob}")
            for row, (lo, hi) in enumerate(ends):                       # the same domains as shared vectors
                _check_layer(LayerSpec(1, m, G, 3, tau[row], coef[row:row + 1], L, SYM_INT8, boundary, oob), x[:, :1].copy(),
                             lk.ALGO_AUTO, what=f"domain [{lo},{hi}] shared b{boundary} o{oob}")


def test_empty_batch_and_argument_errors():
    w = cfg1(B=8)
    s = w.layers[0]
    art, _ = _compile_both(s)
    layer = _device_layer(art, s)
    x0 = torch.empty((0, s.d), dtype=torch.float32, device=DEV)
    y0 = lk.lutkan_forward(layer, x0)
    assert y0.shape == (0, s.m)
    x = torch.from_numpy(w.x).to(DEV)
    with pytest.raises(lk.LutKanError, match="workspace"):
        lk.lutkan_forward(layer, x, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    bad = layer.with_contract(7, CLIP_X)
    with pytest.raises(lk.LutKanError, match="boundary"):
        lk.lutkan_forward(bad, x)
    nul = layer.with_contract(CLOSED, CLIP_X)
    nul.c.table = None
    with pytest.raises(lk.LutKanError, match="table"):
        lk.lutkan_forward(nul, x)
    buf = torch.empty((1 << 18,), dtype=torch.float32, device=DEV)
    rc = lk.load_library().lutkan_forward(layer.c, buf.data_ptr(), 8, buf.data_ptr(), None, buf.data_ptr(), buf.numel() * 4, None)
    assert rc == -1 and "alias" in lk.lutkan_last_error()
    torch.cuda.synchronize()


def test_repeatable_bitwise():
    w = random_layer(401, 50, 256, 8, 64, SYM_INT8, CLOSED, CLIP_X, 3000)
    s = w.layers[0]
    art, _ = _compile_both(s)
    xg = torch.from_numpy(w.x).to(DEV)
    for algo in (lk.ALGO_GATHER, lk.ALGO_TILED):
        layer = _device_layer(art, s, algo)
        a = lk.lutkan_forward(layer, xg).clone()
        b = lk.lutkan_forward(layer, xg)
        assert torch.equal(a, b)


def _chain_check(w, what):
    """Each layer against the oracle on the SAME input (the GPU's own activation of the previous layer), and the
    chained entry point bit-identical to the layer-by-layer GPU calls."""
    arts, layers = [], []
    for s in w.layers:
        art, ora = _compile_both(s)
        arts.append((art, ora))
        layers.append(_device_layer(art, s))
    xg = torch.from_numpy(w.x).to(DEV)
    stats = torch.zeros((len(layers), 2), dtype=torch.int64, device=DEV)
    y_model = lk.lutkan_model_forward(layers, xg, stats=stats)
    cur = xg
    for li, (s, (art, ora), layer) in enumerate(zip(w.layers, arts, layers)):
        _say(f"case {what} layer {li}: {s.d}->{s.m} B={cur.shape[0]}")
        nxt = lk.lutkan_forward(layer, cur)
        x_host = cur.cpu().numpy()
        ref = oracle.lut_forward(ora, s.boundary, s.oob, x_host)
        _assert_close(nxt.cpu().numpy(), ref, f"{what} layer {li}")
        st = stats[li].cpu().numpy()
        assert (int(st[0]), int(st[1])) == (ref.oob_count, ref.oob_any_rows)
        cur = nxt
    assert torch.equal(cur, y_model)


def test_cfg2_tabular_two_layer_chain_full_size():
    _chain_check(cfg2(), "cfg2")


@pytest.mark.parametrize("B", [1, 300, 5000])
def test_cfg2_tabular_chain_at_small_batches(B):
    """Up to about 10000 rows every layer of this network runs as a launch of the chain kernel, and lutkan_model_forward
    runs the whole network as one launch of it: same arithmetic, so still bit-identical to the layer-by-layer calls."""
    _chain_check(cfg2(B=B), f"cfg2 B={B}")


@pytest.mark.parametrize("boundary,oob", [(HALF_OPEN, CLIP_X), (HALF_OPEN, ZERO_SPLINE), (CLOSED, CLIP_X), (CLOSED, ZERO_SPLINE)])
def test_cfg5_deep_chain_robustness_matrix(boundary, oob):
    _chain_check(cfg5(B=16384 + 77, boundary=boundary, oob=oob), f"cfg5 b{boundary} o{oob}")


@pytest.mark.parametrize("L", [16, 32, 64, 128])
@pytest.mark.parametrize("scheme", [SYM_INT8, ASYM_UINT8])
def test_cfg3_sweep_point_reduced_batch(L, scheme):
    w = cfg3(L=L, scheme=scheme, B=1024 + 19)
    _check_layer(w.layers[0], w.x, lk.ALGO_AUTO, what=w.name)


@pytest.mark.parametrize("L", [16, 32, 64, 128])
@pytest.mark.parametrize("scheme", [SYM_INT8, ASYM_UINT8])
def test_cfg3_sweep_point_full_batch_every_row(L, scheme):
    """Every point of the L x scheme sweep at its stated batch (16384 rows, the launch plan a user gets): k, l0, In(x),
    w and the counters bit-exact and every output within the tolerance, on all rows."""
    w = cfg3(L=L, scheme=scheme)
    assert w.x.shape[0] == 16384
    _check_layer(w.layers[0], w.x, lk.ALGO_AUTO, what=w.name)


def _sampled_rows_check(w, n_rows, what, seed=0):
    """Full-size launch (the configuration the benchmark times).  The oracle recomputes a seeded random sample of at
    least n_rows rows (plus the first and the last one): k, l0, In(x), w bit-exact and the outputs of both the traced
    and the plain launch within the tolerance on them; the OOB counters are exact over ALL rows."""
    s = w.layers[0]
    art, ora = _compile_both(s)
    layer = _device_layer(art, s)
    xg = torch.from_numpy(w.x).to(DEV)
    B = w.x.shape[0]
    rng = np.random.Generator(np.random.PCG64(seed))
    rows = np.unique(np.concatenate([rng.choice(B, size=min(B, n_rows), replace=False), [0, B - 1]]))
    _say(f"case {what} full size B={B} sampled rows={rows.size}")
    stats = torch.zeros(2, dtype=torch.int64, device=DEV)
    y = lk.lutkan_forward(layer, xg, stats=stats)
    plan = lk.lutkan_last_plan()
    y_t, k, l0, inside, wgt, _ = lk.lutkan_forward_trace(layer, xg)
    assert lk.lutkan_last_plan() == plan.replace("oob; ", "")           # the traced launch is the plain launch's plan
    torch.cuda.synchronize()
    rows_t = torch.from_numpy(rows).to(DEV)
    ref = oracle.lut_forward(ora, s.boundary, s.oob, w.x[rows], trace=True)
    np.testing.assert_array_equal(k[rows_t].cpu().numpy(), ref.k)
    np.testing.assert_array_equal(l0[rows_t].cpu().numpy(), ref.l0)
    np.testing.assert_array_equal(inside[rows_t].cpu().numpy(), ref.inside)
    np.testing.assert_array_equal(wgt[rows_t].cpu().numpy().view(np.uint32), ref.w.view(np.uint32))
    _assert_close(y[rows_t].cpu().numpy(), ref, what)
    _assert_close(y_t[rows_t].cpu().numpy(), ref, what + " (traced launch)")
    T = ora.knots
    inside_all = (w.x >= T[0]) & (w.x <= T[-1]) if s.boundary == CLOSED else (w.x >= T[0]) & (w.x < T[-1])
    st = stats.cpu().numpy()
    assert int(st[0]) == int((~inside_all).sum()) and int(st[1]) == int((~inside_all).any(axis=1).sum())


@pytest.mark.parametrize("boundary,oob", [(HALF_OPEN, CLIP_X), (HALF_OPEN, ZERO_SPLINE), (CLOSED, CLIP_X), (CLOSED, ZERO_SPLINE)])
def test_cfg5_full_batch_chain_every_row(boundary, oob):
    """cfg5 at its full batch (131072 rows, the launch shapes a user gets) under each of the four boundary x policy
    contracts: every layer against the oracle on ALL rows, fed with the GPU's own activations of the previous layer;
    the per-layer OOB counters exact; the chained entry point bit-identical to the layer-by-layer calls."""
    w = cfg5(boundary=boundary, oob=oob)
    B = w.x.shape[0]
    assert B == 131072
    layers, oras = [], []
    for s in w.layers:
        art, ora = _compile_both(s)
        layers.append(_device_layer(art, s))
        oras.append(ora)
    cur = torch.from_numpy(w.x).to(DEV)
    stats = torch.zeros((len(layers), 2), dtype=torch.int64, device=DEV)
    y_model = lk.lutkan_model_forward(layers, cur, stats=stats)
    for li, (s, layer, ora) in enumerate(zip(w.layers, layers, oras)):
        _say(f"case cfg5 b{boundary} o{oob} full batch layer {li}: {s.d}->{s.m} B={B}")
        nxt = lk.lutkan_forward(layer, cur)
        ref = oracle.lut_forward(ora, s.boundary, s.oob, cur.cpu().numpy())
        _assert_close(nxt.cpu().numpy(), ref, f"cfg5 full layer {li}")
        st = stats[li].cpu().numpy()
        assert (int(st[0]), int(st[1])) == (ref.oob_count, ref.oob_any_rows)
        cur = nxt
    assert torch.equal(cur, y_model)


@pytest.mark.parametrize("B", [1, 7, 64, 100, 256, 4096])
def test_cfg4_wide_layer_every_row(B):
    """The widest workload at its batches of 256 and 4096 rows, and at batches of a few rows, where AUTO runs the
    gather kernel with the inputs split into chunks (partial sums added in chunk order): all rows against the oracle."""
    w = cfg4(B=B)
    _check_layer(w.layers[0], w.x, lk.ALGO_AUTO, what=f"cfg4 B={B}")


@pytest.mark.parametrize("L,scheme,B", [(32, ASYM_UINT8, 200), (48, SYM_INT8, 300)], ids=["L32_uint8_200rows", "L48_int8_300rows"])
def test_table_streaming_from_hbm_runs_with_two_slices_in_flight(L, scheme, B):
    """A table of more than 128 MiB at a few hundred rows: the launch waits for the table to stream from HBM and the
    tiled kernel keeps two slices in flight, waiting on a count of its own outstanding copies.  Other slice sizes than
    the widest workload's (two resp. three copies per wave and input at least), both schemes, every row against the oracle."""
    w = random_layer(810 + L, 1024, 1024, 10, L, scheme, CLOSED, ZERO_SPLINE, B, oob_frac=0.1)
    art, _ = _compile_both(w.layers[0])
    assert art.info.table_bytes > 128 << 20
    _check_layer(w.layers[0], w.x, lk.ALGO_TILED, what=w.name)
    layer = _device_layer(art, w.layers[0], lk.ALGO_TILED)
    lk.lutkan_forward(layer, torch.from_numpy(w.x).to(DEV))
    assert " pipe=4; " in lk.lutkan_last_plan(), lk.lutkan_last_plan()


def test_cfg4_wide_layer_largest_batch_sampled_rows():
    """The configuration the benchmark times (1024 -> 1024 at 32768 rows): 4096 random rows against the oracle, the
    OOB counters exact over all rows."""
    _sampled_rows_check(cfg4(B=32768), 4096, "cfg4 B=32768")


@pytest.mark.parametrize("B", [1, 5, 16, 17])
def test_bspline_wide_layer_small_batches(B):
    """The B-spline layer at a few rows: up to 16 rows AUTO takes the gather kernel with the inputs split into chunks."""
    w = cfg4(B=B)
    s = w.layers[0]
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob)
    y = lk.bspline_kan_forward(art.bspline_to_device(DEV), torch.from_numpy(w.x).to(DEV))
    ref = oracle.bspline_forward(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.boundary, s.oob, w.x)
    _assert_close(y.cpu().numpy(), ref, f"bspline cfg4 B={B}")


def test_two_million_rows_sampled():
    """A batch far beyond the workloads (2^21 rows, 2048 row tiles, 1 GiB of lookup records): 64-bit row indexing in
    every kernel, checked on sampled rows and through the exact OOB counters."""
    w = random_layer(351, 64, 48, 6, 32, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 1 << 21)
    _sampled_rows_check(w, 4096, "2^21 rows, 64 -> 48")


# ---------------------------------------------------------------- B-spline baseline
def _check_bspline(s, x, algo, what):
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob,
                            edge_scales=s.edge_scales)
    layer = art.bspline_to_device(DEV, algo)
    _say(f"case bspline {what} d={s.d} m={s.m} G={s.G} boundary={s.boundary} oob={s.oob} B={x.shape[0]} algo={algo}")
    y = lk.bspline_kan_forward(layer, torch.from_numpy(x).to(DEV))
    torch.cuda.synchronize()
    ref = oracle.bspline_forward(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.boundary, s.oob, x, edge_scalars=s.edge_scales)
    _assert_close(y.cpu().numpy(), ref, "bspline " + what)


@pytest.mark.parametrize("case", PROPERTY_CASES[1:] + [(c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[7], c[8], c[0] % 2 == 0) for c in TILED_CASES[:5]],
                         ids=lambda c: f"seed{c[0]}")
def test_bspline_layers(case):
    seed, d, m, G, L, scheme, boundary, oob, B, uniform = case
    w = random_layer(seed, d, m, G, L, scheme, boundary, oob, B, uniform=uniform)
    _check_bspline(w.layers[0], w.x, lk.ALGO_GATHER, w.name)
    _check_bspline(w.layers[0], w.x, lk.ALGO_TILED, w.name)


def test_bspline_special_inputs():
    w = random_layer(302, 6, 140, 5, 32, ASYM_UINT8, CLOSED, ZERO_SPLINE, 40)
    x = w.x.copy()
    x[3, 2] = np.nan
    x[5, :] = np.inf
    x[6, :] = -np.inf
    s = w.layers[0]
    for boundary in (HALF_OPEN, CLOSED):
        for oob in (CLIP_X, ZERO_SPLINE):
            s.boundary, s.oob = boundary, oob
            _check_bspline(s, x, lk.ALGO_TILED, "special")
            _check_bspline(s, x, lk.ALGO_GATHER, "special")


def test_bspline_cfg4_every_row():
    w = cfg4(B=4096)
    s = w.layers[0]
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob)
    layer = art.bspline_to_device(DEV)
    y = lk.bspline_kan_forward(layer, torch.from_numpy(w.x).to(DEV))
    ref = oracle.bspline_forward(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.boundary, s.oob, w.x)
    _assert_close(y.cpu().numpy(), ref, "bspline cfg4, all 4096 rows")


# ---------------------------------------------------------------- value_repr = spline_component (Eq. 2, Sec. 4.3 B)
SC_CASES = [
    # seed, d, m, G, L, scheme, boundary, oob, B
    (501, 1, 1, 4, 16, SYM_INT8, CLOSED, CLIP_X, 50),
    (502, 10, 8, 8, 64, SYM_INT8, HALF_OPEN, ZERO_SPLINE, 1024),
    (503, 7, 3, 5, 32, ASYM_UINT8, CLOSED, ZERO_SPLINE, 333),
    (504, 40, 70, 6, 16, ASYM_UINT8, HALF_OPEN, CLIP_X, 2100),
    (505, 64, 256, 8, 64, SYM_INT8, CLOSED, ZERO_SPLINE, 5000),
    (506, 33, 130, 10, 64, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 1025),
]


@pytest.mark.parametrize("case", SC_CASES, ids=lambda c: f"seed{c[0]}")
def test_spline_component_layers(case):
    seed, d, m, G, L, scheme, boundary, oob, B = case
    w = random_layer(seed, d, m, G, L, scheme, boundary, oob, B, uniform=(seed % 2 == 0), oob_frac=0.5, with_base=True)
    s = w.layers[0]
    _check_layer(s, w.x, lk.ALGO_GATHER, codes=(B * d * m <= 2_000_000), what=w.name)
    _check_layer(s, w.x, lk.ALGO_TILED, what=w.name)
    _check_bspline(s, w.x, lk.ALGO_GATHER, w.name)
    _check_bspline(s, w.x, lk.ALGO_TILED, w.name)


BASE_PRODUCT_CASES = [
    # seed, d, m, G, L, scheme, boundary, oob, B, per_input, param_fp16      batch * d * m >= 5e8, d a multiple of 32, m >= 64
    (551, 64, 256, 8, 64, SYM_INT8, CLOSED, ZERO_SPLINE, 32768 + 5, False, False),      # ragged last row tile of the product
    (552, 96, 130, 6, 16, ASYM_UINT8, HALF_OPEN, CLIP_X, 41000, False, False),          # ragged column tile (130 of 256 columns)
    (553, 32, 64, 5, 32, SYM_INT8, HALF_OPEN, ZERO_SPLINE, 250001, False, True),        # the narrowest product; float16 parameters
    (554, 128, 128, 5, 32, ASYM_UINT8, CLOSED, CLIP_X, 33000, True, False),             # one knot vector per input
    (555, 1024, 1024, 10, 64, SYM_INT8, CLOSED, CLIP_X, 2048, False, False),            # the widest layer: inputs split, summing pass adds to y
]


@pytest.mark.parametrize("case", BASE_PRODUCT_CASES, ids=lambda c: f"seed{c[0]}")
def test_spline_component_with_the_base_branch_as_a_matrix_product(case):
    """From about 5e8 edge evaluations per call a spline_component layer evaluates its base branch (Eq. 2: s_out * s_base *
    SiLU(x), summed over the inputs) as one [B, d] x [d, m] product on the matrix cores, fp32 operands as three bf16
    pieces, and the LUT edge kernel adds the spline branch on top.  Same bar as every other path: k, l0, In, w bit-exact,
    outputs within the tolerance, on all rows; a NaN input poisons its own row only."""
    seed, d, m, G, L, scheme, boundary, oob, B, per_input, half = case
    if per_input:
        w = per_input_layer(seed, d, m, G, L, scheme, boundary, oob, B, with_base=True)
    else:
        w = random_layer(seed, d, m, G, L, scheme, boundary, oob, B, uniform=(seed % 2 == 0), oob_frac=0.3, with_base=True)
    s = w.layers[0]
    x = w.x.copy()
    x[B // 2, d // 3] = np.nan
    x[B // 3, :] = 30.0                                 # SiLU(x) ~ x
    x[B // 5, :] = -90.0                                # SiLU(x) underflows to -0
    _check_layer(s, x, lk.ALGO_AUTO, what=w.name, param_fp16=half)
    assert "base_product; tiled" in lk.lutkan_last_plan(), lk.lutkan_last_plan()
    # the same layer through the entry points that take the two phases apart, and through the built-in scratch
    art, ora = _compile_both(s, half)
    layer = _device_layer(art, s)
    xg = torch.from_numpy(x).to(DEV)
    y_ref = lk.lutkan_forward(layer, xg)
    ws = torch.empty(lk.lutkan_forward_workspace_bytes(layer, B), dtype=torch.uint8, device=DEV)
    lk.lutkan_forward_locate(layer, xg, ws)
    y_two = lk.lutkan_forward_edges(layer, B, torch.full((B, m), 3.0, dtype=torch.float32, device=DEV), ws)
    same = lambda p, q: bool(((p == q) | (torch.isnan(p) & torch.isnan(q))).all())
    assert same(y_two, y_ref)
    if lk.lutkan_forward_workspace_bytes(layer, B) <= lk.STATIC_SCRATCH_BYTES:
        y_static = lk.lutkan_forward_static_scratch(layer, xg, torch.full((B, m), -3.0, dtype=torch.float32, device=DEV))
        assert same(y_static, y_ref)


@pytest.mark.parametrize("boundary,oob", [(HALF_OPEN, CLIP_X), (HALF_OPEN, ZERO_SPLINE), (CLOSED, CLIP_X), (CLOSED, ZERO_SPLINE)])
def test_case_a_sweep_shape_spline_component(boundary, oob):
    """The paper's controlled-sweep layer (10->8, grid 8, spline_component) with inputs clipped onto the domain."""
    for L, scheme in ((16, ASYM_UINT8), (64, SYM_INT8), (128, ASYM_UINT8)):
        w = case_a(seed=1, L=L, scheme=scheme, boundary=boundary, oob=oob)
        _check_layer(w.layers[0], w.x, lk.ALGO_AUTO, codes=True, what=w.name)


def test_spline_component_special_inputs():
    w = random_layer(507, 6, 140, 5, 32, SYM_INT8, HALF_OPEN, ZERO_SPLINE, 40, with_base=True)
    x = w.x.copy()
    x[3, 2] = np.nan
    x[5, :] = 80.0          # SiLU(x) ~ x, exp(-x) underflows
    x[6, :] = -120.0        # exp(-x) overflows to inf: SiLU -> -0
    x[7, :] = np.inf
    s = w.layers[0]
    for algo in (lk.ALGO_GATHER, lk.ALGO_TILED):
        _check_layer(s, x[:7], algo, what="sc special")


STATS_CASES = [
    # seed, B, d, m, boundary, spread of x around the domain [-1, 1]
    (701, 1, 1, 1, CLOSED, 1.5),
    (702, 63, 7, 5, HALF_OPEN, 1.2),
    (703, 1000, 70, 130, CLOSED, 1.05),
    (704, 4099, 64, 8, HALF_OPEN, 1.0),          # U(-1, 1): every row in-range
    (705, 300, 300, 3, CLOSED, 3.0),             # every row has an input outside
    (706, 20000, 16, 64, HALF_OPEN, 1.01),
]


@pytest.mark.parametrize("case", STATS_CASES, ids=lambda c: f"seed{c[0]}")
def test_error_stats_kernel(case):
    """Sec. 5.6 statistics reduced on the device against their plain definition: counts and maxima exact, fp64 sums
    up to the order of summation."""
    seed, B, d, m, boundary, spread = case
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.uniform(-spread, spread, size=(B, d)).astype(np.float32)
    x.reshape(-1)[rng.integers(0, B * d, size=max(1, B * d // 50))] = np.float32(1.0)      # inputs exactly on t_K
    y = rng.normal(size=(B, m)).astype(np.float32)
    r = (y + rng.normal(scale=1e-3, size=(B, m))).astype(np.float32)
    if B > 10:
        x[B // 2, 0] = np.nan
        y[B // 3, m // 2] = np.nan
    _say(f"case stats seed={seed} B={B} d={d} m={m} boundary={boundary}")
    got = lk.lutkan_error_stats(torch.from_numpy(y).to(DEV), torch.from_numpy(r).to(DEV), torch.from_numpy(x).to(DEV),
                                -1.0, 1.0, boundary)
    want = oracle.error_stats(y, r, x, -1.0, 1.0, boundary)
    _same_error_summary(got, want)


def _same_error_summary(got, want):
    """Every field of lutkan_error_summary against the oracle's: counts, maxima and the OOB fraction exact, the fp64
    sums and means up to the order of summation."""
    assert set(got) == set(want)
    for key in ("rows_in", "rows_oob", "nan_in", "nan_oob", "max_abs_in", "max_abs_oob", "oob_any_frac"):
        assert got[key] == want[key], key
    for key in ("sum_abs_in", "sum_abs_oob", "mae_in", "mae_oob"):
        if np.isnan(want[key]):
            assert np.isnan(got[key]), key
        else:
            assert abs(got[key] - want[key]) <= 1e-12 * abs(want[key]) + 1e-300, key


def test_error_stats_mean_leaves_nan_outputs_out_of_the_count():
    """NaN outputs inside both subsets (several per subset, so that rows * m and the number of differences that exist
    differ visibly): the device divides each sum by the latter, as the oracle does; a subset of NaN outputs only has
    no mean."""
    rng = np.random.Generator(np.random.PCG64(720))
    B, d, m = 500, 6, 10
    x = rng.uniform(-1.1, 1.1, size=(B, d)).astype(np.float32)
    y = rng.normal(size=(B, m)).astype(np.float32)
    r = (y + rng.normal(scale=1e-2, size=(B, m))).astype(np.float32)
    y.reshape(-1)[rng.choice(B * m, size=B * m // 5, replace=False)] = np.nan
    _say(f"case stats with NaN outputs in both subsets B={B} d={d} m={m}")
    got = lk.lutkan_error_stats(torch.from_numpy(y).to(DEV), torch.from_numpy(r).to(DEV), torch.from_numpy(x).to(DEV),
                                -1.0, 1.0, CLOSED)
    want = oracle.error_stats(y, r, x, -1.0, 1.0, CLOSED)
    assert want["nan_in"] > 50 and want["nan_oob"] > 50 and want["rows_in"] > 50 and want["rows_oob"] > 50
    _same_error_summary(got, want)
    assert abs(got["mae_in"] - got["sum_abs_in"] / (got["rows_in"] * m - got["nan_in"])) <= 1e-15
    assert got["mae_in"] > 1.1 * got["sum_abs_in"] / (got["rows_in"] * m)          # the other denominator is 20 % larger
    y[:] = np.nan
    got = lk.lutkan_error_stats(torch.from_numpy(y).to(DEV), torch.from_numpy(r).to(DEV), torch.from_numpy(x).to(DEV),
                                -1.0, 1.0, CLOSED)
    _same_error_summary(got, oracle.error_stats(y, r, x, -1.0, 1.0, CLOSED))
    assert np.isnan(got["mae_in"]) and np.isnan(got["mae_oob"]) and got["nan_in"] == got["rows_in"] * m


def test_error_stats_of_a_lut_layer_against_its_spline_layer():
    """The protocol end to end on one layer: LUT output vs B-spline output, subsets by In(x)."""
    w = random_layer(711, 8, 128, 5, 32, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 8192)
    s = w.layers[0]
    art, _ = _compile_both(s)
    xg = torch.from_numpy(w.x).to(DEV)
    y_lut = lk.lutkan_forward(_device_layer(art, s), xg)
    y_ref = lk.bspline_kan_forward(art.bspline_to_device(DEV).with_contract(CLOSED, CLIP_X), xg)
    got = lk.lutkan_error_stats(y_lut, y_ref, xg, float(art.knots[0]), float(art.knots[-1]), s.boundary)
    torch.cuda.synchronize()
    want = oracle.error_stats(y_lut.cpu().numpy(), y_ref.cpu().numpy(), w.x, art.knots[0], art.knots[-1], s.boundary)
    assert (got["rows_in"], got["rows_oob"]) == (want["rows_in"], want["rows_oob"]) and min(got["rows_in"], got["rows_oob"]) > 100
    assert got["max_abs_in"] == want["max_abs_in"] and got["max_abs_oob"] == want["max_abs_oob"]
    assert abs(got["mae_in"] - want["mae_in"]) <= 1e-12 * want["mae_in"]
    assert got["mae_oob"] > 2 * got["mae_in"]                     # zero_spline drops the OOB inputs' contributions


def test_model_forward_replays_correctly_from_a_hip_graph():
    """The chain launches only kernels (no allocation, no memset, no synchronisation), so it can be captured;
    every replay, with eager work in between, reproduces the eager result bit for bit."""
    w = cfg2(B=5000)
    arts = [lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob) for s in w.layers]
    layers = [a.to_device(DEV) for a in arts]
    x = torch.from_numpy(w.x).to(DEV)
    B = x.shape[0]
    ws = torch.empty(lk.lutkan_model_workspace_bytes(layers, B), dtype=torch.uint8, device=DEV)
    y = torch.empty((B, layers[-1].m), dtype=torch.float32, device=DEV)
    stats = torch.zeros((len(layers), 2), dtype=torch.int64, device=DEV)
    _say(f"case graph capture {w.name} B={B}")
    lk.lutkan_model_forward(layers, x, y, stats=stats, workspace=ws)           # warm-up: one-time kernel attributes
    torch.cuda.synchronize()
    y_eager, stats_eager = y.clone(), stats.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        lk.lutkan_model_forward(layers, x, y, stats=stats, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lk.lutkan_model_forward(layers, x, y, stats=stats, workspace=ws)
    for _ in range(3):
        y.fill_(7.0)
        stats.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager) and torch.equal(stats, stats_eager)
        lk.lutkan_model_forward(layers, x, y, workspace=ws)                    # eager work between replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("B", [256, 5000])
def test_fused_chain_replays_correctly_from_a_hip_graph(B):
    """One kernel launch and nothing else: captured after one eager call (which sets the kernel's one-time
    attribute), every replay with eager work in between reproduces the eager result bit for bit."""
    w = cfg2(B=B)
    arts = [lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob) for s in w.layers]
    layers = [a.to_device(DEV) for a in arts]
    x = torch.from_numpy(w.x).to(DEV)
    y = torch.empty((B, layers[-1].m), dtype=torch.float32, device=DEV)
    stats = torch.zeros((len(layers), 2), dtype=torch.int64, device=DEV)
    _say(f"case graph capture of the fused chain {w.name} B={B}")
    lk.lutkan_chain_forward(layers, x, y, stats=stats)
    torch.cuda.synchronize()
    y_eager, stats_eager = y.clone(), stats.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        lk.lutkan_chain_forward(layers, x, y, stats=stats)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lk.lutkan_chain_forward(layers, x, y, stats=stats)
    for _ in range(3):
        y.fill_(7.0)
        stats.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager) and torch.equal(stats, stats_eager)
        lk.lutkan_chain_forward(layers, x, y)                                  # eager work between replays
        torch.cuda.synchronize()


def test_random_shapes_and_contracts():
    """Sixty layers with shapes, grids, table sizes and contracts drawn at random (seeded), covering every tile width,
    ragged tiles and batches, both value representations, both parameter dtypes and both kernel families; the LUT
    layer (trace and plain launch, counters) and the B-spline layer against the oracle."""
    rng = np.random.Generator(np.random.PCG64(2024))
    worst = 0.0
    for it in range(60):
        G = int(rng.choice([1, 2, 3, 5, 8, 10, 17, 33, 64]))
        L = int(rng.choice([2, 3, 5, 16, 31, 64, 128, 512]))
        L = min(L, 65535 // G)
        d = int(rng.integers(1, 41))
        m = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 16, 17, 31, 32, 33, 64, 65, 100, 128, 129, 200, 300]))
        B = int(rng.choice([1, 2, 15, 16, 17, 63, 64, 65, 255, 256, 257, 1000, 1024, 1025, 2500]))
        scheme, boundary, oob = (int(rng.integers(0, 2)) for _ in range(3))
        base = bool(rng.integers(0, 2))
        half = bool(rng.integers(0, 2))
        algo = int(rng.choice([lk.ALGO_AUTO, lk.ALGO_GATHER]))
        w = random_layer(2000 + it, d, m, G, L, scheme, boundary, oob, B, uniform=bool(rng.integers(0, 2)), with_base=base)
        s = w.layers[0]
        _say(f"case random {it}: d={d} m={m} G={G} L={L} B={B} scheme={scheme} boundary={boundary} oob={oob} base={base} "
             f"fp16={half} algo={algo}")
        worst = max(worst, _check_layer(s, w.x, algo, what=w.name, param_fp16=half))
        yb = lk.bspline_kan_forward(_compile_both(s, half)[0].bspline_to_device(DEV), torch.from_numpy(w.x).to(DEV))
        torch.cuda.synchronize()
        refb = oracle.bspline_forward(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.boundary, s.oob, w.x, edge_scalars=s.edge_scales)
        worst = max(worst, _assert_close(yb.cpu().numpy(), refb, w.name + " bspline"))
    _say(f"random layers: worst error / tolerance = {worst:.3f}")


# ---- fused chain: the whole narrow network in one launch ----

def _narrow_chain(seed, widths, G, L, scheme, boundary, oob, B, with_base=False, lo=-2.0, hi=2.0):
    """Layers of a narrow network on [lo, hi] with coefficients ~ N(0, 1/sqrt(d)); x ~ N(0,1) with heavy tails."""
    from lutkan_inputs import LayerSpec, draw_edge_scales, uniform_ext_knots
    rng = np.random.Generator(np.random.PCG64(seed))
    layers = []
    for d, m in zip(widths[:-1], widths[1:]):
        coef = rng.normal(0.0, 1.0 / np.sqrt(d), size=(d, m, G + 3)).astype(np.float32)
        s = LayerSpec(d, m, G, 3, uniform_ext_knots(lo, hi, G, 3), coef, L, scheme, boundary, oob)
        if with_base:
            s.edge_scales = draw_edge_scales(rng, d, m)
        layers.append(s)
    x = np.where(rng.random((B, widths[0])) < 0.1, rng.standard_t(3.0, size=(B, widths[0])), rng.normal(size=(B, widths[0]))).astype(np.float32)
    return layers, x


def _fused_chain_check(specs, x, what, param_fp16=False):
    """Every layer of the fused launch against the oracle on the SAME input (the launch's own hidden activation of
    the previous layer), its counters against the oracle's, and the result against the layer-by-layer chain."""
    compiled = [_compile_both_uncached(s, param_fp16) for s in specs]
    layers = [_device_layer(art, s) for s, (art, _) in zip(specs, compiled)]
    B = x.shape[0]
    xg = torch.from_numpy(x).to(DEV)
    hidden = torch.full((B * sum(s.m for s in specs[:-1]) + 1,), float("nan"), dtype=torch.float32, device=DEV)
    stats = torch.zeros((len(specs), 2), dtype=torch.int64, device=DEV)
    _say(f"case {what}: fused chain {[s.d for s in specs] + [specs[-1].m]} B={B} fp16={param_fp16}")
    y = lk.lutkan_chain_forward(layers, xg, stats=stats, hidden=hidden)
    y_plain = lk.lutkan_chain_forward(layers, xg)
    torch.cuda.synchronize()
    assert torch.equal(y, y_plain) or np.array_equal(np.isnan(y.cpu().numpy()), np.isnan(y_plain.cpu().numpy()))
    h = hidden.cpu().numpy()
    assert np.isnan(h[-1])                                # nothing written past the trace
    cur, off, worst = x, 0, 0.0
    for li, (s, (art, ora)) in enumerate(zip(specs, compiled)):
        ref = oracle.lut_forward(ora, s.boundary, s.oob, cur, edge_scalars=s.edge_scales)
        if li + 1 < len(specs):
            nxt = h[off:off + B * s.m].reshape(B, s.m)
            off += B * s.m
        else:
            nxt = y.cpu().numpy()
        worst = max(worst, _assert_close(nxt, ref, f"{what} layer {li}"))
        st = stats[li].cpu().numpy()
        assert (int(st[0]), int(st[1])) == (ref.oob_count, ref.oob_any_rows), f"{what} layer {li} counters"
        cur = nxt
    y_model = lk.lutkan_model_forward(layers, xg).cpu().numpy()
    scale = np.abs(y_model[np.isfinite(y_model)]).max() if np.isfinite(y_model).any() else 1.0
    ok = np.isfinite(y_model)
    assert np.abs(y.cpu().numpy()[ok] - y_model[ok]).max() <= 1e-3 * max(scale, 1.0)
    return worst


def _compile_both_uncached(s, param_fp16):
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob,
                            edge_scales=s.edge_scales, param_dtype=lk.PARAM_FP16 if param_fp16 else lk.PARAM_FP32)
    ora = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, param_fp16=param_fp16)
    assert np.array_equal(art.q, ora.q) and np.array_equal(art.scale, ora.scale) and np.array_equal(art.y_min, ora.y_min)
    return art, ora


FUSED_CHAIN_CASES = [
    # seed, widths, G, L, scheme, boundary, oob, B, with_base, param_fp16
    (901, (78, 16, 2), 5, 64, ASYM_UINT8, CLOSED, CLIP_X, 256, False, False),          # the tabular shape at the latency batch
    (902, (78, 32, 16, 1), 5, 64, SYM_INT8, CLOSED, CLIP_X, 256, True, False),         # the case study's network (Sec. 8)
    (903, (78, 32, 16, 1), 5, 64, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 1027, True, True),
    (904, (10, 8), 8, 16, SYM_INT8, HALF_OPEN, ZERO_SPLINE, 1, False, False),           # one layer, one row
    (905, (5, 64, 3, 64, 4), 3, 8, ASYM_UINT8, CLOSED, ZERO_SPLINE, 3, False, True),    # 64-column layers, one group per wave
    (906, (1024, 4, 1), 4, 32, SYM_INT8, CLOSED, CLIP_X, 70, False, False),             # the widest input, 16 groups of inputs
    (907, (3, 5, 7, 9, 11, 13, 15, 17, 2), 6, 16, ASYM_UINT8, HALF_OPEN, CLIP_X, 4099, True, False),   # eight layers
]


@pytest.mark.parametrize("case", FUSED_CHAIN_CASES, ids=lambda c: f"seed{c[0]}")
def test_fused_chain(case):
    seed, widths, G, L, scheme, boundary, oob, B, with_base, half = case
    specs, x = _narrow_chain(seed, widths, G, L, scheme, boundary, oob, B, with_base)
    if B > 10:
        x[B // 2, 0] = np.nan                       # poisons its own row only
        x[B // 3, :] = 50.0                         # every input out of domain
    _fused_chain_check(specs, x, f"fused seed{seed}", half)


@pytest.mark.parametrize("B", [3, 300, 3000])
def test_fused_chain_with_one_knot_vector_per_input(B):
    """A network whose layers each have per-input knot vectors (the grids of a model after per-feature grid updates):
    the fused launch locates every input on its own vector, read from global memory."""
    rng = np.random.Generator(np.random.PCG64(930))
    widths, G, L = (20, 9, 5, 2), 6, 32
    specs = []
    for li, (d, m) in enumerate(zip(widths[:-1], widths[1:])):
        s = per_input_layer(931 + li, d, m, G, L, ASYM_UINT8 if li % 2 else SYM_INT8, HALF_OPEN, ZERO_SPLINE, 4, with_base=(li == 1)).layers[0]
        s.coef = (s.coef / np.sqrt(d)).astype(np.float32)
        specs.append(s)
    x = per_input_layer(931, widths[0], widths[1], G, L, SYM_INT8, HALF_OPEN, ZERO_SPLINE, B).x     # covers layer 0's own domains
    compiled = [_compile_both(s) for s in specs]
    layers = [_device_layer(art, s) for s, (art, _) in zip(specs, compiled)]
    xg = torch.from_numpy(x).to(DEV)
    hidden = torch.zeros(B * sum(widths[1:-1]), dtype=torch.float32, device=DEV)
    stats = torch.zeros((len(specs), 2), dtype=torch.int64, device=DEV)
    _say(f"case fused chain with per-input knots {widths} B={B}")
    y = lk.lutkan_chain_forward(layers, xg, stats=stats, hidden=hidden)
    y_model = lk.lutkan_model_forward(layers, xg)
    torch.cuda.synchronize()
    assert torch.equal(y, y_model)                          # every layer is a small one: the same single launch
    h, cur, off = hidden.cpu().numpy(), x, 0
    for li, (s, (art, ora)) in enumerate(zip(specs, compiled)):
        ref = oracle.lut_forward(ora, s.boundary, s.oob, cur, edge_scalars=s.edge_scales)
        nxt = h[off:off + B * s.m].reshape(B, s.m) if li + 1 < len(specs) else y.cpu().numpy()
        off += B * s.m
        _assert_close(nxt, ref, f"per-input chain layer {li}")
        st = stats[li].cpu().numpy()
        assert (int(st[0]), int(st[1])) == (ref.oob_count, ref.oob_any_rows)
        cur = nxt


@pytest.mark.parametrize("boundary", [HALF_OPEN, CLOSED])
def test_every_kernel_locates_bit_exactly_through_a_revealing_table(boundary):
    """A one-edge layer whose table makes the output spell out the lookup: codes q[k][l] = l, alpha_k = 2^k, y_min = 0,
    so y = 2^k * (l0 + w) = 2^k * z exactly (z - l0 = w and l0 + w = z are exact in fp32).  The oracle's (k, l0, w)
    therefore fix the output of every edge kernel bit for bit -- also of the kernels that have no trace outputs
    (the tiled kernel and the fused chain)."""
    G, L, B = 7, 64, 4000
    rng = np.random.Generator(np.random.PCG64(77 + boundary))
    knots = np.unique(np.sort(rng.uniform(-2.0, 3.0, size=G + 1)).astype(np.float32))   # no knot at 0: a subnormal x
    # next to it gives a subnormal z, which the tiled kernel's 2^-24-scaled sums flush (far below the tolerance)
    K = knots.size - 1
    q = np.tile(np.arange(L, dtype=np.uint8), (1, K, 1))
    scale = (2.0 ** np.arange(K)).astype(np.float32).reshape(1, K)
    art = lk.lutkan_artifact_from_arrays(1, 1, knots, q, scale, np.zeros((1, K), np.float32), boundary, CLIP_X)
    x = rng.uniform(knots[0] - 0.5, knots[-1] + 0.5, size=(B, 1)).astype(np.float32)
    special = np.concatenate([knots, np.nextafter(knots, np.float32(-np.inf)), np.nextafter(knots, np.float32(np.inf))])
    x[:special.size, 0] = special
    ora = SimpleNamespace(d=1, m=1, K=K, L=L, scheme=ASYM_UINT8, knots=knots, q=q, scale=scale, y_min=np.zeros((1, K), np.float32))
    ref = oracle.lut_forward(ora, boundary, CLIP_X, x, trace=True)
    z = ref.l0[:, 0].astype(np.float32) + ref.w[:, 0]
    want = np.ldexp(z, ref.k[:, 0]).astype(np.float32)
    xg = torch.from_numpy(x).to(DEV)
    outs = {"tiled": lk.lutkan_forward(art.to_device(DEV, lk.ALGO_TILED), xg),
            "gather": lk.lutkan_forward(art.to_device(DEV, lk.ALGO_GATHER), xg),
            "chain, a work-group per row": lk.lutkan_chain_forward([art.to_device(DEV)], xg[:900].contiguous()),
            "chain, a wave per row": lk.lutkan_chain_forward([art.to_device(DEV)], xg),
            "auto": lk.lutkan_forward(art.to_device(DEV), xg)}
    torch.cuda.synchronize()
    for name, y in outs.items():
        got = y.cpu().numpy()[:, 0]
        np.testing.assert_array_equal(got.view(np.uint32), want[:got.size].view(np.uint32), err_msg=name)


def test_fused_chain_refuses_what_it_cannot_hold():
    specs, x = _narrow_chain(920, (8, 128, 4), 4, 8, SYM_INT8, CLOSED, CLIP_X, 8)
    layers = [_device_layer(_compile_both_uncached(s, False)[0], s) for s in specs]
    xg = torch.from_numpy(x).to(DEV)
    with pytest.raises(lk.LutKanError) as e:        # a 128-column layer
        lk.lutkan_chain_forward(layers, xg)
    assert str(e.value).startswith("[-5]")
    with pytest.raises(lk.LutKanError) as e:        # widths that do not chain
        lk.lutkan_chain_forward([layers[0], layers[0]], xg)
    assert str(e.value).startswith("[-2]")


def test_last_plan_reports_what_auto_dispatch_launched():
    """lutkan_last_plan names the kernels of the last forward call: the dispatch rules of algo = AUTO, observed."""
    w = cfg4(B=4096)
    s = w.layers[0]
    art, _ = _compile_both(s)
    layer = _device_layer(art, s)
    xg = torch.from_numpy(w.x).to(DEV)
    _say("case last plan: cfg4 at 1, 64 and 4096 rows")
    import re

    def tiled_groups(plan, B, jt, n_tiles):
        """Work-groups of the tiled launch named in `plan`, and its chunk count: the launch shape comes out of a
        fitted cost model, so only its invariants are asserted -- a legal row-step count, whole rounds' worth of
        work-groups, and a summing pass exactly when the inputs were split."""
        mt = re.search(r"tiled np=(\d+) split=(\d+) pipe=(\d); ", plan)
        assert mt, plan
        np_, split, pipe = int(mt.group(1)), int(mt.group(2)), int(mt.group(3))
        rows_per_wave = (64 // (jt // 4)) * np_
        assert np_ in (1, 2, 4, 8, 16) and rows_per_wave <= 64 and 1 <= split <= 128 and pipe in (2, 3, 4)
        assert plan.endswith("sum; ") == (split > 1), plan
        return -(-B // (16 * rows_per_wave)) * n_tiles * split, split

    lk.lutkan_forward(layer, xg[:1])
    plan = lk.lutkan_last_plan()                                                # a few rows: only the touched table rows,
    assert re.fullmatch(r"locate; gather split=(\d+); sum; ", plan), plan      # the inputs split over the GPU
    lk.lutkan_forward(layer, xg[:64])
    assert lk.lutkan_last_plan().startswith("locate; gather split=")
    lk.lutkan_forward(layer, xg)
    plan = lk.lutkan_last_plan()
    assert plan.startswith("locate; tiled np="), plan
    groups, _ = tiled_groups(plan, 4096, art.info.jt, art.info.n_tiles)
    assert groups >= 256, plan                                                  # at least one work-group per compute unit
    assert " pipe=3; " in plan, plan                                            # three slice buffers fit: reads carried across inputs
    lk.lutkan_forward(layer, xg[:256])                                          # the 686 MiB table streaming from HBM is the launch's time:
    assert re.search(r"tiled np=\d+ split=\d+ pipe=4; ", lk.lutkan_last_plan()), lk.lutkan_last_plan()      # two slices in flight
    lk.lutkan_forward(layer, xg)
    stats = torch.zeros(2, dtype=torch.int64, device=DEV)
    lk.lutkan_forward(layer, xg, stats=stats)
    assert lk.lutkan_last_plan() == plan.replace("locate; ", "locate; oob; ")   # the counters add one launch, nothing else
    lk.bspline_kan_forward(art.bspline_to_device(DEV), xg)
    assert lk.lutkan_last_plan().startswith("bspline_locate; bspline_tiled np=")
    _say("case last plan: cfg2 at 300, 5000, 20000 and 40000 rows")
    w2 = cfg2(B=40000)
    layers = []
    keep = []
    for s2 in w2.layers:
        a2, _ = _compile_both(s2)
        keep.append(a2)
        layers.append(_device_layer(a2, s2))
    x2 = torch.from_numpy(w2.x).to(DEV)
    lk.lutkan_model_forward(layers, x2[:300])
    assert lk.lutkan_last_plan() == "chain layers=2 wpr=4; "                   # every layer small: one launch, a work-group per row
    lk.lutkan_model_forward(layers, x2[:5000])
    assert lk.lutkan_last_plan() == "chain layers=2 wpr=1; "                   # beyond 1024 rows: a wave per row
    lk.lutkan_forward(layers[0], x2[:300])
    assert lk.lutkan_last_plan() == "chain layers=1 wpr=4; "                   # a single small layer runs as a one-layer chain
    lk.lutkan_model_forward(layers, x2[:20000])
    plan = lk.lutkan_last_plan()                                               # 78x16 has outgrown the chain kernel, 16x2 has not yet
    assert plan.count("locate; tiled np=") == 1 and plan.endswith("chain layers=1 wpr=1; "), plan
    lk.lutkan_model_forward(layers, x2)
    plan = lk.lutkan_last_plan()
    assert plan.count("locate; tiled np=") == 2 and "chain" not in plan, plan  # large batches: locate + tiled kernel per layer
    torch.cuda.synchronize()


def test_measurement_probes_report_their_work():
    """The peak-rate probes behind the roofline terms: each kind launches and reports the work of one launch (the
    count the rate is computed from), which follows from the launch shape and the iteration count; the rate itself is
    only required to be a finite positive number here -- its value belongs to the benchmark's record, not to a test."""
    buf = torch.zeros((1 << 30) // 4 + 4, dtype=torch.float32, device=DEV)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    kinds = {lk.PROBE_VALU_FMA: 2048, lk.PROBE_VALU_FMAC: 2048, lk.PROBE_VALU_MIX: 2048, lk.PROBE_LDS_READ: 512, lk.PROBE_L2_READ: 4,
             lk.PROBE_HBM_READ: 2}
    for kind, iters in kinds.items():
        lk.lutkan_probe_launch(kind, buf, iters)             # warm-up
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        work = lk.lutkan_probe_launch(kind, buf, iters)
        e1.record()
        torch.cuda.synchronize()
        half = lk.lutkan_probe_launch(kind, buf, iters // 2)
        torch.cuda.synchronize()
        rate = work / (e0.elapsed_time(e1) * 1e-3)
        _say(f"probe kind {kind}: work {work:.4g}, {rate:.3g} per second on {cus} compute units")
        assert work > 0 and work == 2 * half                 # proportional to the iterations inside the kernel
        assert np.isfinite(rate) and rate > 0
    assert lk.lutkan_probe_launch(lk.PROBE_HBM_READ, buf, 2) == 2.0 * (buf.numel() * 4 - 16)      # the buffer, once per pass
    with pytest.raises(lk.LutKanError):
        lk.lutkan_probe_launch(99, buf, 1)
    with pytest.raises(lk.LutKanError):
        lk.lutkan_probe_launch(lk.PROBE_HBM_READ, buf[:1024], 1)
