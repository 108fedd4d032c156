"""The entry point for callers that cannot allocate (lutkan_forward_static_scratch): its scratch is an array inside
the library, so it must give what lutkan_forward gives with a caller's workspace -- the same kernels run, hence bit
for bit -- also on a second call with a smaller input that finds the first call's records still in the array."""
import numpy as np
import pytest

import oracle
from lutkan_inputs import ASYM_UINT8, CLOSED, CLIP_X, HALF_OPEN, SYM_INT8, ZERO_SPLINE, random_layer

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2601_03332_amd as lk  # noqa: E402

DEV = "cuda:0"


def _both_ways(layer, x):
    """(static-scratch result, workspace result, their counters) for one input."""
    B = x.shape[0]
    y_static = torch.full((B, layer.m), 7.0, dtype=torch.float32, device=DEV)
    y_ws = torch.full((B, layer.m), -7.0, dtype=torch.float32, device=DEV)
    st_static = torch.zeros(2, dtype=torch.int64, device=DEV)
    st_ws = torch.zeros(2, dtype=torch.int64, device=DEV)
    lk.lutkan_forward_static_scratch(layer, x, y_static, stats=st_static)
    plan_static = lk.lutkan_last_plan()
    lk.lutkan_forward(layer, x, y_ws, stats=st_ws)
    assert lk.lutkan_last_plan() == plan_static          # the same kernels in the same launch shapes
    torch.cuda.synchronize()
    return y_static, y_ws, st_static, st_ws


@pytest.mark.parametrize("case", [
    # seed, d, m, G, L, scheme, boundary, oob, first batch, second (smaller) batch, algo
    (1201, 70, 130, 6, 32, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 5000, 1300, lk.ALGO_AUTO),     # tiled, inputs split, partial sums
    (1202, 33, 40, 9, 16, SYM_INT8, CLOSED, CLIP_X, 20000, 777, lk.ALGO_TILED),               # several row tiles, then one
    (1203, 50, 9, 5, 64, SYM_INT8, HALF_OPEN, CLIP_X, 3000, 33, lk.ALGO_GATHER),              # gather kernel with chunks
], ids=lambda c: f"seed{c[0]}")
def test_static_scratch_matches_caller_workspace_on_two_calls_in_a_row(case):
    seed, d, m, G, L, scheme, boundary, oob, B1, B2, algo = case
    w = random_layer(seed, d, m, G, L, scheme, boundary, oob, B1, uniform=(seed % 2 == 0))
    s = w.layers[0]
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob)
    ora = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme)
    layer = art.to_device(DEV, algo)
    assert lk.lutkan_forward_workspace_bytes(layer, B1) <= lk.STATIC_SCRATCH_BYTES
    x1 = torch.from_numpy(w.x).to(DEV)
    x2 = torch.from_numpy(np.ascontiguousarray(w.x[B1 - B2:])).to(DEV)       # other rows than the first call's first B2
    for x in (x1, x2):                                                       # the second call follows the first directly
        print(f"case static scratch seed={seed} d={d} m={m} B={x.shape[0]} algo={algo}", flush=True)
        y_static, y_ws, st_static, st_ws = _both_ways(layer, x)
        assert torch.equal(y_static, y_ws) and torch.equal(st_static, st_ws)
        ref = oracle.lut_forward(ora, s.boundary, s.oob, x.cpu().numpy())
        err = np.abs(y_static.cpu().numpy().astype(np.float64) - ref.y)
        assert np.all(err <= 1e-5 * ref.A + 1e-6)
        assert (int(st_static[0]), int(st_static[1])) == (ref.oob_count, ref.oob_any_rows)


def test_static_scratch_refuses_what_does_not_fit():
    w = random_layer(1210, 64, 64, 5, 16, SYM_INT8, CLOSED, CLIP_X, 8)
    s = w.layers[0]
    layer = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob).to_device(DEV)
    B = lk.STATIC_SCRATCH_BYTES // (8 * s.d) + 1024
    x = torch.zeros((B, s.d), dtype=torch.float32, device=DEV)
    y = torch.zeros((B, s.m), dtype=torch.float32, device=DEV)
    with pytest.raises(lk.LutKanError) as e:
        lk.lutkan_forward_static_scratch(layer, x, y)
    assert str(e.value).startswith("[-2]") and "built-in array" in str(e.value)
    assert lk.lutkan_last_plan() == ""                    # nothing was launched
