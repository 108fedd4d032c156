"""ctypes binding of include/lutkan.h.  Same entry-point names as the C ABI; argument marshalling only."""
from __future__ import annotations

import ctypes as C
import json
import os
from types import SimpleNamespace
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

SYM_INT8, ASYM_UINT8 = 0, 1
HALF_OPEN, CLOSED = 0, 1
CLIP_X, ZERO_SPLINE = 0, 1
ALGO_AUTO, ALGO_GATHER, ALGO_TILED, ALGO_TILED_WIDE = 0, 1, 2, 3
PARAM_FP32, PARAM_FP16 = 0, 1
SPAN_DOMAIN, SPAN_EXTENDED = 0, 1
PROBE_VALU_FMA, PROBE_LDS_READ, PROBE_L2_READ, PROBE_HBM_READ, PROBE_VALU_MIX, PROBE_VALU_FMAC = 0, 1, 2, 3, 4, 5
REPR_PHI, REPR_SPLINE_COMPONENT = 0, 1
MAX_K = 64


class LutKanError(RuntimeError):
    pass


class _LayerDesc(C.Structure):
    _fields_ = [("d", C.c_int32), ("m", C.c_int32), ("G", C.c_int32), ("degree", C.c_int32),
                ("ext_knots", C.c_void_p), ("coef", C.c_void_p),
                ("L", C.c_int32), ("scheme", C.c_int32), ("boundary", C.c_int32), ("oob", C.c_int32),
                ("value_repr", C.c_int32), ("edge_base_scale", C.c_void_p), ("edge_spline_scale", C.c_void_p),
                ("edge_out_scale", C.c_void_p), ("param_dtype", C.c_int32), ("knot_span", C.c_int32),
                ("knots_per_input", C.c_int32)]


class _ArtifactArrays(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d", "m", "K", "L", "scheme", "boundary", "oob", "value_repr", "param_dtype",
                                         "knots_per_input")] + \
               [(n, C.c_void_p) for n in ("knots", "q_table", "scale", "y_min", "edge_base_scale", "edge_spline_scale",
                                          "edge_out_scale")]


class _Info(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d", "m", "K", "L", "G", "degree", "scheme", "boundary", "oob", "value_repr",
                                         "param_dtype", "knot_span", "knots_per_input", "jt", "n_tiles", "blob_bytes",
                                         "coef_jt", "coef_n_tiles", "coef_blob_bytes")] + \
               [("t0", C.c_float), ("tK", C.c_float), ("tK_star", C.c_float)] + \
               [(n, C.c_size_t) for n in ("q_canonical_bytes", "params_canonical_bytes", "table_bytes",
                                          "coef_table_bytes", "artifact_bytes")]


class _DevLayer(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d", "m", "K", "L", "scheme", "boundary", "oob", "value_repr", "param_dtype",
                                         "jt", "n_tiles", "blob_bytes", "algo")] + \
               [("knots", C.c_float * (MAX_K + 1)), ("table", C.c_void_p), ("knots_per_input", C.c_int32),
                ("input_knots", C.c_void_p), ("wide_table", C.c_void_p), ("wide_blob_bytes", C.c_int32),
                ("wide_code_bytes", C.c_int32)]


class _SplineDevLayer(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d", "m", "G", "degree", "boundary", "oob", "value_repr", "knot_span", "jt",
                                         "n_tiles", "coef_blob_bytes", "algo")] + \
               [("ext_knots", C.c_float * (MAX_K + 7)), ("coef_table", C.c_void_p), ("knots_per_input", C.c_int32),
                ("input_ext_knots", C.c_void_p)]


EXPORTS = [
    "lutkan_last_error", "lutkan_last_plan", "lutkan_version", "lutkan_compile", "lutkan_artifact_free", "lutkan_artifact_info",
    "lutkan_artifact_q", "lutkan_artifact_scale", "lutkan_artifact_ymin", "lutkan_artifact_knots",
    "lutkan_artifact_ext_knots", "lutkan_artifact_table", "lutkan_artifact_coef_table",
    "lutkan_artifact_edge_base_scale", "lutkan_artifact_edge_spline_scale", "lutkan_artifact_edge_out_scale",
    "lutkan_dev_layer_init", "bspline_dev_layer_init", "lutkan_forward_workspace_bytes",
    "bspline_forward_workspace_bytes", "lutkan_forward", "lutkan_forward_trace", "bspline_kan_forward",
    "lutkan_model_workspace_bytes", "lutkan_model_forward", "lutkan_chain_forward", "lutkan_forward_locate", "lutkan_forward_edges",
    "bspline_forward_locate", "bspline_forward_edges", "lutkan_probe_launch", "lutkan_artifact_from_arrays",
    "lutkan_error_stats_workspace_bytes", "lutkan_error_stats", "lutkan_forward_static_scratch",
    "lutkan_wide_table_bytes", "lutkan_wide_table_build",
]

_lib = None


def library_path() -> str:
    return _build.LIB


def load_library():
    """Loads liblutkan.so, building it first only when no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()
    lib = C.CDLL(_build.LIB)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    lib.lutkan_last_error.restype = C.c_char_p
    lib.lutkan_last_plan.restype = C.c_char_p
    lib.lutkan_version.restype = C.c_char_p
    lib.lutkan_compile.argtypes = [C.POINTER(_LayerDesc), i32, C.POINTER(vp)]
    lib.lutkan_artifact_from_arrays.argtypes = [C.POINTER(_ArtifactArrays), C.POINTER(vp)]
    lib.lutkan_artifact_free.argtypes = [vp]
    lib.lutkan_artifact_free.restype = None
    lib.lutkan_artifact_info.argtypes = [vp, C.POINTER(_Info)]
    for n in ("q", "scale", "ymin", "knots", "ext_knots", "table", "coef_table", "edge_base_scale", "edge_spline_scale",
              "edge_out_scale"):
        f = getattr(lib, "lutkan_artifact_" + n)
        f.argtypes = [vp]
        f.restype = vp
    lib.lutkan_dev_layer_init.argtypes = [vp, C.POINTER(_DevLayer)]
    lib.bspline_dev_layer_init.argtypes = [vp, C.POINTER(_SplineDevLayer)]
    lib.lutkan_wide_table_bytes.argtypes = [C.POINTER(_DevLayer), C.c_int32]
    lib.lutkan_wide_table_bytes.restype = sz
    lib.lutkan_wide_table_build.argtypes = [C.POINTER(_DevLayer), C.c_int32, vp, sz, vp]
    lib.lutkan_forward_workspace_bytes.argtypes = [C.POINTER(_DevLayer), i64]
    lib.lutkan_forward_workspace_bytes.restype = sz
    lib.bspline_forward_workspace_bytes.argtypes = [C.POINTER(_SplineDevLayer), i64]
    lib.bspline_forward_workspace_bytes.restype = sz
    lib.lutkan_forward.argtypes = [C.POINTER(_DevLayer), vp, i64, vp, vp, vp, sz, vp]
    lib.lutkan_forward_static_scratch.argtypes = [C.POINTER(_DevLayer), vp, i64, vp, vp, vp]
    lib.lutkan_forward_trace.argtypes = [C.POINTER(_DevLayer), vp, i64, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.bspline_kan_forward.argtypes = [C.POINTER(_SplineDevLayer), vp, i64, vp, vp, sz, vp]
    lib.lutkan_forward_locate.argtypes = [C.POINTER(_DevLayer), vp, i64, vp, vp, sz, vp]
    lib.lutkan_forward_edges.argtypes = [C.POINTER(_DevLayer), i64, vp, vp, sz, vp]
    lib.bspline_forward_locate.argtypes = [C.POINTER(_SplineDevLayer), vp, i64, vp, sz, vp]
    lib.bspline_forward_edges.argtypes = [C.POINTER(_SplineDevLayer), i64, vp, vp, sz, vp]
    lib.lutkan_model_workspace_bytes.argtypes = [C.POINTER(_DevLayer), i32, i64]
    lib.lutkan_model_workspace_bytes.restype = sz
    lib.lutkan_model_forward.argtypes = [C.POINTER(_DevLayer), i32, vp, i64, vp, vp, vp, sz, vp]
    lib.lutkan_chain_forward.argtypes = [C.POINTER(_DevLayer), i32, vp, i64, vp, vp, vp, vp]
    lib.lutkan_probe_launch.argtypes = [i32, vp, sz, i32, C.POINTER(C.c_double), vp]
    lib.lutkan_error_stats_workspace_bytes.argtypes = [i64]
    lib.lutkan_error_stats_workspace_bytes.restype = sz
    lib.lutkan_error_stats.argtypes = [vp, vp, i64, i32, vp, i32, C.c_float, C.c_float, vp, i32, vp, vp, sz, vp]
    _lib = lib
    return lib


def lutkan_last_error() -> str:
    return load_library().lutkan_last_error().decode()


def lutkan_last_plan() -> str:
    """Which kernels the last forward call of this thread launched (one clause per launch)."""
    return load_library().lutkan_last_plan().decode()


def lutkan_version() -> str:
    return load_library().lutkan_version().decode()


def _check(rc: int):
    if rc != 0:
        raise LutKanError(f"[{rc}] {lutkan_last_error()}")


def _view(ptr, nbytes, dtype, shape, owner):
    """numpy view of library-owned host memory; the view keeps `owner` (the Artifact) alive."""
    buf = (C.c_char * nbytes).from_address(ptr)
    buf._owner = owner
    return np.frombuffer(buf, dtype=dtype).reshape(shape)


class Artifact:
    """Host LUT artifact (Sec. 4.6) owned by the library.  The array attributes are numpy views of the library's
    memory, made on access; each view keeps the artifact alive, and the artifact is freed with its last reference."""

    def __init__(self, handle):
        self._h = handle
        info = _Info()
        _check(load_library().lutkan_artifact_info(handle, C.byref(info)))
        self.info = info

    def _array(self, getter, count, dtype, shape):
        return _view(getattr(load_library(), getter)(self._h), count * np.dtype(dtype).itemsize, dtype, shape, self)

    @property
    def q(self):
        E, K, L = self.info.d * self.info.m, self.info.K, self.info.L
        return self._array("lutkan_artifact_q", E * K * L, np.int8 if self.info.scheme == SYM_INT8 else np.uint8, (E, K, L))

    @property
    def scale(self):
        E, K = self.info.d * self.info.m, self.info.K
        return self._array("lutkan_artifact_scale", E * K, np.float32, (E, K))

    @property
    def y_min(self):
        E, K = self.info.d * self.info.m, self.info.K
        return self._array("lutkan_artifact_ymin", E * K, np.float32, (E, K))

    @property
    def knots(self):
        """[K+1], or [d, K+1] with one knot vector per input."""
        I = self.info
        shape = (I.d, I.K + 1) if I.knots_per_input else (I.K + 1,)
        return self._array("lutkan_artifact_knots", int(np.prod(shape)), np.float32, shape)

    @property
    def ext_knots(self):
        """None for an artifact rebuilt from stored arrays (it has no spline side)."""
        I = self.info
        shape = (I.d, I.G + 7) if I.knots_per_input else (I.G + 7,)
        return self._array("lutkan_artifact_ext_knots", int(np.prod(shape)), np.float32, shape) if I.G > 0 else None

    @property
    def table(self):
        return self._array("lutkan_artifact_table", self.info.table_bytes, np.uint8, (self.info.table_bytes,))

    @property
    def coef_table(self):
        n = self.info.coef_table_bytes // 4
        return self._array("lutkan_artifact_coef_table", n, np.float32, (n,)) if self.info.G > 0 else None

    @property
    def edge_scales(self):
        """(s_base, s_spline, s_out), each [E], with value_repr = spline_component; else None."""
        if self.info.value_repr != REPR_SPLINE_COMPONENT:
            return None
        E = self.info.d * self.info.m
        return tuple(self._array("lutkan_artifact_edge_" + n, E, np.float32, (E,)) for n in ("base_scale", "spline_scale", "out_scale"))

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.lutkan_artifact_free(h)

    def save(self, path: str) -> None:
        """Writes the artifact as a compressed NPZ whose `manifest` entry is the JSON manifest (Sec. 4.6): metadata
        format_version, value_repr, interp, boundary_mode, oob_policy, scheme; grid knots, L; tables q_table, scale,
        y_min (float16 arrays with float16 parameters); the reconstruction scalars and base_kind with
        spline_component."""
        I = self.info
        pdt = np.float16 if I.param_dtype == PARAM_FP16 else np.float32
        manifest = {"format_version": 1, "value_repr": "spline_component" if I.value_repr == REPR_SPLINE_COMPONENT else "phi",
                    "interp": "linear", "boundary_mode": "closed" if I.boundary == CLOSED else "half_open",
                    "oob_policy": "zero_spline" if I.oob == ZERO_SPLINE else "clip_x",
                    "scheme": "symmetric_int8" if I.scheme == SYM_INT8 else "asymmetric_uint8",
                    "L": int(I.L), "K": int(I.K), "in_features": int(I.d), "out_features": int(I.m),
                    "param_dtype": "float16" if I.param_dtype == PARAM_FP16 else "float32",
                    "knots_per_input": bool(I.knots_per_input)}
        arrays = {"knots": self.knots, "q_table": self.q, "scale": self.scale.astype(pdt), "y_min": self.y_min.astype(pdt)}
        if self.edge_scales is not None:
            manifest["base_kind"] = "silu"
            arrays.update(edge_base_scale=self.edge_scales[0], edge_spline_scale=self.edge_scales[1],
                          edge_out_scale=self.edge_scales[2])
        with open(path, "wb") as f:
            np.savez_compressed(f, manifest=np.frombuffer(json.dumps(manifest, sort_keys=True).encode(), dtype=np.uint8),
                                **arrays)

    def to_device(self, device="cuda:0", algo: int = ALGO_AUTO, wide=None) -> "LutLayer":
        """wide: also hold a wide form of the table (lutkan_wide_table_build).  2: binary16 codes; 4: fp32 values;
        True: fp32 values if the layer has that form, else binary16 codes; False: none.  None: for layers of at
        least 4096 edges, fp32 values if the layer has that form, else (symmetric int8 only) binary16 codes."""
        return LutLayer(self, device, algo, wide)

    def bspline_to_device(self, device="cuda:0", algo: int = ALGO_AUTO) -> "BsplineLayer":
        return BsplineLayer(self, device, algo)


def lutkan_compile(d: int, m: int, G: int, degree: int, ext_knots, coef, L: int, scheme: int, boundary: int,
                   oob: int, n_threads: int = 0, edge_scales=None, param_dtype: int = PARAM_FP32,
                   knot_span: int = SPAN_DOMAIN, knots_per_input: bool = False) -> Artifact:
    """Host-only LUT compilation of one dense B-spline KAN layer (Sec. 4.2-4.6).
    knots_per_input: ext_knots is [d, G + 2*degree + 1], one knot vector per input dimension (Sec. 6.2).
    edge_scales = (s_base, s_spline, s_out), each [d, m], selects value_repr = spline_component (Eq. 2).
    param_dtype = PARAM_FP16 stores scale and y_min as binary16 values (Sec. 4.6).
    knot_span = SPAN_EXTENDED makes every interval of the extended knot vector a LUT segment (K = G + 2*degree)."""
    lib = load_library()
    tau = np.ascontiguousarray(ext_knots, dtype=np.float32)
    cf = np.ascontiguousarray(coef, dtype=np.float32)
    if tau.size != (d if knots_per_input else 1) * (G + 2 * degree + 1) or cf.size != d * m * (G + degree):
        raise LutKanError("lutkan_compile: ext_knots / coef have the wrong number of elements")
    keep = [np.ascontiguousarray(a, dtype=np.float32).reshape(-1) for a in edge_scales] if edge_scales is not None else []
    if keep and any(a.size != d * m for a in keep):
        raise LutKanError("lutkan_compile: every edge scale array needs d*m elements")
    desc = _LayerDesc(d, m, G, degree, tau.ctypes.data, cf.ctypes.data, L, scheme, boundary, oob,
                      REPR_SPLINE_COMPONENT if keep else REPR_PHI, *[a.ctypes.data for a in keep])
    desc.param_dtype = param_dtype
    desc.knot_span = knot_span
    desc.knots_per_input = int(bool(knots_per_input))
    out = C.c_void_p()
    _check(lib.lutkan_compile(C.byref(desc), n_threads, C.byref(out)))
    return Artifact(out.value)


def lutkan_artifact_from_arrays(d: int, m: int, knots, q_table, scale, y_min, boundary: int, oob: int,
                                edge_scales=None, param_dtype: int = PARAM_FP32, knots_per_input: bool = False) -> Artifact:
    """Artifact (with its device table) from stored arrays: q_table int8 (symmetric) or uint8 (asymmetric) [d*m, K, L];
    knots [K+1], or [d, K+1] with knots_per_input."""
    q = np.ascontiguousarray(q_table)
    if q.dtype not in (np.int8, np.uint8) or q.ndim != 3 or q.shape[0] != d * m:
        raise LutKanError("lutkan_artifact_from_arrays: q_table must be int8 or uint8 with shape [d*m, K, L]")
    K, L = int(q.shape[1]), int(q.shape[2])
    kn = np.ascontiguousarray(knots, dtype=np.float32).reshape(-1)
    sc = np.ascontiguousarray(scale, dtype=np.float32).reshape(-1)
    ym = np.ascontiguousarray(y_min, dtype=np.float32).reshape(-1)
    if kn.size != (d if knots_per_input else 1) * (K + 1) or sc.size != d * m * K or ym.size != d * m * K:
        raise LutKanError("lutkan_artifact_from_arrays: knots / scale / y_min do not match q_table's shape")
    keep = [np.ascontiguousarray(a, dtype=np.float32).reshape(-1) for a in edge_scales] if edge_scales is not None else []
    if keep and any(a.size != d * m for a in keep):
        raise LutKanError("lutkan_artifact_from_arrays: every edge scale array needs d*m elements")
    arr = _ArtifactArrays(d, m, K, L, SYM_INT8 if q.dtype == np.int8 else ASYM_UINT8, boundary, oob,
                          REPR_SPLINE_COMPONENT if keep else REPR_PHI, param_dtype, int(bool(knots_per_input)),
                          kn.ctypes.data, q.ctypes.data,
                          sc.ctypes.data, ym.ctypes.data, *[a.ctypes.data for a in keep])
    out = C.c_void_p()
    _check(load_library().lutkan_artifact_from_arrays(C.byref(arr), C.byref(out)))
    return Artifact(out.value)


def lutkan_artifact_load(path: str) -> Artifact:
    """Reads an artifact written by Artifact.save (NPZ + JSON manifest, Sec. 4.6).  Nothing in the file is executed."""
    with np.load(path, allow_pickle=False) as z:
        man = json.loads(bytes(z["manifest"]).decode())
        if man.get("format_version") != 1 or man.get("interp") != "linear":
            raise LutKanError(f"lutkan_artifact_load: unsupported manifest {man}")
        names = {"boundary_mode": {"half_open": HALF_OPEN, "closed": CLOSED}, "oob_policy": {"clip_x": CLIP_X, "zero_spline": ZERO_SPLINE},
                 "scheme": {"symmetric_int8": SYM_INT8, "asymmetric_uint8": ASYM_UINT8}, "param_dtype": {"float32": PARAM_FP32, "float16": PARAM_FP16},
                 "value_repr": {"phi": REPR_PHI, "spline_component": REPR_SPLINE_COMPONENT}}
        try:
            f = {k: v[man[k]] for k, v in names.items()}
        except KeyError as e:
            raise LutKanError(f"lutkan_artifact_load: bad manifest field {e}") from None
        q = z["q_table"]
        if (q.dtype == np.int8) != (f["scheme"] == SYM_INT8):
            raise LutKanError("lutkan_artifact_load: q_table dtype does not match the manifest's scheme")
        scales = None
        if f["value_repr"] == REPR_SPLINE_COMPONENT:
            if man.get("base_kind") != "silu":
                raise LutKanError("lutkan_artifact_load: only base_kind = silu is supported")
            scales = (z["edge_base_scale"], z["edge_spline_scale"], z["edge_out_scale"])
        return lutkan_artifact_from_arrays(int(man["in_features"]), int(man["out_features"]), z["knots"], q, z["scale"],
                                           z["y_min"], f["boundary_mode"], f["oob_policy"], scales, f["param_dtype"],
                                           bool(man.get("knots_per_input", False)))


def _torch():
    import torch
    return torch


def _upload(arr: np.ndarray, device):
    torch = _torch()
    return torch.from_numpy(arr).to(device)


class LutLayer:
    """Device-side LUT layer: the lutkan_dev_layer struct plus the torch tensor that owns its table."""

    def __init__(self, art: Artifact, device, algo: int = ALGO_AUTO, wide=None):
        lib = load_library()
        self.c = _DevLayer()
        _check(lib.lutkan_dev_layer_init(art._h, C.byref(self.c)))
        self.c.algo = algo
        self.table = _upload(art.table, device)
        self.c.table = self.table.data_ptr()
        self.input_knots = _upload(art.knots, device) if art.info.knots_per_input else None     # [d, K+1]
        self.c.input_knots = self.input_knots.data_ptr() if self.input_knots is not None else None
        self.device = self.table.device
        self.d, self.m = self.c.d, self.c.m
        self.wide_table = None
        n_wide = {cb: lib.lutkan_wide_table_bytes(C.byref(self.c), cb) for cb in (2, 4)}
        if wide is None or wide is True:
            asked = wide is True
            wide = 4 if n_wide[4] else 2 if n_wide[2] else 0
            if not asked:               # what the launch planning would ever pick, on a layer of some size
                if self.d * self.m < 4096 or (wide == 2 and self.c.scheme != SYM_INT8):
                    wide = 0
            elif not wide:
                raise LutKanError("this layer has no wide table form")
        if wide:
            torch = _torch()
            if wide not in (2, 4):
                raise LutKanError("wide: 2 (binary16 codes) or 4 (fp32 values)")
            if n_wide[wide] == 0:
                raise LutKanError("this layer has no wide table form of %d bytes per code" % wide)
            self.wide_table = torch.empty(n_wide[wide], dtype=torch.uint8, device=self.device)
            with torch.cuda.device(self.device):
                _check(lib.lutkan_wide_table_build(C.byref(self.c), wide, self.wide_table.data_ptr(), n_wide[wide], _stream(self.device)))

    def with_contract(self, boundary: int, oob: int, algo: Optional[int] = None) -> "LutLayer":
        """Same tables under another boundary_mode / oob_policy (the contract is not baked into the codes)."""
        other = object.__new__(LutLayer)
        other.c = _DevLayer.from_buffer_copy(self.c)
        other.c.boundary, other.c.oob = boundary, oob
        if algo is not None:
            other.c.algo = algo
        other.table, other.device, other.d, other.m = self.table, self.device, self.d, self.m
        other.input_knots, other.wide_table = self.input_knots, self.wide_table
        return other


class BsplineLayer:
    def __init__(self, art: Artifact, device, algo: int = ALGO_AUTO):
        self.c = _SplineDevLayer()
        _check(load_library().bspline_dev_layer_init(art._h, C.byref(self.c)))
        self.c.algo = algo
        self.coef_table = _upload(art.coef_table, device)
        self.c.coef_table = self.coef_table.data_ptr()
        self.input_ext_knots = _upload(art.ext_knots, device) if art.info.knots_per_input else None   # [d, G+7]
        self.c.input_ext_knots = self.input_ext_knots.data_ptr() if self.input_ext_knots is not None else None
        self.device = self.coef_table.device
        self.d, self.m = self.c.d, self.c.m

    def with_contract(self, boundary: int, oob: int, algo: Optional[int] = None) -> "BsplineLayer":
        other = object.__new__(BsplineLayer)
        other.c = _SplineDevLayer.from_buffer_copy(self.c)
        other.c.boundary, other.c.oob = boundary, oob
        if algo is not None:
            other.c.algo = algo
        other.coef_table, other.device, other.d, other.m = self.coef_table, self.device, self.d, self.m
        other.input_ext_knots = self.input_ext_knots
        return other


def _stream(device) -> int:
    return _torch().cuda.current_stream(device).cuda_stream


def _require(t, dtype, what):
    torch = _torch()
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise LutKanError(f"{what} must be a contiguous CUDA tensor of dtype {dtype}")


def _check_io(who, layer, x=None, y=None, workspace=None, stats=None, n_stats=1):
    """Shapes, dtypes and devices of the tensors handed to a forward call, checked before any pointer reaches the
    library: the kernels index x as [B, d] and y as [B, m] on trust.  Returns B."""
    torch = _torch()
    B = None
    for t, what, width in ((x, "x", layer.d), (y, "y", layer.m)):
        if t is None:
            continue
        if not isinstance(t, torch.Tensor) or t.dtype != torch.float32 or t.dim() != 2 or t.shape[1] != width:
            raise LutKanError(f"{who}: {what} must be a float32 tensor of shape [B, {width}]")
        if B is not None and t.shape[0] != B:
            raise LutKanError(f"{who}: y must have as many rows as x ({B})")
        B = t.shape[0]
    if stats is not None and (not isinstance(stats, torch.Tensor) or stats.dtype != torch.int64 or stats.numel() != 2 * n_stats):
        raise LutKanError(f"{who}: stats must be an int64 tensor of {2 * n_stats} elements")
    if workspace is not None and (not isinstance(workspace, torch.Tensor) or workspace.dtype != torch.uint8):
        raise LutKanError(f"{who}: workspace must be a uint8 tensor")
    for t, what in ((x, "x"), (y, "y"), (workspace, "workspace"), (stats, "stats")):
        if t is None:
            continue
        if not t.is_cuda or not t.is_contiguous():
            raise LutKanError(f"{who}: {what} must be a contiguous CUDA tensor")
        if t.device != layer.device:
            raise LutKanError(f"{who}: {what} is on {t.device}, the layer's tables are on {layer.device}")
    return B


def _check_chain(who, layers):
    if len(layers) < 1:
        raise LutKanError(f"{who}: need at least one layer")
    if any(l.device != layers[0].device for l in layers):        # (that the widths chain is the library's own check)
        raise LutKanError(f"{who}: the layers' tables must be on one device")
    return SimpleNamespace(d=layers[0].d, m=layers[-1].m, device=layers[0].device)


def lutkan_forward_workspace_bytes(layer: LutLayer, B: int) -> int:
    return int(load_library().lutkan_forward_workspace_bytes(C.byref(layer.c), B))


def bspline_forward_workspace_bytes(layer: BsplineLayer, B: int) -> int:
    return int(load_library().bspline_forward_workspace_bytes(C.byref(layer.c), B))


def lutkan_model_workspace_bytes(layers: Sequence[LutLayer], B: int) -> int:
    arr = (_DevLayer * len(layers))(*[l.c for l in layers])
    return int(load_library().lutkan_model_workspace_bytes(arr, len(layers), B))


def _workspace(nbytes, device, workspace):
    torch = _torch()
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    _require(workspace, torch.uint8, "workspace")
    return workspace


def lutkan_forward(layer: LutLayer, x, y=None, stats=None, workspace=None):
    """y[B,m] = LUT layer forward of x[B,d] on the current stream.  stats: optional int64[2] CUDA tensor (added to)."""
    torch = _torch()
    B = _check_io("lutkan_forward", layer, x=x, y=y, workspace=workspace, stats=stats)
    if y is None:
        y = torch.empty((B, layer.m), dtype=torch.float32, device=x.device)
    ws = _workspace(lutkan_forward_workspace_bytes(layer, B), x.device, workspace)
    _check(load_library().lutkan_forward(C.byref(layer.c), x.data_ptr(), B, y.data_ptr(),
                                         stats.data_ptr() if stats is not None else None,
                                         ws.data_ptr(), ws.numel(), _stream(x.device)))
    return y


STATIC_SCRATCH_BYTES = 64 << 20


def lutkan_forward_static_scratch(layer: LutLayer, x, y, stats=None):
    """lutkan_forward without a workspace: the scratch is an array inside the library (see lutkan.h).  Nothing is
    allocated, here or in the library, so the caller brings y."""
    if y is None:
        raise LutKanError("lutkan_forward_static_scratch: the caller brings y")
    B = _check_io("lutkan_forward_static_scratch", layer, x=x, y=y, stats=stats)
    _check(load_library().lutkan_forward_static_scratch(C.byref(layer.c), x.data_ptr(), B, y.data_ptr(),
                                                        stats.data_ptr() if stats is not None else None,
                                                        _stream(x.device)))
    return y


def lutkan_forward_locate(layer: LutLayer, x, workspace, stats=None):
    """Phase 1 of lutkan_forward: fills `workspace` with the per-(row,input) lookup records."""
    B = _check_io("lutkan_forward_locate", layer, x=x, workspace=workspace, stats=stats)
    _check(load_library().lutkan_forward_locate(C.byref(layer.c), x.data_ptr(), B,
                                                stats.data_ptr() if stats is not None else None,
                                                workspace.data_ptr(), workspace.numel(), _stream(x.device)))


def lutkan_forward_edges(layer: LutLayer, B: int, y, workspace):
    """Phase 2 of lutkan_forward: gathers, dequantises, interpolates and sums from the records that
    lutkan_forward_locate left in `workspace` for the same layer and the same B."""
    if _check_io("lutkan_forward_edges", layer, y=y, workspace=workspace) != B:
        raise LutKanError(f"lutkan_forward_edges: y must have B = {B} rows")
    _check(load_library().lutkan_forward_edges(C.byref(layer.c), B, y.data_ptr(), workspace.data_ptr(),
                                               workspace.numel(), _stream(y.device)))
    return y


def bspline_forward_locate(layer: "BsplineLayer", x, workspace):
    B = _check_io("bspline_forward_locate", layer, x=x, workspace=workspace)
    _check(load_library().bspline_forward_locate(C.byref(layer.c), x.data_ptr(), B, workspace.data_ptr(),
                                                 workspace.numel(), _stream(x.device)))


def bspline_forward_edges(layer: "BsplineLayer", B: int, y, workspace):
    if _check_io("bspline_forward_edges", layer, y=y, workspace=workspace) != B:
        raise LutKanError(f"bspline_forward_edges: y must have B = {B} rows")
    _check(load_library().bspline_forward_edges(C.byref(layer.c), B, y.data_ptr(), workspace.data_ptr(),
                                                workspace.numel(), _stream(y.device)))
    return y


def lutkan_forward_trace(layer: LutLayer, x, codes: bool = False, workspace=None):
    """Forward plus the bit-exact quantities of the contract: (y, k, l0, inside, w, q01 or None)."""
    torch = _torch()
    B = _check_io("lutkan_forward_trace", layer, x=x, workspace=workspace)
    d, m = layer.d, layer.m
    dev = x.device
    y = torch.empty((B, m), dtype=torch.float32, device=dev)
    k = torch.empty((B, d), dtype=torch.int32, device=dev)
    l0 = torch.empty((B, d), dtype=torch.int32, device=dev)
    inside = torch.empty((B, d), dtype=torch.uint8, device=dev)
    w = torch.empty((B, d), dtype=torch.float32, device=dev)
    q01 = torch.empty((B, d, m, 2), dtype=torch.int16, device=dev) if codes else None
    ws = _workspace(lutkan_forward_workspace_bytes(layer, B), dev, workspace)
    _check(load_library().lutkan_forward_trace(C.byref(layer.c), x.data_ptr(), B, y.data_ptr(), k.data_ptr(),
                                               l0.data_ptr(), inside.data_ptr(), w.data_ptr(),
                                               q01.data_ptr() if codes else None, ws.data_ptr(), ws.numel(),
                                               _stream(dev)))
    return y, k, l0, inside, w, q01


def bspline_kan_forward(layer: BsplineLayer, x, y=None, workspace=None):
    torch = _torch()
    B = _check_io("bspline_kan_forward", layer, x=x, y=y, workspace=workspace)
    if y is None:
        y = torch.empty((B, layer.m), dtype=torch.float32, device=x.device)
    ws = _workspace(bspline_forward_workspace_bytes(layer, B), x.device, workspace)
    _check(load_library().bspline_kan_forward(C.byref(layer.c), x.data_ptr(), B, y.data_ptr(), ws.data_ptr(),
                                              ws.numel(), _stream(x.device)))
    return y


def lutkan_model_forward(layers: List[LutLayer], x, y=None, stats=None, workspace=None):
    """Chained forward: layer l's output is layer l+1's input.  stats: optional int64[n_layers,2] CUDA tensor."""
    torch = _torch()
    ends = _check_chain("lutkan_model_forward", layers)
    B = _check_io("lutkan_model_forward", ends, x=x, y=y, workspace=workspace, stats=stats, n_stats=len(layers))
    arr = (_DevLayer * len(layers))(*[l.c for l in layers])
    if y is None:
        y = torch.empty((B, layers[-1].m), dtype=torch.float32, device=x.device)
    need = int(load_library().lutkan_model_workspace_bytes(arr, len(layers), B))
    ws = _workspace(need, x.device, workspace)
    _check(load_library().lutkan_model_forward(arr, len(layers), x.data_ptr(), B, y.data_ptr(),
                                               stats.data_ptr() if stats is not None else None,
                                               ws.data_ptr(), ws.numel(), _stream(x.device)))
    return y


def lutkan_chain_forward(layers: List[LutLayer], x, y=None, stats=None, hidden=None):
    """The chain in one launch (narrow layers, small batches; see lutkan.h).  hidden: optional float32 CUDA tensor of
    sum_{l < n-1} B*m_l elements that receives the activations between the layers."""
    torch = _torch()
    ends = _check_chain("lutkan_chain_forward", layers)
    B = _check_io("lutkan_chain_forward", ends, x=x, y=y, stats=stats, n_stats=len(layers))
    arr = (_DevLayer * len(layers))(*[l.c for l in layers])
    if y is None:
        y = torch.empty((B, layers[-1].m), dtype=torch.float32, device=x.device)
    if hidden is not None:
        _require(hidden, torch.float32, "hidden")
        if hidden.numel() < B * sum(l.m for l in layers[:-1]) or hidden.device != x.device:
            raise LutKanError("lutkan_chain_forward: hidden is too small or on another device")
    _check(load_library().lutkan_chain_forward(arr, len(layers), x.data_ptr(), B, y.data_ptr(),
                                               hidden.data_ptr() if hidden is not None else None,
                                               stats.data_ptr() if stats is not None else None, _stream(x.device)))
    return y


def lutkan_probe_launch(kind: int, buffer, iters: int) -> float:
    """Launches one measurement kernel (see lutkan.h) on the current stream; returns the flop or bytes it performs."""
    torch = _torch()
    if not buffer.is_cuda or not buffer.is_contiguous():
        raise LutKanError("lutkan_probe_launch: buffer must be a contiguous device tensor")
    work = C.c_double(0.0)
    _check(load_library().lutkan_probe_launch(kind, buffer.data_ptr(), buffer.numel() * buffer.element_size(), iters,
                                              C.byref(work), _stream(buffer.device)))
    return work.value


def lutkan_error_stats(y, y_ref, x, t0: float, tK: float, boundary: int, input_domain=None) -> dict:
    """|y - y_ref| statistics on the in-range and the OOB-only samples (Sec. 5.6), reduced on the device.
    input_domain: optional device tensor [d, 2] fp32 of per-input {t0, tK} (layers with one knot vector per input).
    Returns the fields of lutkan_error_summary as a dict: rows_in, rows_oob, nan_in, nan_oob, sum_abs_*, max_abs_*,
    mae_* and oob_any_frac, all computed on the device."""
    torch = _torch()
    for t, what in ((y, "y"), (y_ref, "y_ref"), (x, "x")):
        _require(t, torch.float32, what)
    if y.dim() != 2 or x.dim() != 2:
        raise LutKanError("lutkan_error_stats: y, y_ref must be [B,m] and x [B,d]")
    B, m, d = y.shape[0], y.shape[1], x.shape[1]
    if y_ref.shape != y.shape or x.shape[0] != B:
        raise LutKanError("lutkan_error_stats: y, y_ref must be [B,m] and x [B,d]")
    if y_ref.device != y.device or x.device != y.device:
        raise LutKanError("lutkan_error_stats: y, y_ref and x must be on one device")
    if input_domain is not None:
        _require(input_domain, torch.float32, "input_domain")
        if tuple(input_domain.shape) != (d, 2) or input_domain.device != y.device:
            raise LutKanError("lutkan_error_stats: input_domain must be [d, 2] on the device of y")
    lib = load_library()
    out = torch.zeros(_ERROR_SUMMARY_WORDS, dtype=torch.float64, device=y.device)
    ws = torch.empty(max(16, lib.lutkan_error_stats_workspace_bytes(B)), dtype=torch.uint8, device=y.device)
    _check(lib.lutkan_error_stats(y.data_ptr(), y_ref.data_ptr(), B, m, x.data_ptr(), d, float(t0), float(tK),
                                  input_domain.data_ptr() if input_domain is not None else None, boundary,
                                  out.data_ptr(), ws.data_ptr(), ws.numel(), _stream(y.device)))
    raw = out.cpu().numpy()
    res = {name: int(v) for name, v in zip(_ERROR_SUMMARY_COUNTS, raw[:4].view(np.uint64))}
    res.update({name: float(v) for name, v in zip(_ERROR_SUMMARY_REALS, raw[4:])})
    return res


# lutkan_error_summary: four uint64 counters, then seven doubles
_ERROR_SUMMARY_COUNTS = ("rows_in", "rows_oob", "nan_in", "nan_oob")
_ERROR_SUMMARY_REALS = ("sum_abs_in", "sum_abs_oob", "max_abs_in", "max_abs_oob", "mae_in", "mae_oob", "oob_any_frac")
_ERROR_SUMMARY_WORDS = len(_ERROR_SUMMARY_COUNTS) + len(_ERROR_SUMMARY_REALS)
