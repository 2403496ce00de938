"""Thin ctypes binding of libxl.so: argument marshalling only.

Every step of the hot path runs inside the library's HIP kernels; PyTorch is
used by callers for device memory and streams.  The names mirror include/xl.h.
There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("XL_LIBRARY_PATH") or os.path.join(_HERE, "libxl.so")

XL_OK = 0
XL_E_NULL, XL_E_SHAPE, XL_E_UNSUPPORTED, XL_E_LDS_BUDGET = -1, -2, -3, -4
XL_E_DEVICE, XL_E_ALIGN, XL_E_LAUNCH, XL_E_GRAPH, XL_E_STATE, XL_E_SCRATCH = -5, -6, -7, -8, -9, -10
XL_STATIC_SCRATCH_BYTES = 64 << 20

XL_CONV, XL_MAXPOOL, XL_GLOBAL_AVGPOOL, XL_ADD, XL_CONCAT = 0, 1, 2, 3, 4
XL_SINGLE, XL_STRAIGHT, XL_SPLIT, XL_MERGE = 0, 1, 2, 3

OPS = {"conv": XL_CONV, "maxpool": XL_MAXPOOL, "gap": XL_GLOBAL_AVGPOOL, "add": XL_ADD, "concat": XL_CONCAT}
MODES = {"single": XL_SINGLE, "straight": XL_STRAIGHT, "split": XL_SPLIT, "merge": XL_MERGE}

# every symbol include/xl.h declares
EXPORTS = [
    "xl_plan_create", "xl_plan_destroy", "xl_plan_num_groups", "xl_plan_query", "xl_plan_workspace_bytes",
    "xl_prepare", "xl_run", "xl_tune", "xl_plan_num_launches", "xl_tuner_candidates", "xl_required_extent",
    "xl_strerror", "xl_plan_last_error", "xl_version",
    "xl_plan_num_candidates", "xl_plan_candidate_info", "xl_plan_select_candidate", "xl_run_static", "xl_profile", "xl_measure_peaks",
    "xl_plan_set_block_fused", "xl_plan_block_is_fused",
]


class xl_shape(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int), ("c", ctypes.c_int), ("h", ctypes.c_int), ("w", ctypes.c_int)]


class xl_layer(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int), ("in_", ctypes.c_int * 2), ("out", ctypes.c_int),
                ("cin", ctypes.c_int), ("cout", ctypes.c_int),
                ("k", ctypes.c_int), ("stride", ctypes.c_int), ("pad", ctypes.c_int), ("groups", ctypes.c_int),
                ("relu", ctypes.c_int),
                ("w_slot", ctypes.c_int), ("scale_slot", ctypes.c_int), ("shift_slot", ctypes.c_int)]


class xl_group(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int), ("nlayers", ctypes.c_int), ("layer_ids", ctypes.POINTER(ctypes.c_int))]


class xl_options(ctypes.Structure):
    _fields_ = [("lds_budget_bytes", ctypes.c_int), ("num_cus", ctypes.c_int),
                ("force_tile_h", ctypes.c_int), ("force_tile_w", ctypes.c_int),
                ("force_cout_split", ctypes.c_int), ("paper_tuner_only", ctypes.c_int),
                ("force_threads", ctypes.c_int), ("precision", ctypes.c_int),
                ("keep_blocks_fused", ctypes.c_int)]


class xl_group_info(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int), ("first_layer", ctypes.c_int), ("nlayers", ctypes.c_int),
                ("tile_h", ctypes.c_int), ("tile_w", ctypes.c_int),
                ("mid_h", ctypes.c_int), ("mid_w", ctypes.c_int),
                ("in_h", ctypes.c_int), ("in_w", ctypes.c_int),
                ("tiles_y", ctypes.c_int), ("tiles_x", ctypes.c_int),
                ("cout_split", ctypes.c_int), ("workgroups", ctypes.c_int), ("threads", ctypes.c_int),
                ("lds_bytes", ctypes.c_int), ("workgroups_per_cu", ctypes.c_int), ("chunk_channels", ctypes.c_int),
                ("bytes_fused", ctypes.c_longlong), ("bytes_unfused", ctypes.c_longlong),
                ("stores_fused", ctypes.c_longlong), ("stores_unfused", ctypes.c_longlong),
                ("flops", ctypes.c_longlong), ("flops_executed", ctypes.c_longlong),
                ("redundancy", ctypes.c_double), ("precision", ctypes.c_int)]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_}


class xl_launch_info(ctypes.Structure):
    _fields_ = [("group", ctypes.c_int), ("first_layer", ctypes.c_int), ("nlayers", ctypes.c_int),
                ("is_block_kernel", ctypes.c_int), ("candidate", ctypes.c_int), ("variant", ctypes.c_int),
                ("tile_h", ctypes.c_int), ("tile_w", ctypes.c_int), ("threads", ctypes.c_int),
                ("cout_split", ctypes.c_int), ("waves_cout_1", ctypes.c_int), ("waves_cout_2", ctypes.c_int),
                ("chunk_channels", ctypes.c_int), ("lds_bytes", ctypes.c_int), ("workgroups", ctypes.c_int),
                ("precision", ctypes.c_int), ("model_cost_us", ctypes.c_double)]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_}


class XlError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"xl status {status}: {message}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Load libxl.so (raises OSError when it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError(f"{LIB_PATH} is missing: run `python -m paper_2007_06000_amd.build` (there is no fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i = ctypes.c_void_p, ctypes.c_int
        L.xl_plan_create.argtypes = [ctypes.POINTER(xl_layer), i, ctypes.POINTER(xl_shape), i,
                                     ctypes.POINTER(xl_group), i, i, ctypes.POINTER(xl_options),
                                     ctypes.POINTER(vp)]
        L.xl_plan_create.restype = i
        L.xl_plan_destroy.argtypes = [vp]
        L.xl_plan_destroy.restype = None
        L.xl_plan_num_groups.argtypes = [vp]
        L.xl_plan_num_groups.restype = i
        L.xl_plan_query.argtypes = [vp, i, ctypes.POINTER(xl_group_info)]
        L.xl_plan_query.restype = i
        L.xl_plan_workspace_bytes.argtypes = [vp]
        L.xl_plan_workspace_bytes.restype = ctypes.c_size_t
        L.xl_prepare.argtypes = [vp, ctypes.POINTER(vp), i, vp, vp]
        L.xl_prepare.restype = i
        L.xl_run.argtypes = [vp, ctypes.POINTER(vp), i, vp, vp, i]
        L.xl_run.restype = i
        L.xl_tune.argtypes = [vp, ctypes.POINTER(vp), i, vp, vp, i]
        L.xl_tune.restype = i
        L.xl_plan_num_launches.argtypes = [vp, i]
        L.xl_plan_num_launches.restype = i
        L.xl_tuner_candidates.argtypes = [i, ctypes.POINTER(i), ctypes.POINTER(i), i]
        L.xl_tuner_candidates.restype = i
        L.xl_required_extent.argtypes = [i, i, i]
        L.xl_required_extent.restype = i
        L.xl_strerror.argtypes = [i]
        L.xl_strerror.restype = ctypes.c_char_p
        L.xl_plan_last_error.argtypes = [vp]
        L.xl_plan_last_error.restype = ctypes.c_char_p
        L.xl_plan_num_candidates.argtypes = [vp, i, i]
        L.xl_plan_num_candidates.restype = i
        L.xl_plan_candidate_info.argtypes = [vp, i, i, i, ctypes.POINTER(xl_launch_info)]
        L.xl_plan_candidate_info.restype = i
        L.xl_plan_select_candidate.argtypes = [vp, i, i, i]
        L.xl_plan_select_candidate.restype = i
        L.xl_plan_set_block_fused.argtypes = [vp, i, i]
        L.xl_plan_set_block_fused.restype = i
        L.xl_plan_block_is_fused.argtypes = [vp, i]
        L.xl_plan_block_is_fused.restype = i
        L.xl_run_static.argtypes = [vp, ctypes.POINTER(vp), i, ctypes.POINTER(vp), i, vp, i, i]
        L.xl_run_static.restype = i
        L.xl_profile.argtypes = [vp, ctypes.POINTER(vp), i, vp, vp, i, i, ctypes.POINTER(ctypes.c_float), i]
        L.xl_profile.restype = i
        dp = ctypes.POINTER(ctypes.c_double)
        L.xl_measure_peaks.argtypes = [vp, vp, ctypes.c_size_t, vp, dp, dp, dp, dp]
        L.xl_measure_peaks.restype = i
        L.xl_version.argtypes = []
        L.xl_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def xl_version() -> str:
    return lib().xl_version().decode()


def xl_strerror(status: int) -> str:
    return lib().xl_strerror(status).decode()


def xl_tuner_candidates(out_size: int) -> List[tuple]:
    n = lib().xl_tuner_candidates(out_size, None, None, 0)
    t = (ctypes.c_int * max(n, 1))()
    g = (ctypes.c_int * max(n, 1))()
    lib().xl_tuner_candidates(out_size, t, g, n)
    return [(t[i], g[i]) for i in range(n)]


def xl_required_extent(t: int, k: int, stride: int) -> int:
    return lib().xl_required_extent(t, k, stride)


def xl_measure_peaks(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> dict:
    """Measured copy bandwidth and arithmetic rates of the current device (see include/xl.h)."""
    v = [ctypes.c_double() for _ in range(4)]
    st = lib().xl_measure_peaks(ctypes.c_void_p(dst_ptr), ctypes.c_void_p(src_ptr), nbytes, ctypes.c_void_p(stream),
                                *[ctypes.byref(d) for d in v])
    if st != XL_OK:
        raise XlError(st, xl_strerror(st))
    return {"copy_gbs": v[0].value, "mfma_f32_tflops": v[1].value, "mfma_bf16_tflops": v[2].value,
            "valu_f32_tflops": v[3].value}


class Plan:
    """Owns an xl_plan handle.  Built from a workload description (layers with
    op / inputs / out / cin / cout / k / stride / pad / groups / relu / bias / bn,
    tensor shapes, fusion groups); weight slots are assigned here:
    slot 3*i = filter, 3*i+1 = scale, 3*i+2 = shift of layer i."""

    def __init__(self, workload, device: int = -1, **options):
        L = lib()
        self.workload = workload
        nl, nt = len(workload.layers), len(workload.shapes)
        layers = (xl_layer * nl)()
        for i, ly in enumerate(workload.layers):
            c = layers[i]
            c.op = OPS[ly.op]
            ins = list(ly.inputs) + [-1, -1]
            c.in_[0], c.in_[1] = ins[0], ins[1]
            c.out = ly.out
            c.cin, c.cout, c.k, c.stride, c.pad, c.groups = ly.cin, ly.cout, ly.k, ly.stride, ly.pad, ly.groups
            c.relu = int(ly.relu)
            c.w_slot = 3 * i if ly.op == "conv" else -1
            c.scale_slot = 3 * i + 1 if (ly.op == "conv" and ly.bn) else -1
            c.shift_slot = 3 * i + 2 if (ly.op == "conv" and (ly.bn or ly.bias)) else -1
        shapes = (xl_shape * nt)(*[xl_shape(*s) for s in workload.shapes])
        ng = len(workload.groups)
        groups = (xl_group * max(ng, 1))()
        self._keep = []
        for gi, g in enumerate(workload.groups):
            ids = (ctypes.c_int * len(g.layers))(*g.layers)
            self._keep.append(ids)
            groups[gi].mode = MODES[g.mode]
            groups[gi].nlayers = len(g.layers)
            groups[gi].layer_ids = ids
        opts = xl_options(**options)
        handle = ctypes.c_void_p()
        st = L.xl_plan_create(layers, nl, shapes, nt, groups, ng, device, ctypes.byref(opts), ctypes.byref(handle))
        if st != XL_OK:
            raise XlError(st, L.xl_plan_last_error(None).decode() or xl_strerror(st))
        self.handle = handle
        self.nweights = 3 * nl
        self.ntensors = nt

    def close(self):
        if getattr(self, "handle", None):
            lib().xl_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != XL_OK:
            raise XlError(st, lib().xl_plan_last_error(self.handle).decode() or xl_strerror(st))

    @property
    def num_groups(self) -> int:
        return lib().xl_plan_num_groups(self.handle)

    def query(self, group: int) -> dict:
        info = xl_group_info()
        self._check(lib().xl_plan_query(self.handle, group, ctypes.byref(info)))
        return info.as_dict()

    def workspace_bytes(self) -> int:
        return int(lib().xl_plan_workspace_bytes(self.handle))

    def num_launches(self, fused: bool) -> int:
        return lib().xl_plan_num_launches(self.handle, int(fused))

    def num_candidates(self, fused: bool, launch: int) -> int:
        return lib().xl_plan_num_candidates(self.handle, int(fused), launch)

    def candidate_info(self, fused: bool, launch: int, candidate: int = -1) -> dict:
        info = xl_launch_info()
        self._check(lib().xl_plan_candidate_info(self.handle, int(fused), launch, candidate, ctypes.byref(info)))
        return info.as_dict()

    def select_candidate(self, fused: bool, launch: int, candidate: int):
        self._check(lib().xl_plan_select_candidate(self.handle, int(fused), launch, candidate))

    def set_block_fused(self, group: int, fused: bool):
        self._check(lib().xl_plan_set_block_fused(self.handle, group, int(fused)))

    def block_is_fused(self, group: int) -> bool:
        return bool(lib().xl_plan_block_is_fused(self.handle, group))

    def prepare(self, weight_ptrs: Sequence[Optional[int]], workspace_ptr: int, stream: int = 0):
        arr = (ctypes.c_void_p * self.nweights)(*[ctypes.c_void_p(p) if p else None for p in weight_ptrs])
        self._check(lib().xl_prepare(self.handle, arr, self.nweights, ctypes.c_void_p(workspace_ptr),
                                     ctypes.c_void_p(stream)))

    def run(self, tensor_ptrs: Dict[int, int], workspace_ptr: int, stream: int = 0, fused: bool = True):
        arr = (ctypes.c_void_p * self.ntensors)()
        for t, p in tensor_ptrs.items():
            arr[t] = p
        self._check(lib().xl_run(self.handle, arr, self.ntensors, ctypes.c_void_p(workspace_ptr),
                                 ctypes.c_void_p(stream), int(fused)))

    def run_static(self, weight_ptrs: Optional[Sequence[Optional[int]]], tensor_ptrs: Dict[int, int], stream: int = 0,
                   fused: bool = True, relayout: bool = True):
        warr = None
        if weight_ptrs is not None:
            warr = (ctypes.c_void_p * self.nweights)(*[ctypes.c_void_p(p) if p else None for p in weight_ptrs])
        arr = (ctypes.c_void_p * self.ntensors)()
        for t, p in tensor_ptrs.items():
            arr[t] = p
        self._check(lib().xl_run_static(self.handle, warr, self.nweights, arr, self.ntensors, ctypes.c_void_p(stream),
                                        int(fused), int(relayout)))

    def profile(self, tensor_ptrs: Dict[int, int], workspace_ptr: int, stream: int = 0, fused: bool = True,
                reps: int = 5) -> List[float]:
        """Average duration of every launch of one mode, in microseconds (synchronises)."""
        arr = (ctypes.c_void_p * self.ntensors)()
        for t, p in tensor_ptrs.items():
            arr[t] = p
        n = self.num_launches(fused)
        out = (ctypes.c_float * max(n, 1))()
        self._check(lib().xl_profile(self.handle, arr, self.ntensors, ctypes.c_void_p(workspace_ptr),
                                     ctypes.c_void_p(stream), int(fused), int(reps), out, n))
        return [out[k] for k in range(n)]

    def tune(self, tensor_ptrs: Dict[int, int], workspace_ptr: int, stream: int = 0, reps: int = 5):
        arr = (ctypes.c_void_p * self.ntensors)()
        for t, p in tensor_ptrs.items():
            arr[t] = p
        self._check(lib().xl_tune(self.handle, arr, self.ntensors, ctypes.c_void_p(workspace_ptr),
                                  ctypes.c_void_p(stream), int(reps)))
