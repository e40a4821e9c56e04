"""ctypes binding of libdgc: argument marshalling only.

The function names mirror the C ABI declared in include/dgc.h.  torch is used
for device memory and streams; every step of the path runs in the library's
HIP kernels.  There is no fallback: if libdgc.so has not been built, `load()`
raises.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import List, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
# DGC_LIBRARY selects another build of the library (e.g. one compiled with different tile constants).
LIB_PATH = os.environ.get("DGC_LIBRARY") or os.path.join(HERE, "libdgc.so")

DGC_OK = 0
DGC_ERR_INVALID_ARG = -1
DGC_ERR_ALIGNMENT = -2
DGC_ERR_CAPACITY = -3
DGC_ERR_HIP = -4
DGC_ERR_STATE = -5

DGC_FLAG_NESTEROV = 1 << 0
DGC_FLAG_NO_FACTOR_MASKING = 1 << 1
DGC_FLAG_EXACT_SELECT = 1 << 2
DGC_FLAG_DETERMINISTIC_ACCUMULATE = 1 << 3
DGC_FLAG_SORTED_OUTPUT = 1 << 4

DGC_DIAG_OVERFLOW = 1 << 0
DGC_DIAG_NONFINITE = 1 << 1
DGC_DIAG_BAD_INDEX = 1 << 2
DGC_DIAG_UNSORTED = 1 << 3

EXPORTS = [
    "dgc_config_default", "dgc_status_string", "dgc_create", "dgc_destroy", "dgc_invalidate_workspace",
    "dgc_set_scale_override", "dgc_set_density",
    "dgc_set_warmup_schedule", "dgc_set_warmup_stage_length", "dgc_set_iteration_density", "dgc_query_plan", "dgc_workspace_bytes", "dgc_workspace_bytes_warmup",
    "dgc_recommended_payload_layout", "dgc_compress", "dgc_compress_static", "dgc_get_diagnostics",
    "dgc_decompress_accumulate", "dgc_decompress_accumulate_regions", "dgc_decompress_replace_regions",
    "dgc_dense_clear_regions",
    "dgc_version", "dgc_last_error_string", "dgc_profile_enable", "dgc_profile_collect",
    "dgc_profile_disable", "dgc_sparse_sgd_apply", "dgc_sparse_sgd_apply_regions",
    "dgc_encode_max_entries", "dgc_encode", "dgc_decode_accumulate", "dgc_profile_stream_ceiling",
]


class DgcConfig(C.Structure):
    _fields_ = [
        ("momentum", C.c_float),
        ("clip_threshold", C.c_float),
        ("num_workers", C.c_int32),
        ("flags", C.c_uint32),
        ("density", C.c_double),
        ("sample_ratio", C.c_double),
        ("sample_min", C.c_int32),
        ("sample_max", C.c_int32),
        ("sample_block", C.c_int32),
        ("scale_override", C.c_float),
        ("seed", C.c_uint64),
        ("refine_alpha", C.c_float),
        ("reserved", C.c_uint32),
    ]


class DgcDiagnostics(C.Structure):
    _fields_ = [("norm", C.c_double), ("scale", C.c_float), ("flags", C.c_uint32)]


class DgcError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status}")
        self.status = status


_lib = None


def load() -> C.CDLL:
    """Open libdgc.so and declare its prototypes.  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_1712_01887_amd.build`")
    # torch ships its own HIP runtime under the same soname.  Importing torch first makes
    # libdgc bind to that copy, so the tensors' device context and the kernels share one runtime.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u64, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_double
    P = C.POINTER
    lib.dgc_version.restype = i32
    lib.dgc_version.argtypes = []
    lib.dgc_status_string.restype = C.c_char_p
    lib.dgc_status_string.argtypes = [i32]
    lib.dgc_last_error_string.restype = C.c_char_p
    lib.dgc_last_error_string.argtypes = []
    lib.dgc_config_default.restype = i32
    lib.dgc_config_default.argtypes = [P(DgcConfig)]
    lib.dgc_create.restype = i32
    lib.dgc_create.argtypes = [P(vp), P(DgcConfig), i32, P(i64)]
    lib.dgc_destroy.restype = i32
    lib.dgc_destroy.argtypes = [vp]
    lib.dgc_invalidate_workspace.restype = i32
    lib.dgc_invalidate_workspace.argtypes = [vp]
    lib.dgc_set_scale_override.restype = i32
    lib.dgc_set_scale_override.argtypes = [vp, C.c_float]
    lib.dgc_set_density.restype = i32
    lib.dgc_set_density.argtypes = [vp, dbl]
    lib.dgc_set_warmup_schedule.restype = i32
    lib.dgc_set_warmup_schedule.argtypes = [vp, P(dbl), i32]
    lib.dgc_set_warmup_stage_length.restype = i32
    lib.dgc_set_warmup_stage_length.argtypes = [vp, i64]
    lib.dgc_set_iteration_density.restype = i32
    lib.dgc_set_iteration_density.argtypes = [vp, i64]
    lib.dgc_query_plan.restype = i32
    lib.dgc_query_plan.argtypes = [vp, i32, P(i64), P(i64), P(i64), P(i64)]
    lib.dgc_workspace_bytes.restype = i32
    lib.dgc_workspace_bytes.argtypes = [vp, P(C.c_size_t)]
    lib.dgc_workspace_bytes_warmup.restype = i32
    lib.dgc_workspace_bytes_warmup.argtypes = [vp, P(C.c_size_t)]
    lib.dgc_recommended_payload_layout.restype = i32
    lib.dgc_recommended_payload_layout.argtypes = [vp, dbl, P(i64)]
    lib.dgc_compress.restype = i32
    lib.dgc_compress.argtypes = [vp, vp, vp, vp, vp, vp, P(i64), vp, vp, u64, vp, C.c_size_t, vp]
    lib.dgc_compress_static.restype = i32
    lib.dgc_compress_static.argtypes = [vp, vp, vp, vp, vp, vp, P(i64), vp, vp, u64, vp]
    lib.dgc_get_diagnostics.restype = i32
    lib.dgc_get_diagnostics.argtypes = [vp, vp, P(DgcDiagnostics), vp]
    lib.dgc_decompress_accumulate.restype = i32
    lib.dgc_decompress_accumulate.argtypes = [vp, vp, i64, i32, P(vp), P(vp), P(i64), vp, vp]
    lib.dgc_decompress_accumulate_regions.restype = i32
    lib.dgc_decompress_accumulate_regions.argtypes = [vp, vp, i32, P(vp), P(vp), P(vp), P(i64), vp,
                                                      C.c_size_t, vp]
    lib.dgc_decompress_replace_regions.restype = i32
    lib.dgc_decompress_replace_regions.argtypes = [vp, vp, i32, P(vp), P(vp), P(vp), i32, P(vp), P(vp), P(i64), vp,
                                                   C.c_size_t, vp]
    lib.dgc_dense_clear_regions.restype = i32
    lib.dgc_dense_clear_regions.argtypes = [vp, vp, i32, P(vp), P(vp), P(i64), vp, C.c_size_t, vp]
    lib.dgc_sparse_sgd_apply.restype = i32
    lib.dgc_sparse_sgd_apply.argtypes = [vp, vp, i64, C.c_float, i32, P(vp), P(vp), P(i64), vp, vp]
    lib.dgc_sparse_sgd_apply_regions.restype = i32
    lib.dgc_sparse_sgd_apply_regions.argtypes = [vp, vp, C.c_float, i32, P(vp), P(vp), P(vp), P(i64), vp,
                                                 C.c_size_t, vp]
    lib.dgc_encode_max_entries.restype = i32
    lib.dgc_encode_max_entries.argtypes = [vp, i64, P(i64)]
    lib.dgc_encode.restype = i32
    lib.dgc_encode.argtypes = [vp, vp, vp, vp, P(i64), vp, vp, i64, vp, vp, C.c_size_t, vp]
    lib.dgc_decode_accumulate.restype = i32
    lib.dgc_decode_accumulate.argtypes = [vp, vp, i64, i32, P(vp), P(vp), P(i64), vp, vp, C.c_size_t, vp]
    lib.dgc_profile_stream_ceiling.restype = i32
    lib.dgc_profile_stream_ceiling.argtypes = [vp, vp, vp, i64, i32, vp]
    lib.dgc_profile_enable.restype = i32
    lib.dgc_profile_enable.argtypes = [vp, i32]
    lib.dgc_profile_collect.restype = i32
    lib.dgc_profile_collect.argtypes = [vp, P(i32), P(dbl), P(dbl), P(dbl), P(dbl)]
    lib.dgc_profile_disable.restype = i32
    lib.dgc_profile_disable.argtypes = [vp]
    _lib = lib
    return lib


def _check(status: int, what: str) -> None:
    if status != DGC_OK:
        detail = load().dgc_last_error_string().decode() if status == DGC_ERR_HIP else ""
        raise DgcError(status, f"{what}: {load().dgc_status_string(status).decode()} {detail}".rstrip())


def dgc_config_default() -> DgcConfig:
    cfg = DgcConfig()
    _check(load().dgc_config_default(C.byref(cfg)), "dgc_config_default")
    return cfg


def make_config(**kw) -> DgcConfig:
    cfg = dgc_config_default()
    for k, v in kw.items():
        if not hasattr(cfg, k):
            raise AttributeError(k)
        setattr(cfg, k, v)
    return cfg


def _i64_array(values: Sequence[int]):
    arr = (C.c_int64 * len(values))(*[int(x) for x in values])
    return arr


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


def _stream() -> int:
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


def _ptr_array(tensors) -> "C.Array":
    return (C.c_void_p * len(tensors))(*[_ptr(t) for t in tensors])


def dgc_profile_stream_ceiling(a, b, c, groups_per_cu: int = 0) -> None:
    """One launch of the bare three-read / two-write kernel over a, b, c (same length)."""
    _check(load().dgc_profile_stream_ceiling(_ptr(a), _ptr(b), _ptr(c), int(a.numel()), int(groups_per_cu),
                                             _stream()),
           "dgc_profile_stream_ceiling")


class Dgc:
    """One gradient set on one worker: the handle of the C ABI plus its workspace."""

    def __init__(self, cfg: DgcConfig, offsets: Sequence[int], warmup_workspace: bool = False):
        self.lib = load()
        self.cfg = cfg
        # allocate the workspace with the staging arrays that speed up compress above 0.5 % density
        self.warmup_workspace = bool(warmup_workspace)
        self.offsets = [int(x) for x in offsets]
        self.num_tensors = len(self.offsets) - 1
        self.n = self.offsets[-1]
        self._h = C.c_void_p()
        _check(self.lib.dgc_create(C.byref(self._h), C.byref(cfg), self.num_tensors,
                                   _i64_array(self.offsets)), "dgc_create")
        self.workspace = None
        self._layout = None
        self._layout_c = None

    def close(self) -> None:
        if self._h:
            self.lib.dgc_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- host-only calls ---------------------------------------------------
    def dgc_invalidate_workspace(self) -> None:
        _check(self.lib.dgc_invalidate_workspace(self._h), "dgc_invalidate_workspace")

    def dgc_set_scale_override(self, scale: float) -> None:
        _check(self.lib.dgc_set_scale_override(self._h, float(scale)), "dgc_set_scale_override")

    def dgc_set_density(self, density: float) -> None:
        _check(self.lib.dgc_set_density(self._h, float(density)), "dgc_set_density")

    def dgc_set_warmup_schedule(self, densities: Sequence[float]) -> None:
        arr = (C.c_double * len(densities))(*[float(d) for d in densities])
        _check(self.lib.dgc_set_warmup_schedule(self._h, arr, len(densities)), "dgc_set_warmup_schedule")

    def dgc_set_warmup_stage_length(self, iterations_per_stage: int) -> None:
        _check(self.lib.dgc_set_warmup_stage_length(self._h, int(iterations_per_stage)),
               "dgc_set_warmup_stage_length")

    def dgc_set_iteration_density(self, iteration: int) -> None:
        _check(self.lib.dgc_set_iteration_density(self._h, int(iteration)), "dgc_set_iteration_density")

    def dgc_query_plan(self, j: int):
        k, s, r, d = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
        _check(self.lib.dgc_query_plan(self._h, int(j), C.byref(k), C.byref(s), C.byref(r), C.byref(d)),
               "dgc_query_plan")
        return k.value, s.value, r.value, d.value

    def dgc_workspace_bytes(self) -> int:
        b = C.c_size_t()
        _check(self.lib.dgc_workspace_bytes(self._h, C.byref(b)), "dgc_workspace_bytes")
        return int(b.value)

    def dgc_workspace_bytes_warmup(self) -> int:
        b = C.c_size_t()
        _check(self.lib.dgc_workspace_bytes_warmup(self._h, C.byref(b)), "dgc_workspace_bytes_warmup")
        return int(b.value)

    def dgc_recommended_payload_layout(self, density: float) -> List[int]:
        arr = (C.c_int64 * (self.num_tensors + 1))()
        _check(self.lib.dgc_recommended_payload_layout(self._h, float(density), arr),
               "dgc_recommended_payload_layout")
        return list(arr)

    # -- device memory (torch is the allocator) -----------------------------------
    def set_layout(self, out_offsets: Sequence[int]) -> None:
        self._layout = [int(x) for x in out_offsets]
        self._layout_c = _i64_array(self._layout)

    def ensure_workspace(self, device="cuda"):
        import torch
        if self.workspace is None:
            nbytes = self.dgc_workspace_bytes_warmup() if self.warmup_workspace else self.dgc_workspace_bytes()
            self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
            base = self.workspace.data_ptr()
            self._ws_ptr = (base + 255) // 256 * 256
            self._ws_bytes = nbytes
        return self.workspace

    def alloc_payload(self, device="cuda"):
        """(out_idx, out_val, out_counts, out_thr) sized for the current layout."""
        import torch
        total = max(1, self._layout[-1])
        return (torch.empty(total, dtype=torch.int32, device=device),
                torch.empty(total, dtype=torch.float32, device=device),
                torch.zeros(self.num_tensors, dtype=torch.int32, device=device),
                torch.empty(self.num_tensors, dtype=torch.float32, device=device))

    # -- the hot path --------------------------------------------------------------
    def dgc_compress(self, g, u, v, out_idx, out_val, out_counts, out_thr, iteration: int) -> None:
        self.ensure_workspace(g.device)
        _check(self.lib.dgc_compress(self._h, _ptr(g), _ptr(u), _ptr(v), _ptr(out_idx), _ptr(out_val),
                                     self._layout_c, _ptr(out_counts), _ptr(out_thr), int(iteration),
                                     self._ws_ptr, self._ws_bytes, _stream()), "dgc_compress")

    def dgc_compress_static(self, g, u, v, out_idx, out_val, out_counts, out_thr, iteration: int) -> None:
        """dgc_compress on the library's static scratch array: no workspace, nothing allocated."""
        _check(self.lib.dgc_compress_static(self._h, _ptr(g), _ptr(u), _ptr(v), _ptr(out_idx), _ptr(out_val),
                                            self._layout_c, _ptr(out_counts), _ptr(out_thr), int(iteration),
                                            _stream()), "dgc_compress_static")

    def dgc_get_diagnostics(self, static: bool = False) -> DgcDiagnostics:
        d = DgcDiagnostics()
        _check(self.lib.dgc_get_diagnostics(self._h, None if static else self._ws_ptr, C.byref(d), _stream()),
               "dgc_get_diagnostics")
        return d

    def dgc_profile_enable(self, max_calls: int) -> None:
        _check(self.lib.dgc_profile_enable(self._h, int(max_calls)), "dgc_profile_enable")

    def dgc_profile_collect(self):
        """(calls, norm_ms, select_ms, stream_ms, emit_ms) summed over the recorded calls."""
        calls, a, b, c, d = C.c_int32(), C.c_double(), C.c_double(), C.c_double(), C.c_double()
        _check(self.lib.dgc_profile_collect(self._h, C.byref(calls), C.byref(a), C.byref(b), C.byref(c),
                                            C.byref(d)), "dgc_profile_collect")
        return calls.value, a.value, b.value, c.value, d.value

    def dgc_profile_disable(self) -> None:
        _check(self.lib.dgc_profile_disable(self._h), "dgc_profile_disable")

    def dgc_decompress_accumulate(self, dense, idx_list, val_list, counts: Sequence[int],
                                  diag_flags=None) -> None:
        n = len(idx_list)
        _check(self.lib.dgc_decompress_accumulate(self._h, _ptr(dense), int(dense.numel()), n,
                                                  _ptr_array(idx_list), _ptr_array(val_list),
                                                  _i64_array(counts), _ptr(diag_flags), _stream()),
               "dgc_decompress_accumulate")

    def dgc_decompress_accumulate_regions(self, dense, idx_list, val_list, count_list) -> None:
        self.ensure_workspace(dense.device)
        _check(self.lib.dgc_decompress_accumulate_regions(
            self._h, _ptr(dense), len(idx_list), _ptr_array(idx_list), _ptr_array(val_list),
            _ptr_array(count_list), self._layout_c, self._ws_ptr, self._ws_bytes, _stream()),
            "dgc_decompress_accumulate_regions")

    def dgc_decompress_replace_regions(self, dense, idx_list, val_list, count_list, previous_idx_list=(),
                                       previous_count_list=()) -> None:
        self.ensure_workspace(dense.device)
        m = len(previous_idx_list)
        _check(self.lib.dgc_decompress_replace_regions(
            self._h, _ptr(dense), len(idx_list), _ptr_array(idx_list), _ptr_array(val_list), _ptr_array(count_list),
            m, _ptr_array(previous_idx_list) if m else None, _ptr_array(previous_count_list) if m else None,
            self._layout_c, self._ws_ptr, self._ws_bytes, _stream()), "dgc_decompress_replace_regions")

    def dgc_sparse_sgd_apply(self, theta, learning_rate: float, idx_list, val_list, counts: Sequence[int],
                             diag_flags=None) -> None:
        _check(self.lib.dgc_sparse_sgd_apply(self._h, _ptr(theta), int(theta.numel()), float(learning_rate),
                                             len(idx_list), _ptr_array(idx_list), _ptr_array(val_list),
                                             _i64_array(counts), _ptr(diag_flags), _stream()),
               "dgc_sparse_sgd_apply")

    def dgc_sparse_sgd_apply_regions(self, theta, learning_rate: float, idx_list, val_list, count_list) -> None:
        self.ensure_workspace(theta.device)
        _check(self.lib.dgc_sparse_sgd_apply_regions(
            self._h, _ptr(theta), float(learning_rate), len(idx_list), _ptr_array(idx_list),
            _ptr_array(val_list), _ptr_array(count_list), self._layout_c, self._ws_ptr, self._ws_bytes,
            _stream()), "dgc_sparse_sgd_apply_regions")

    # -- wire format ---------------------------------------------------------------
    def dgc_encode_max_entries(self, pairs: int) -> int:
        e = C.c_int64()
        _check(self.lib.dgc_encode_max_entries(self._h, int(pairs), C.byref(e)), "dgc_encode_max_entries")
        return int(e.value)

    def dgc_encode(self, out_idx, out_val, out_counts, runs, vals, num_entries) -> None:
        """runs: int16/uint16 tensor, vals: float32 tensor of the same length, num_entries: int32[1]."""
        self.ensure_workspace(out_idx.device)
        _check(self.lib.dgc_encode(self._h, _ptr(out_idx), _ptr(out_val), _ptr(out_counts), self._layout_c,
                                   _ptr(runs), _ptr(vals), int(min(runs.numel(), vals.numel())),
                                   _ptr(num_entries), self._ws_ptr, self._ws_bytes, _stream()), "dgc_encode")

    def dgc_decode_accumulate(self, dense, runs_list, vals_list, counts: Sequence[int], diag_flags=None) -> None:
        self.ensure_workspace(dense.device)
        _check(self.lib.dgc_decode_accumulate(self._h, _ptr(dense), int(dense.numel()), len(runs_list),
                                              _ptr_array(runs_list), _ptr_array(vals_list), _i64_array(counts),
                                              _ptr(diag_flags), self._ws_ptr, self._ws_bytes, _stream()),
               "dgc_decode_accumulate")

    def dgc_dense_clear_regions(self, dense, idx_list, count_list) -> None:
        self.ensure_workspace(dense.device)
        _check(self.lib.dgc_dense_clear_regions(
            self._h, _ptr(dense), len(idx_list), _ptr_array(idx_list), _ptr_array(count_list),
            self._layout_c, self._ws_ptr, self._ws_bytes, _stream()), "dgc_dense_clear_regions")
