"""Thin ctypes binding of libsdkde.so: argument marshalling only.

Function names and argument order mirror include/sdkde.h.  Tensors must be CUDA(HIP) fp32 and
contiguous; PyTorch supplies device memory and the stream, every arithmetic step runs inside
the library's kernels.  A missing library is an error: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

SDKDE_OK = 0
SDKDE_PREC_FP32 = 0
SDKDE_PREC_FP16X2 = 1
SDKDE_PREC_FP16X2_ALL = 2
SDKDE_PREC_FP16X2_PHI16 = 3
SDKDE_FLAG_MAX_SHIFT = 16
SDKDE_FLAG_SYMMETRIC = 32
SDKDE_FLAG_SAMPLES_PREPARED = 64
SDKDE_MAX_D = 128
(SDKDE_TUNE_SCORE_ROW_TILES, SDKDE_TUNE_SCORE_SPLITS, SDKDE_TUNE_EVAL_ROW_TILES, SDKDE_TUNE_EVAL_SPLITS,
 SDKDE_TUNE_SYM_BLOCK_ROWS, SDKDE_TUNE_SYM_GROUPS, SDKDE_TUNE_SYM_MIN_ITEMS, SDKDE_TUNE_SEPARATE_PREP) = range(8)
SDKDE_ETOOLARGE = 5
SDKDE_STATIC_SCRATCH_BYTES = 64 * 1024 * 1024

_lib = None


class SdkdeError(RuntimeError):
    def __init__(self, call: str, status: int, text: str):
        super().__init__(f"{call} failed: status {status} ({text})")
        self.status = status


def load() -> ctypes.CDLL:
    """Loads the built library, building it first if it is missing or was built from other sources than the
    tree holds now (an edited kernel or header must never be tested against an old binary)."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.build(force=False)
    lib = ctypes.CDLL(path)
    c_fp = ctypes.c_void_p
    i64, i32, u32, f64 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_double
    lib.sdkde_workspace_bytes.argtypes = [i64, i64, i32, u32, ctypes.POINTER(ctypes.c_size_t)]
    lib.sdkde_score.argtypes = [c_fp, i64, c_fp, i64, i32, f64, c_fp, c_fp, ctypes.c_size_t, u32, c_fp]
    lib.sdkde_debias.argtypes = [c_fp, c_fp, i64, i32, f64, c_fp, c_fp]
    lib.sdkde_eval.argtypes = [c_fp, i64, c_fp, i64, i32, f64, c_fp, c_fp, c_fp, ctypes.c_size_t, u32, c_fp]
    lib.sdkde_fit_eval.argtypes = [c_fp, i64, c_fp, i64, i32, f64, c_fp, c_fp, c_fp, c_fp, c_fp, ctypes.c_size_t, u32, c_fp]
    lib.sdkde_fit_eval_static.argtypes = [c_fp, i64, c_fp, i64, i32, f64, c_fp, c_fp, c_fp, c_fp, u32, c_fp]
    lib.sdkde_eval_laplace.argtypes = [c_fp, i64, c_fp, i64, i32, f64, c_fp, c_fp, ctypes.c_size_t, u32, c_fp]
    lib.sdkde_describe_plan.argtypes = [i64, i64, i32, i32, u32, ctypes.POINTER(ctypes.c_int64), i32]
    lib.sdkde_set_tuning.argtypes = [ctypes.c_int, ctypes.c_int]
    lib.sdkde_status_string.argtypes = [ctypes.c_int]
    lib.sdkde_status_string.restype = ctypes.c_char_p
    lib.sdkde_profile_enable.argtypes = [ctypes.c_int]
    lib.sdkde_profile_summary.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float)]
    for name in ("sdkde_workspace_bytes", "sdkde_score", "sdkde_debias", "sdkde_eval", "sdkde_eval_laplace", "sdkde_fit_eval", "sdkde_fit_eval_static", "sdkde_describe_plan",
                 "sdkde_profile_enable", "sdkde_profile_summary", "sdkde_set_tuning"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def sdkde_status_string(status: int) -> str:
    return load().sdkde_status_string(int(status)).decode()


def _check(call: str, status: int) -> None:
    if status != SDKDE_OK:
        raise SdkdeError(call, status, sdkde_status_string(status))


def _dev_f32(t: torch.Tensor, name: str) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.float32 or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous fp32 tensor on the GPU")
    return t


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def sdkde_workspace_bytes(n: int, m: int, d: int, flags: int = SDKDE_PREC_FP32) -> int:
    out = ctypes.c_size_t(0)
    _check("sdkde_workspace_bytes", load().sdkde_workspace_bytes(n, m, d, flags, ctypes.byref(out)))
    return int(out.value)


PLAN_FIELDS = ("thin", "dp", "row_tiles", "rows_per_block", "row_blocks", "splits", "tiles_per_split", "tiles",
               "n_pad", "m_pad", "workspace_bytes", "off_xs", "off_xt", "off_xn", "off_ps", "off_pn", "off_part_t",
               "off_part_d", "partial_slots", "xt_scale", "symmetric", "sym_block_rows", "sym_blocks_per_group",
               "sym_groups", "last_block_mfmas", "fit_eval_fused_prep")


def sdkde_describe_plan(n: int, m: int, d: int, call: int, flags: int = SDKDE_PREC_FP32) -> dict:
    """Grid decomposition and workspace layout for call 0 (score at samples), 1 (score at points) or 2 (eval)."""
    out = (ctypes.c_int64 * len(PLAN_FIELDS))()
    _check("sdkde_describe_plan", load().sdkde_describe_plan(n, m, d, call, flags, out, len(PLAN_FIELDS)))
    return dict(zip(PLAN_FIELDS, (int(v) for v in out)))


def workspace_bytes_any_precision(n: int, m: int, d: int, flags: int = SDKDE_PREC_FP32) -> int:
    """The largest of sdkde_workspace_bytes over the precision modes, with and without the max-shifted
    sums, the other flags as given: the grid decomposition (and with it the number of partial-sum slots) depends
    on the precision mode, and the mode a score at separate points runs in depends on the shift."""
    other = flags & ~(15 | SDKDE_FLAG_MAX_SHIFT)
    return max(sdkde_workspace_bytes(n, m, d, other | prec | shift)
               for prec in (SDKDE_PREC_FP32, SDKDE_PREC_FP16X2, SDKDE_PREC_FP16X2_ALL, SDKDE_PREC_FP16X2_PHI16)
               for shift in (0, SDKDE_FLAG_MAX_SHIFT))


def make_workspace(n: int, m: int, d: int, device="cuda", flags: int = SDKDE_PREC_FP32) -> torch.Tensor:
    """A device byte buffer large enough for every call at these sizes in every precision mode, with or without
    SDKDE_FLAG_MAX_SHIFT (the symmetric score needs its flag here; a buffer made with it also serves calls
    without it)."""
    need = max(workspace_bytes_any_precision(n, m, d, flags), workspace_bytes_any_precision(n, m, d, flags & ~SDKDE_FLAG_SYMMETRIC))
    return torch.empty(need, dtype=torch.uint8, device=device)


def _workspace(ws, n, m, d, device, flags=SDKDE_PREC_FP32, stream=None):
    if ws is None:
        if flags & SDKDE_FLAG_SAMPLES_PREPARED:
            raise ValueError("SDKDE_FLAG_SAMPLES_PREPARED needs the workspace of the call that prepared the samples")
        # A temporary workspace is freed when the wrapper returns, while the kernels that use it are still queued
        # on `stream`: allocate it on that stream, so that the caching allocator hands the block out again only to
        # work ordered after them.
        if stream is not None and stream != torch.cuda.current_stream():
            with torch.cuda.stream(stream):
                ws = make_workspace(n, m, d, device, flags)
        else:
            ws = make_workspace(n, m, d, device, flags)
    if not ws.is_cuda or ws.dtype != torch.uint8 or not ws.is_contiguous():
        raise TypeError("workspace must be a contiguous uint8 tensor on the GPU")
    return ws


def sdkde_score(samples, h, points=None, out=None, workspace=None, flags=SDKDE_PREC_FP32, stream=None):
    """score_out[m,d]: empirical KDE score at `points` (None: at the samples)."""
    x = _dev_f32(samples, "samples")
    n, d = x.shape
    if points is None:
        m, p_ptr = n, None
    else:
        p = _dev_f32(points, "points")
        if p.dim() != 2 or p.shape[1] != d:
            raise ValueError("points must be [m, d]")
        m, p_ptr = p.shape[0], p.data_ptr()
    if out is None:
        out = torch.empty((m, d), dtype=torch.float32, device=x.device)
    _dev_f32(out, "out")
    if tuple(out.shape) != (m, d):
        raise ValueError("out must be [m, d]")
    ws = _workspace(workspace, n, m, d, x.device, flags, stream)
    _check("sdkde_score", load().sdkde_score(x.data_ptr(), n, p_ptr, m, d, float(h), out.data_ptr(),
                                             ws.data_ptr(), ws.numel(), flags, _stream_handle(stream)))
    return out


def sdkde_debias(samples, score, h, out=None, stream=None):
    """samples + (h^2/2) score, elementwise."""
    x, s = _dev_f32(samples, "samples"), _dev_f32(score, "score")
    if x.shape != s.shape:
        raise ValueError("samples and score differ in shape")
    n, d = x.shape
    if out is None:
        out = torch.empty_like(x)
    _dev_f32(out, "out")
    if out.shape != x.shape:
        raise ValueError("out must have the shape of samples")
    _check("sdkde_debias", load().sdkde_debias(x.data_ptr(), s.data_ptr(), n, d, float(h), out.data_ptr(),
                                               _stream_handle(stream)))
    return out


def sdkde_eval(samples_sd, queries, h, density_out=None, log_density_out=None, want="density",
               workspace=None, flags=SDKDE_PREC_FP32, stream=None):
    """KDE of samples_sd at the queries.  want: "density", "log" or "both" selects which outputs
    are allocated when none is passed in.  Returns (density, log_density), None for the absent one."""
    x, q = _dev_f32(samples_sd, "samples_sd"), _dev_f32(queries, "queries")
    n, d = x.shape
    if q.dim() != 2 or q.shape[1] != d:
        raise ValueError("queries must be [m, d]")
    m = q.shape[0]
    if density_out is None and log_density_out is None:
        if want in ("density", "both"):
            density_out = torch.empty(m, dtype=torch.float32, device=x.device)
        if want in ("log", "both"):
            log_density_out = torch.empty(m, dtype=torch.float32, device=x.device)
    for t, name in ((density_out, "density_out"), (log_density_out, "log_density_out")):
        if t is not None:
            _dev_f32(t, name)
            if t.numel() != m:
                raise ValueError(f"{name} must have m elements")
    ws = _workspace(workspace, n, m, d, x.device, flags, stream)
    _check("sdkde_eval", load().sdkde_eval(
        x.data_ptr(), n, q.data_ptr(), m, d, float(h),
        None if density_out is None else density_out.data_ptr(),
        None if log_density_out is None else log_density_out.data_ptr(),
        ws.data_ptr(), ws.numel(), flags, _stream_handle(stream)))
    return density_out, log_density_out


def sdkde_fit_eval(samples, queries, h, score_out=None, samples_sd_out=None, density_out=None, log_density_out=None,
                   want="density", workspace=None, flags=SDKDE_PREC_FP32, stream=None):
    """Score at the samples, shift and KDE at the queries in one call.
    Returns (samples_sd, density, log_density); score_out is filled if given."""
    x, q = _dev_f32(samples, "samples"), _dev_f32(queries, "queries")
    n, d = x.shape
    if q.dim() != 2 or q.shape[1] != d:
        raise ValueError("queries must be [m, d]")
    m = q.shape[0]
    if samples_sd_out is None:
        samples_sd_out = torch.empty_like(x)
    if density_out is None and log_density_out is None:
        if want in ("density", "both"):
            density_out = torch.empty(m, dtype=torch.float32, device=x.device)
        if want in ("log", "both"):
            log_density_out = torch.empty(m, dtype=torch.float32, device=x.device)
    for t, name, shape in ((score_out, "score_out", x.shape), (samples_sd_out, "samples_sd_out", x.shape),
                           (density_out, "density_out", (m,)), (log_density_out, "log_density_out", (m,))):
        if t is not None:
            _dev_f32(t, name)
            if tuple(t.shape) != tuple(shape):
                raise ValueError(f"{name} has the wrong shape")
    ws = _workspace(workspace, n, m, d, x.device, flags, stream)
    ptr = lambda t: None if t is None else t.data_ptr()
    _check("sdkde_fit_eval", load().sdkde_fit_eval(
        x.data_ptr(), n, q.data_ptr(), m, d, float(h), ptr(score_out), samples_sd_out.data_ptr(), ptr(density_out),
        ptr(log_density_out), ws.data_ptr(), ws.numel(), flags, _stream_handle(stream)))
    return samples_sd_out, density_out, log_density_out


def sdkde_fit_eval_static(samples, queries, h, samples_sd_out, score_out=None, density_out=None, log_density_out=None,
                          flags=SDKDE_PREC_FP32, stream=None):
    """sdkde_fit_eval on the library's built-in scratch buffer: no workspace, and nothing is allocated here
    either, so every output the caller wants is passed in (samples_sd_out is required)."""
    x, q = _dev_f32(samples, "samples"), _dev_f32(queries, "queries")
    n, d = x.shape
    if q.dim() != 2 or q.shape[1] != d:
        raise ValueError("queries must be [m, d]")
    m = q.shape[0]
    for t, name, shape in ((score_out, "score_out", x.shape), (samples_sd_out, "samples_sd_out", x.shape),
                           (density_out, "density_out", (m,)), (log_density_out, "log_density_out", (m,))):
        if t is not None:
            _dev_f32(t, name)
            if tuple(t.shape) != tuple(shape):
                raise ValueError(f"{name} has the wrong shape")
    ptr = lambda t: None if t is None else t.data_ptr()
    _check("sdkde_fit_eval_static", load().sdkde_fit_eval_static(
        x.data_ptr(), n, q.data_ptr(), m, d, float(h), ptr(score_out), ptr(samples_sd_out), ptr(density_out),
        ptr(log_density_out), flags, _stream_handle(stream)))
    return samples_sd_out, density_out, log_density_out


def sdkde_eval_laplace(samples, queries, h, density_out=None, workspace=None, flags=SDKDE_PREC_FP32, stream=None):
    """Laplace-corrected KDE of the (unshifted) samples at the queries; signed density [m]."""
    x, q = _dev_f32(samples, "samples"), _dev_f32(queries, "queries")
    n, d = x.shape
    if q.dim() != 2 or q.shape[1] != d:
        raise ValueError("queries must be [m, d]")
    m = q.shape[0]
    if density_out is None:
        density_out = torch.empty(m, dtype=torch.float32, device=x.device)
    _dev_f32(density_out, "density_out")
    if density_out.numel() != m:
        raise ValueError("density_out must have m elements")
    ws = _workspace(workspace, n, m, d, x.device, flags, stream)
    _check("sdkde_eval_laplace", load().sdkde_eval_laplace(
        x.data_ptr(), n, q.data_ptr(), m, d, float(h), density_out.data_ptr(), ws.data_ptr(), ws.numel(), flags,
        _stream_handle(stream)))
    return density_out


def sdkde_set_tuning(knob: int, value: int) -> None:
    """Test / sweep hook: overrides one choice of the host-side plan (0 restores the library's own)."""
    _check("sdkde_set_tuning", load().sdkde_set_tuning(int(knob), int(value)))


def sdkde_profile_enable(on: bool) -> None:
    _check("sdkde_profile_enable", load().sdkde_profile_enable(1 if on else 0))


def sdkde_profile_summary(which: int):
    """(launches, total_ms) of the main pair kernel for which = 0 (score) or 1 (eval)."""
    count, total = ctypes.c_int(0), ctypes.c_float(0.0)
    _check("sdkde_profile_summary", load().sdkde_profile_summary(which, ctypes.byref(count), ctypes.byref(total)))
    return int(count.value), float(total.value)
