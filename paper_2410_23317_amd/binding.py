"""Thin ctypes binding over libvlcache.so: argument marshalling only.

Every function has the name and argument order of its C-ABI entry point (include/vlcache.h).
Tensors are torch CUDA tensors (PyTorch is used for device memory and streams only); their
data_ptr() is handed to the library together with torch's current stream.  Nothing here
computes: if the shared library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvlcache.so")

VLC_OK, VLC_ERR_INVALID_ARG, VLC_ERR_SHAPE, VLC_ERR_DTYPE, VLC_ERR_CAPACITY, VLC_ERR_HIP, VLC_ERR_UNIMPLEMENTED = range(7)
VLC_F32, VLC_BF16 = 0, 1
STATUS_NAMES = ["VLC_OK", "VLC_ERR_INVALID_ARG", "VLC_ERR_SHAPE", "VLC_ERR_DTYPE", "VLC_ERR_CAPACITY",
                "VLC_ERR_HIP", "VLC_ERR_UNIMPLEMENTED"]


class VlcError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {message}")
        self.status = status


class vlc_shape(C.Structure):
    _fields_ = ([(n, C.c_int32) for n in ("B", "L", "Hq", "Hkv", "d", "m", "tau", "dtype")] + [("lens", C.c_void_p)] +
                [("flags", C.c_int32), ("reserved", C.c_int32)])


class vlc_cache_layout(C.Structure):
    _fields_ = [("status_off", C.c_size_t), ("slot_off_off", C.c_size_t), ("kept_off", C.c_size_t),
                ("kv_off", C.c_size_t), ("idx_off", C.c_size_t), ("scratch_off", C.c_size_t),
                ("total_bytes", C.c_size_t), ("slots_per_request", C.c_int64), ("scale_off", C.c_size_t),
                ("kv_fp8", C.c_int32), ("unit_slots", C.c_int32), ("tail_unit_slots", C.c_int32),
                ("layer_unit_slots", C.c_int32), ("appended_off", C.c_size_t),
                ("list_items_off", C.c_size_t * 3), ("list_index_off", C.c_size_t * 3),
                ("list_by_size", C.c_int32 * 3), ("list_reserved", C.c_int32)]


class vlc_cache_options(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kv_fp8", "unit_slots", "tail_unit_slots", "layer_unit_slots", "decode_order",
                                         "decode_merge", "decode_zigzag", "gather_rows", "select_fold")] + \
               [("reserved", C.c_int32 * 7)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, sz, i32, i64, f32 = C.c_void_p, C.c_size_t, C.c_int32, C.c_int64, C.c_float
    shp = C.POINTER(vlc_shape)
    lib.vlc_last_error_string.restype = C.c_char_p
    lib.vlc_version.restype = C.c_char_p
    lib.vlc_workspace_bytes.restype = sz
    lib.vlc_workspace_bytes.argtypes = [shp]
    lib.vlc_score.restype = C.c_int
    lib.vlc_score.argtypes = [shp, vp, vp, vp, f32, vp, vp, vp, vp, vp, sz, vp]
    lib.vlc_score_static_max_workspace.restype = sz
    lib.vlc_score_static_max_workspace.argtypes = []
    lib.vlc_score_static.restype = C.c_int
    lib.vlc_score_static.argtypes = [shp, vp, vp, vp, f32, vp, vp, vp, vp, vp]
    lib.vlc_sparsity.restype = C.c_int
    lib.vlc_sparsity.argtypes = [shp, vp, vp, vp, vp, f32, vp, vp, vp, sz, vp]
    lib.vlc_window_attn_workspace_bytes.restype = C.c_int
    lib.vlc_window_attn_workspace_bytes.argtypes = [shp, C.POINTER(sz)]
    lib.vlc_window_attn.restype = C.c_int
    lib.vlc_window_attn.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.vlc_score_from_stats.restype = C.c_int
    lib.vlc_score_from_stats.argtypes = [shp, vp, vp, vp, f32, vp, vp, vp, vp, vp]
    lib.vlc_allocate.restype = C.c_int
    lib.vlc_allocate.argtypes = [shp, vp, i64, i64, vp, vp, vp]
    lib.vlc_cache_bytes.restype = sz
    lib.vlc_cache_bytes.argtypes = [shp, i32, i64]
    lib.vlc_cache_create.restype = C.c_int
    lib.vlc_cache_create.argtypes = [shp, i32, i64, vp, sz, C.POINTER(vp)]
    lib.vlc_cache_bytes_fp8.restype = sz
    lib.vlc_cache_bytes_fp8.argtypes = [shp, i32, i64]
    lib.vlc_cache_create_fp8.restype = C.c_int
    lib.vlc_cache_create_fp8.argtypes = [shp, i32, i64, vp, sz, C.POINTER(vp)]
    lib.vlc_cache_bytes_opt.restype = sz
    lib.vlc_cache_bytes_opt.argtypes = [shp, i32, i64, C.POINTER(vlc_cache_options)]
    lib.vlc_cache_create_opt.restype = C.c_int
    lib.vlc_cache_create_opt.argtypes = [shp, i32, i64, C.POINTER(vlc_cache_options), vp, sz, C.POINTER(vp)]
    lib.vlc_cache_destroy.restype = None
    lib.vlc_cache_destroy.argtypes = [vp]
    lib.vlc_cache_get_layout.restype = C.c_int
    lib.vlc_cache_get_layout.argtypes = [vp, C.POINTER(vlc_cache_layout)]
    lib.vlc_cache_status.restype = C.c_int
    lib.vlc_cache_status.argtypes = [vp, vp]
    lib.vlc_topk_compact.restype = C.c_int
    lib.vlc_topk_compact.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp]
    lib.vlc_topk_compact_recent_frac.restype = C.c_int
    lib.vlc_topk_compact_recent_frac.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.vlc_cache_hit_rate.restype = C.c_int
    lib.vlc_cache_hit_rate.argtypes = [vp, vp, vp, vp, vp]
    lib.vlc_decode_attn.restype = C.c_int
    lib.vlc_decode_attn.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.vlc_decode_attn_steps.restype = C.c_int
    lib.vlc_decode_attn_steps.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.vlc_probe_read_stream.restype = C.c_int
    lib.vlc_probe_read_stream.argtypes = [vp, sz, vp, i32, vp]
    return lib


lib = _load()


def _check(status: int) -> None:
    if status != VLC_OK:
        raise VlcError(status, lib.vlc_last_error_string().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors handed to libvlcache must be contiguous CUDA tensors")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


VLC_SHAPE_SCORE_PLAIN_ALU = 1


def make_shape(B, L, Hq, Hkv, d, m, tau, dtype, lens=None, flags=0) -> vlc_shape:
    """lens: optional int32 device tensor [B, 2] of per-request (m_b, tau_b); the caller keeps it alive."""
    code = {torch.float32: VLC_F32, torch.bfloat16: VLC_BF16, "f32": VLC_F32, "bf16": VLC_BF16}.get(dtype, dtype)
    if lens is not None:
        assert lens.dtype == torch.int32 and lens.is_cuda and lens.is_contiguous() and tuple(lens.shape) == (B, 2)
    return vlc_shape(B, L, Hq, Hkv, d, m, tau, code, None if lens is None else lens.data_ptr(), int(flags), 0)


def vlc_version() -> str:
    return lib.vlc_version().decode()


def vlc_last_error_string() -> str:
    return lib.vlc_last_error_string().decode()


def vlc_workspace_bytes(shape: vlc_shape) -> int:
    n = lib.vlc_workspace_bytes(C.byref(shape))
    if n == 0:
        raise VlcError(VLC_ERR_SHAPE, vlc_last_error_string())
    return n


def vlc_score(shape, q_win, k, sm_scale, p, scores, row_max, row_sum, nnz, workspace) -> None:
    _check(lib.vlc_score(C.byref(shape), _ptr(q_win), _ptr(k), _ptr(sm_scale), float(p), _ptr(scores),
                         _ptr(row_max), _ptr(row_sum), _ptr(nnz), _ptr(workspace),
                         0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def vlc_score_static_max_workspace() -> int:
    return lib.vlc_score_static_max_workspace()


def vlc_score_static(shape, q_win, k, sm_scale, p, scores, row_max, row_sum, nnz) -> None:
    _check(lib.vlc_score_static(C.byref(shape), _ptr(q_win), _ptr(k), _ptr(sm_scale), float(p), _ptr(scores),
                                _ptr(row_max), _ptr(row_sum), _ptr(nnz), _stream()))


def vlc_sparsity(shape, q_win, k, sm_scale, row_max, p, nnz, gamma, workspace) -> None:
    _check(lib.vlc_sparsity(C.byref(shape), _ptr(q_win), _ptr(k), _ptr(sm_scale), _ptr(row_max), float(p),
                            _ptr(nnz), _ptr(gamma), _ptr(workspace),
                            0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def vlc_window_attn_workspace_bytes(shape: vlc_shape) -> int:
    n = C.c_size_t(0)
    _check(lib.vlc_window_attn_workspace_bytes(C.byref(shape), C.byref(n)))
    return n.value


def vlc_window_attn(shape, q_win, k, v, sm_scale, out, row_max, row_sum, workspace) -> None:
    _check(lib.vlc_window_attn(C.byref(shape), _ptr(q_win), _ptr(k), _ptr(v), _ptr(sm_scale), _ptr(out),
                               _ptr(row_max), _ptr(row_sum), _ptr(workspace),
                               0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def vlc_score_from_stats(shape, q_win, k, sm_scale, p, row_max, row_sum, scores, nnz) -> None:
    _check(lib.vlc_score_from_stats(C.byref(shape), _ptr(q_win), _ptr(k), _ptr(sm_scale), float(p), _ptr(row_max),
                                    _ptr(row_sum), _ptr(scores), _ptr(nnz), _stream()))


def vlc_allocate(shape, nnz, alpha_num, alpha_den, k_out, beta_out) -> None:
    _check(lib.vlc_allocate(C.byref(shape), _ptr(nnz), int(alpha_num), int(alpha_den), _ptr(k_out),
                            _ptr(beta_out), _stream()))


def vlc_cache_bytes(shape, T_max, sum_k_max) -> int:
    n = lib.vlc_cache_bytes(C.byref(shape), int(T_max), int(sum_k_max))
    if n == 0:
        raise VlcError(VLC_ERR_INVALID_ARG, vlc_last_error_string())
    return n


def vlc_cache_bytes_fp8(shape, T_max, sum_k_max) -> int:
    n = lib.vlc_cache_bytes_fp8(C.byref(shape), int(T_max), int(sum_k_max))
    if n == 0:
        raise VlcError(VLC_ERR_INVALID_ARG, vlc_last_error_string())
    return n


def make_options(**kw) -> vlc_cache_options:
    """vlc_cache_options with the named fields set and everything else 0 (the library's choice)."""
    o = vlc_cache_options()
    for name, value in kw.items():
        if name == "reserved" or name not in {f[0] for f in vlc_cache_options._fields_}:
            raise ValueError(f"vlc_cache_options has no field {name}")
        setattr(o, name, int(value))
    return o


def vlc_cache_bytes_opt(shape, T_max, sum_k_max, options) -> int:
    n = lib.vlc_cache_bytes_opt(C.byref(shape), int(T_max), int(sum_k_max), None if options is None else C.byref(options))
    if n == 0:
        raise VlcError(VLC_ERR_INVALID_ARG, vlc_last_error_string())
    return n


class Cache:
    """Owns the arena tensor and the library's host-side handle."""

    def __init__(self, shape: vlc_shape, T_max: int, sum_k_max: int, device="cuda", fp8: bool = False,
                 options: Optional[vlc_cache_options] = None):
        if options is None:
            options = make_options(kv_fp8=int(bool(fp8)))
        elif fp8:
            options.kv_fp8 = 1
        self.shape, self.T_max, self.sum_k_max, self.fp8 = shape, int(T_max), int(sum_k_max), bool(options.kv_fp8)
        self.options = options
        nbytes = vlc_cache_bytes_opt(shape, T_max, sum_k_max, options)
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=device)
        handle = C.c_void_p()
        _check(lib.vlc_cache_create_opt(C.byref(shape), self.T_max, self.sum_k_max, C.byref(options), self.arena.data_ptr(),
                                        nbytes, C.byref(handle)))
        self.handle = handle
        lay = vlc_cache_layout()
        _check(lib.vlc_cache_get_layout(self.handle, C.byref(lay)))
        self.layout = lay

    def close(self) -> None:
        if self.handle:
            lib.vlc_cache_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def vlc_cache_create(shape, T_max, sum_k_max, device="cuda") -> Cache:
    return Cache(shape, T_max, sum_k_max, device)


def vlc_cache_create_fp8(shape, T_max, sum_k_max, device="cuda") -> Cache:
    return Cache(shape, T_max, sum_k_max, device, fp8=True)


def vlc_cache_create_opt(shape, T_max, sum_k_max, options, device="cuda") -> Cache:
    return Cache(shape, T_max, sum_k_max, device, options=options)


def vlc_cache_status(cache: Cache) -> None:
    """Synchronises the stream; raises VlcError if the device flagged a budget or capacity error."""
    _check(lib.vlc_cache_status(cache.handle, _stream()))


def vlc_topk_compact(cache: Cache, scores, k, n_recent, k_full, v_full, idx_out) -> None:
    _check(lib.vlc_topk_compact(cache.handle, _ptr(scores), _ptr(k), int(n_recent), _ptr(k_full), _ptr(v_full),
                                _ptr(idx_out), _stream()))


def vlc_topk_compact_recent_frac(cache: Cache, scores, k, recent_num, recent_den, k_full, v_full, idx_out) -> None:
    _check(lib.vlc_topk_compact_recent_frac(cache.handle, _ptr(scores), _ptr(k), int(recent_num), int(recent_den),
                                            _ptr(k_full), _ptr(v_full), _ptr(idx_out), _stream()))


def vlc_cache_hit_rate(cache: Cache, scores_star, hits_out, rate_out) -> None:
    _check(lib.vlc_cache_hit_rate(cache.handle, _ptr(scores_star), _ptr(hits_out), _ptr(rate_out), _stream()))


def vlc_decode_attn(cache: Cache, layer_begin, layer_end, q, k_new, v_new, sm_scale, out) -> None:
    _check(lib.vlc_decode_attn(cache.handle, int(layer_begin), int(layer_end), _ptr(q), _ptr(k_new), _ptr(v_new),
                               _ptr(sm_scale), _ptr(out), _stream()))


def vlc_probe_read_stream(buf, sink, blocks) -> None:
    _check(lib.vlc_probe_read_stream(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), int(blocks), _stream()))


def vlc_decode_attn_steps(cache: Cache, layer_begin, layer_end, n_steps, q, k_new, v_new, sm_scale, out) -> None:
    _check(lib.vlc_decode_attn_steps(cache.handle, int(layer_begin), int(layer_end), int(n_steps), _ptr(q),
                                     _ptr(k_new), _ptr(v_new), _ptr(sm_scale), _ptr(out), _stream()))
