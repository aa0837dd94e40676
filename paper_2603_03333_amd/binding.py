"""Thin ctypes binding of libdropmatch.so: argument marshalling only.

Function names mirror the C ABI (include/dropmatch.h).  PyTorch is used for device
memory and streams; every step of the verify path runs in the library's HIP kernels.
There is no fallback: if the library is missing or fails to load, importing the
functions raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

DM_OK, DM_EINVAL, DM_ENOMEM, DM_EHIP, DM_EUNSUPPORTED = 0, -1, -2, -3, -4
DM_F32, DM_BF16 = 0, 1
DM_RULE_ANY, DM_RULE_MAJORITY, DM_RULE_JS, DM_RULE_JS_OR_MAJORITY = 0, 1, 2, 3
DM_FLAG_SHARE_MASK_ACROSS_POS, DM_FLAG_FORCE_GENERIC, DM_FLAG_CLEAN_LAST_PATH, DM_FLAG_SEPARATE_VOTE = 1, 2, 4, 8
DM_FLAG_SAMPLE_PATHS = 16
DM_FLAG_SPARSE_CORRECTION = 32

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdropmatch.so")

EXPORTS = ("dm_create", "dm_destroy", "dm_last_error", "dm_validate", "dropmatch_verify",
           "dm_debug_masks", "dm_debug_logits", "dm_debug_stream_read", "dm_kernel_choice", "dm_set_profiling", "dm_set_profiling_stride", "dm_get_profile",
           "dm_get_profile_stages", "dm_get_profile_samples", "dm_reserve_js", "dropmatch_verify_js", "dropmatch_verify_static")


class dm_params(C.Structure):
    _fields_ = [("B", C.c_int32), ("T", C.c_int32), ("K", C.c_int32), ("d", C.c_int32), ("V", C.c_int32),
                ("dtype", C.c_int32), ("p", C.c_float), ("step", C.c_uint32), ("rule", C.c_int32),
                ("flags", C.c_uint32), ("seeds", C.POINTER(C.c_uint64)), ("parent", C.c_void_p),
                ("temperature", C.c_float), ("top_p", C.c_float), ("step_dev", C.c_void_p)]


class DropMatchError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"dropmatch status {status}: {message}")
        self.status = status
        self.message = message


_lib = None


def load_library():
    """Load libdropmatch.so (building it first if it was never built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build(verbose=False)
    # torch ships its own HIP runtime with the same soname; importing it first makes the
    # library bind to that copy, so device pointers of torch tensors are valid in it.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.dm_create.argtypes = [C.POINTER(vp), C.c_int, i64, i32, i32]
    lib.dm_create.restype = C.c_int
    lib.dm_destroy.argtypes = [vp]
    lib.dm_destroy.restype = C.c_int
    lib.dm_last_error.argtypes = [vp]
    lib.dm_last_error.restype = C.c_char_p
    lib.dm_validate.argtypes = [C.POINTER(dm_params), C.c_char_p, i32]
    lib.dm_validate.restype = C.c_int
    lib.dm_kernel_choice.argtypes = [C.POINTER(dm_params)]
    lib.dm_kernel_choice.restype = i32
    lib.dropmatch_verify.argtypes = [vp, C.POINTER(dm_params)] + [vp] * 11
    lib.dropmatch_verify.restype = C.c_int
    lib.dropmatch_verify_static.argtypes = [C.c_int, C.POINTER(dm_params)] + [vp] * 11
    lib.dropmatch_verify_static.restype = C.c_int
    lib.dm_debug_masks.argtypes = [vp, C.POINTER(dm_params), vp, vp]
    lib.dm_debug_masks.restype = C.c_int
    lib.dm_debug_logits.argtypes = [vp, C.POINTER(dm_params), vp, vp, i32, i32, vp, vp]
    lib.dm_debug_logits.restype = C.c_int
    lib.dm_debug_stream_read.argtypes = [vp, vp, i64, vp]
    lib.dm_debug_stream_read.restype = C.c_int
    lib.dm_set_profiling.argtypes = [vp, i32]
    lib.dm_set_profiling.restype = C.c_int
    lib.dm_set_profiling_stride.argtypes = [vp, i32]
    lib.dm_set_profiling_stride.restype = C.c_int
    lib.dm_get_profile.argtypes = [vp, C.POINTER(i32)] + [C.POINTER(C.c_float)] * 3
    lib.dm_get_profile.restype = C.c_int
    lib.dm_get_profile_stages.argtypes = [vp, C.POINTER(i32), C.POINTER(C.c_float)]
    lib.dm_get_profile_stages.restype = C.c_int
    lib.dm_get_profile_samples.argtypes = [vp, i32, C.POINTER(C.c_float), i32, C.POINTER(i32)]
    lib.dm_get_profile_samples.restype = C.c_int
    lib.dm_reserve_js.argtypes = [vp, i64, i32]
    lib.dm_reserve_js.restype = C.c_int
    lib.dropmatch_verify_js.argtypes = [vp, C.POINTER(dm_params)] + [vp] * 14
    lib.dropmatch_verify_js.restype = C.c_int
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def make_params(B: int, T: int, K: int, d: int, V: int, dtype: int, p: float, seeds: Sequence[int],
                step: int = 0, rule: int = DM_RULE_ANY, flags: int = 0, parent=None, temperature: float = 0.0,
                top_p: float = 0.0, step_dev=None):
    """Fill a dm_params.  Returns (params, keepalive): hold `keepalive` while params is in use."""
    arr = (C.c_uint64 * len(seeds))(*[int(s) & 0xFFFFFFFFFFFFFFFF for s in seeds])
    prm = dm_params(B, T, K, d, V, dtype, p, step, rule, flags, C.cast(arr, C.POINTER(C.c_uint64)), _ptr(parent),
                    temperature, top_p, _ptr(step_dev))
    return prm, (arr, parent, step_dev)


def dm_validate(prm: dm_params):
    buf = C.create_string_buffer(256)
    st = load_library().dm_validate(C.byref(prm), buf, 256)
    return st, buf.value.decode()


def dm_kernel_choice(prm: dm_params) -> int:
    return int(load_library().dm_kernel_choice(C.byref(prm)))


def dm_last_error(ctx) -> str:
    return load_library().dm_last_error(ctx).decode()


def _check(ctx, st: int):
    if st != DM_OK:
        raise DropMatchError(st, dm_last_error(ctx))


def dm_create(device: int, max_rows: int, max_d: int, max_V: int):
    ctx = C.c_void_p()
    st = load_library().dm_create(C.byref(ctx), device, max_rows, max_d, max_V)
    if st != DM_OK:
        raise DropMatchError(st, dm_last_error(None))
    return ctx


def dm_destroy(ctx) -> None:
    st = load_library().dm_destroy(ctx)
    if st != DM_OK:
        raise DropMatchError(st, dm_last_error(None))


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def dropmatch_verify(ctx, prm: dm_params, h, W, draft_ids, accept_len, best_node=None, accept_mask=None,
                     hit=None, path_ids=None, vote_ids=None, vote_cnt=None, stream=None) -> None:
    """Enqueue one verification step on `stream` (default: torch's current stream).
    All tensor arguments are torch CUDA tensors (or None where the ABI allows NULL)."""
    st = load_library().dropmatch_verify(ctx, C.byref(prm), _ptr(h), _ptr(W), _ptr(draft_ids), _ptr(accept_len),
                                         _ptr(best_node), _ptr(accept_mask), _ptr(hit), _ptr(path_ids),
                                         _ptr(vote_ids), _ptr(vote_cnt), _stream_handle(stream))
    _check(ctx, st)


def dropmatch_verify_static(device: int, prm: dm_params, h, W, draft_ids, accept_len, best_node=None, accept_mask=None,
                            hit=None, path_ids=None, vote_ids=None, vote_cnt=None, stream=None) -> None:
    """dropmatch_verify on the library's fixed workspace of GPU `device`: no context, no allocation."""
    st = load_library().dropmatch_verify_static(device, C.byref(prm), _ptr(h), _ptr(W), _ptr(draft_ids),
                                                _ptr(accept_len), _ptr(best_node), _ptr(accept_mask), _ptr(hit),
                                                _ptr(path_ids), _ptr(vote_ids), _ptr(vote_cnt), _stream_handle(stream))
    _check(None, st)


def dm_reserve_js(ctx, max_positions: int, max_K: int) -> None:
    _check(ctx, load_library().dm_reserve_js(ctx, max_positions, max_K))


def dropmatch_verify_js(ctx, prm: dm_params, h, W, draft_ids, draft_probs, accept_len, best_node=None,
                        accept_mask=None, hit=None, path_ids=None, vote_ids=None, vote_cnt=None, js_draft=None,
                        js_heads=None, stream=None) -> None:
    """Enqueue one verification step with a distribution-level rule (Eq. 6 / Algorithm 1)."""
    st = load_library().dropmatch_verify_js(ctx, C.byref(prm), _ptr(h), _ptr(W), _ptr(draft_ids), _ptr(draft_probs),
                                            _ptr(accept_len), _ptr(best_node), _ptr(accept_mask), _ptr(hit),
                                            _ptr(path_ids), _ptr(vote_ids), _ptr(vote_cnt), _ptr(js_draft),
                                            _ptr(js_heads), _stream_handle(stream))
    _check(ctx, st)


def dm_debug_masks(ctx, prm: dm_params, bits, stream=None) -> None:
    st = load_library().dm_debug_masks(ctx, C.byref(prm), _ptr(bits), _stream_handle(stream))
    _check(ctx, st)


def dm_debug_logits(ctx, prm: dm_params, h, W, v0: int, v1: int, logits, stream=None) -> None:
    st = load_library().dm_debug_logits(ctx, C.byref(prm), _ptr(h), _ptr(W), v0, v1, _ptr(logits),
                                        _stream_handle(stream))
    _check(ctx, st)


def dm_debug_stream_read(ctx, src, nbytes: int, stream=None) -> None:
    """Enqueue a bare streaming read of the first nbytes bytes of the CUDA tensor src."""
    _check(ctx, load_library().dm_debug_stream_read(ctx, _ptr(src), int(nbytes), _stream_handle(stream)))


def dm_set_profiling(ctx, enabled) -> None:
    """False/0: off; True/1: events around every kernel; 2: only around the contraction kernel."""
    _check(ctx, load_library().dm_set_profiling(ctx, int(enabled)))


def dm_set_profiling_stride(ctx, stride: int) -> None:
    _check(ctx, load_library().dm_set_profiling_stride(ctx, int(stride)))


def dm_get_profile(ctx):
    """Returns (n_calls, ms_mask, ms_lmhead, ms_vote): mean kernel durations from HIP events."""
    n = C.c_int32()
    a, b, c = C.c_float(), C.c_float(), C.c_float()
    _check(ctx, load_library().dm_get_profile(ctx, C.byref(n), C.byref(a), C.byref(b), C.byref(c)))
    return n.value, a.value, b.value, c.value


def dm_get_profile_stages(ctx):
    """Returns (n_calls, [ms_mask, ms_lmhead, ms_js_pass1, ms_js_pass2, ms_vote])."""
    n = C.c_int32()
    ms = (C.c_float * 5)()
    _check(ctx, load_library().dm_get_profile_stages(ctx, C.byref(n), ms))
    return n.value, [float(x) for x in ms]


def dm_get_profile_samples(ctx, stage: int, n_max: int = 512):
    """The individual durations (ms) of one stage (0 mask rows, 1 LM head, 2/3 JS passes, 4 vote/accept)."""
    n = C.c_int32()
    ms = (C.c_float * n_max)()
    _check(ctx, load_library().dm_get_profile_samples(ctx, stage, ms, n_max, C.byref(n)))
    return [float(ms[i]) for i in range(n.value)]
