"""ctypes binding with the same names as include/freqkv.h (argument marshalling only).

Every step of the compression runs inside libfreqkv's HIP kernels; this module only builds
the C structs from torch tensors (device memory, strides, stream) and raises when the
library is missing or returns an error.  There is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "lib", "libfreqkv.so")
_lib = None

BF16, F32 = 0, 1
FLAG_NO_RESCALE = 0x1
FLAG_DROPPING = 0x2
FLAG_RETAIN_HIGH = 0x4
FLAG_SINGLE_FOLD = 0x8
FLAG_TWO_LEVEL_FOLD = 0x10
FLAG_DENSE = 0x20

OK, NOOP = 0, 1
E_INVALID, E_UNSUPPORTED, E_WORKSPACE, E_HIP, E_ALLOC = -1, -2, -3, -4, -5


class FreqKVError(RuntimeError):
    def __init__(self, status: int, detail: str = ""):
        self.status = status
        name = status_string(status) if _lib is not None else str(status)
        super().__init__(f"{name}{(': ' + detail) if detail else ''}")


class Layout(C.Structure):
    """struct freqkv_layout (include/freqkv.h)."""
    _fields_ = [
        ("dtype", C.c_int32), ("n_layers", C.c_int32), ("batch", C.c_int32), ("token_capacity", C.c_int32),
        ("stride_layer", C.c_int64), ("stride_batch", C.c_int64), ("stride_head", C.c_int64),
        ("stride_token", C.c_int64),
        ("pointer_table", C.c_int32), ("flags", C.c_uint32),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
        ("tap_f32", C.c_void_p),
    ]


class Plan(C.Structure):
    """struct freqkv_plan (include/freqkv.h)."""
    _fields_ = [
        ("span_len", C.c_int32), ("retained_len", C.c_int32), ("new_len", C.c_int32),
        ("head_tensors", C.c_int32), ("variant", C.c_int32), ("reserved", C.c_int32),
        ("workspace_bytes", C.c_size_t), ("workspace_min_bytes", C.c_size_t), ("basis_bytes", C.c_size_t),
        ("flops_dense", C.c_double), ("flops_executed", C.c_double), ("bytes_algorithmic", C.c_double),
    ]


class Profile(C.Structure):
    """struct freqkv_profile (include/freqkv.h)."""
    _fields_ = [
        ("calls", C.c_int64), ("launches_prepare", C.c_int64), ("launches_contract", C.c_int64),
        ("launches_tail", C.c_int64),
        ("ms_prepare", C.c_double), ("ms_contract", C.c_double), ("ms_tail", C.c_double),
        ("launches_attend", C.c_int64), ("ms_attend", C.c_double),
    ]


class PrefillPlan(C.Structure):
    """struct freqkv_prefill_plan (include/freqkv.h)."""
    _fields_ = [
        ("workspace_bytes", C.c_size_t), ("key_tiles", C.c_int32), ("query_blocks", C.c_int32),
        ("flops", C.c_double), ("bytes_algorithmic", C.c_double),
    ]


class AttendPlan(C.Structure):
    """struct freqkv_attend_plan (include/freqkv.h)."""
    _fields_ = [
        ("n_split", C.c_int32), ("chunk_rows", C.c_int32), ("heads_together", C.c_int32), ("reserved", C.c_int32),
        ("workspace_bytes", C.c_size_t), ("bytes_algorithmic", C.c_double), ("flops", C.c_double),
    ]


def lib_path() -> str:
    return _LIB_PATH


def load() -> C.CDLL:
    """Load libfreqkv.so; fails loudly when it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FreqKVError(E_HIP, f"{_LIB_PATH} is missing: run `python -m paper_2505_00570_amd.build`")
        lib = C.CDLL(_LIB_PATH)
        LP, PP = C.POINTER(Layout), C.POINTER(Plan)
        lib.freqkv_plan.argtypes = [LP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, PP]
        lib.freqkv_plan.restype = C.c_int
        lib.freqkv_compress.argtypes = [C.c_void_p, C.c_void_p, LP, C.c_int, C.c_int, C.c_int, C.c_int,
                                        C.c_int, C.c_double, C.c_void_p]
        lib.freqkv_compress.restype = C.c_int
        lib.freqkv_attend_plan.argtypes = [LP, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(AttendPlan)]
        lib.freqkv_attend_plan.restype = C.c_int
        lib.freqkv_attend_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, LP,
                                             C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_void_p]
        lib.freqkv_attend_decode.restype = C.c_int
        lib.freqkv_attend_decode_noalloc.argtypes = lib.freqkv_attend_decode.argtypes
        lib.freqkv_attend_decode_noalloc.restype = C.c_int
        lib.freqkv_noalloc_scratch_bytes.argtypes = []
        lib.freqkv_noalloc_scratch_bytes.restype = C.c_size_t
        lib.freqkv_attend_decode_ragged.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, LP,
                                                    C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_double,
                                                    C.c_void_p]
        lib.freqkv_attend_decode_ragged.restype = C.c_int
        lib.freqkv_compress_ragged.argtypes = [C.c_void_p, C.c_void_p, LP, C.c_int, C.c_int, C.POINTER(C.c_int32),
                                               C.POINTER(C.c_int32), C.c_int, C.c_int, C.c_double, C.c_void_p]
        lib.freqkv_compress_ragged.restype = C.c_int
        lib.freqkv_power_spectrum.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, LP, C.c_int, C.c_int, C.c_int,
                                              C.c_int, C.c_void_p]
        lib.freqkv_power_spectrum.restype = C.c_int
        lib.freqkv_attend_prefill_plan.argtypes = [LP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(PrefillPlan)]
        lib.freqkv_attend_prefill_plan.restype = C.c_int
        lib.freqkv_attend_prefill.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, LP,
                                              C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_void_p]
        lib.freqkv_attend_prefill.restype = C.c_int
        lib.freqkv_prepare.argtypes = [C.c_int, C.c_uint32, C.c_int, C.c_int, C.c_double, C.c_void_p]
        lib.freqkv_prepare.restype = C.c_int
        lib.freqkv_status_string.argtypes = [C.c_int]
        lib.freqkv_status_string.restype = C.c_char_p
        lib.freqkv_last_error.argtypes = []
        lib.freqkv_last_error.restype = C.c_char_p
        lib.freqkv_shutdown.argtypes = []
        lib.freqkv_shutdown.restype = None
        lib.freqkv_version.argtypes = []
        lib.freqkv_version.restype = C.c_int
        lib.freqkv_profile_enable.argtypes = [C.c_int]
        lib.freqkv_profile_enable.restype = C.c_int
        lib.freqkv_profile_read.argtypes = [C.POINTER(Profile)]
        lib.freqkv_profile_read.restype = C.c_int
        lib.freqkv_calibrate_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p,
                                              C.POINTER(C.c_double)]
        lib.freqkv_calibrate_copy.restype = C.c_int
        lib.freqkv_calibrate_mfma.argtypes = [C.c_int, C.c_void_p, C.POINTER(C.c_double)]
        lib.freqkv_calibrate_mfma.restype = C.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().freqkv_status_string(int(status)).decode()


def last_error() -> str:
    return load().freqkv_last_error().decode()


def version() -> int:
    return load().freqkv_version()


def shutdown() -> None:
    load().freqkv_shutdown()


def _check(rc: int) -> int:
    if rc < 0:
        raise FreqKVError(rc, last_error())
    return rc


def plan(layout: Layout, n_heads: int, head_dim: int, cur_len: int, window: int, n_sink: int,
         retain_ratio: float, check: bool = True):
    """freqkv_plan: returns (status, Plan).  Host arithmetic only."""
    out = Plan()
    rc = load().freqkv_plan(C.byref(layout), n_heads, head_dim, cur_len, window, n_sink,
                            float(retain_ratio), C.byref(out))
    if check:
        _check(rc)
    return rc, out


def prepare(dtype: int, flags: int, window: int, n_sink: int, retain_ratio: float, stream=None) -> int:
    return _check(load().freqkv_prepare(dtype, flags, window, n_sink, float(retain_ratio), _stream_ptr(stream)))


def compress(k, v, layout: Layout, n_heads: int, head_dim: int, cur_len: int, window: int, n_sink: int,
             retain_ratio: float, stream=None, check: bool = True) -> int:
    """freqkv_compress.  k, v: torch CUDA tensors, raw device addresses (int), or ctypes arrays of
    per-layer device pointers when layout.pointer_table == 1.  Returns the status (0 or 1)."""
    rc = load().freqkv_compress(_dev_ptr(k), _dev_ptr(v), C.byref(layout), n_heads, head_dim, cur_len,
                                window, n_sink, float(retain_ratio), _stream_ptr(stream))
    return _check(rc) if check else rc


def attend_plan(layout: Layout, n_q_heads: int, n_kv_heads: int, head_dim: int, cur_len: int, check: bool = True):
    """freqkv_attend_plan: returns (status, AttendPlan).  Host arithmetic only."""
    out = AttendPlan()
    rc = load().freqkv_attend_plan(C.byref(layout), n_q_heads, n_kv_heads, head_dim, cur_len, C.byref(out))
    if check:
        _check(rc)
    return rc, out


def attend_decode(q, k, v, out, lse, layout: Layout, n_q_heads: int, n_kv_heads: int, head_dim: int,
                  cur_len: int, q_pos: int = -1, rope_base: float = 10000.0, stream=None, check: bool = True) -> int:
    """freqkv_attend_decode.  q, out: dense [layer, batch, q_head, dim] device tensors of the cache dtype;
    lse: fp32 [layer, batch, q_head] device tensor or None; k, v as in compress."""
    rc = load().freqkv_attend_decode(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(out), _dev_ptr(lse),
                                     C.byref(layout), n_q_heads, n_kv_heads, head_dim, cur_len, q_pos,
                                     float(rope_base), _stream_ptr(stream))
    return _check(rc) if check else rc


def attend_decode_noalloc(q, k, v, out, lse, layout: Layout, n_q_heads: int, n_kv_heads: int, head_dim: int,
                          cur_len: int, q_pos: int = -1, rope_base: float = 10000.0, stream=None,
                          check: bool = True) -> int:
    """freqkv_attend_decode_noalloc: as attend_decode, scratch inside the library, layout.workspace ignored."""
    rc = load().freqkv_attend_decode_noalloc(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(out), _dev_ptr(lse),
                                             C.byref(layout), n_q_heads, n_kv_heads, head_dim, cur_len, q_pos,
                                             float(rope_base), _stream_ptr(stream))
    return _check(rc) if check else rc


def noalloc_scratch_bytes() -> int:
    return int(load().freqkv_noalloc_scratch_bytes())


def attend_decode_ragged(q, k, v, out, lse, layout: Layout, n_q_heads: int, n_kv_heads: int, head_dim: int,
                         cur_lens, max_cur_len: int, rope_base: float = 10000.0, stream=None, check: bool = True) -> int:
    """freqkv_attend_decode_ragged.  cur_lens: int32 device tensor [batch]."""
    rc = load().freqkv_attend_decode_ragged(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(out), _dev_ptr(lse),
                                            C.byref(layout), n_q_heads, n_kv_heads, head_dim, _dev_ptr(cur_lens),
                                            max_cur_len, float(rope_base), _stream_ptr(stream))
    return _check(rc) if check else rc


def compress_ragged(k, v, layout: Layout, n_heads: int, head_dim: int, cur_lens, window: int, n_sink: int,
                    retain_ratio: float, stream=None, check: bool = True):
    """freqkv_compress_ragged.  cur_lens: sequence of ints (host).  Returns (status, new_lens list)."""
    n = len(cur_lens)
    cl = (C.c_int32 * n)(*[int(c) for c in cur_lens])
    nl = (C.c_int32 * n)()
    rc = load().freqkv_compress_ragged(_dev_ptr(k), _dev_ptr(v), C.byref(layout), n_heads, head_dim, cl, nl,
                                       window, n_sink, float(retain_ratio), _stream_ptr(stream))
    if check:
        _check(rc)
    return rc, list(nl)


def power_spectrum(k, v, out, layout: Layout, n_heads: int, head_dim: int, row0: int, n_rows: int, stream=None,
                   check: bool = True) -> int:
    """freqkv_power_spectrum.  out: fp32 device tensor [2, layers, heads, n_rows]."""
    rc = load().freqkv_power_spectrum(_dev_ptr(k), _dev_ptr(v), _dev_ptr(out), C.byref(layout), n_heads, head_dim,
                                      row0, n_rows, _stream_ptr(stream))
    return _check(rc) if check else rc


def attend_prefill_plan(layout: Layout, n_q_heads: int, n_kv_heads: int, head_dim: int, cur_len: int, q_len: int,
                        check: bool = True):
    """freqkv_attend_prefill_plan: returns (status, PrefillPlan).  Host arithmetic only."""
    out = PrefillPlan()
    rc = load().freqkv_attend_prefill_plan(C.byref(layout), n_q_heads, n_kv_heads, head_dim, cur_len, q_len,
                                           C.byref(out))
    if check:
        _check(rc)
    return rc, out


def attend_prefill(q, k, v, out, lse, layout: Layout, n_q_heads: int, n_kv_heads: int, head_dim: int,
                   cur_len: int, q_len: int, rope_base: float = 10000.0, stream=None, check: bool = True) -> int:
    """freqkv_attend_prefill.  q, out: dense [layer, batch, q_head, q_len, dim] bf16 device tensors."""
    rc = load().freqkv_attend_prefill(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(out), _dev_ptr(lse),
                                      C.byref(layout), n_q_heads, n_kv_heads, head_dim, cur_len, q_len,
                                      float(rope_base), _stream_ptr(stream))
    return _check(rc) if check else rc


def profile_enable(on: bool) -> None:
    _check(load().freqkv_profile_enable(1 if on else 0))


def profile_read() -> Profile:
    out = Profile()
    _check(load().freqkv_profile_read(C.byref(out)))
    return out


def calibrate_copy(dst, src, nbytes: int, repeats: int = 10, stream=None) -> float:
    """freqkv_calibrate_copy: measured read+write GB/s of a plain device copy."""
    out = C.c_double()
    _check(load().freqkv_calibrate_copy(_dev_ptr(dst), _dev_ptr(src), nbytes, repeats, _stream_ptr(stream),
                                        C.byref(out)))
    return out.value


def calibrate_mfma(iters: int = 20000, stream=None) -> float:
    """freqkv_calibrate_mfma: measured TFLOP/s of a register-only fp16 MFMA loop on random operands."""
    out = C.c_double()
    _check(load().freqkv_calibrate_mfma(iters, _stream_ptr(stream), C.byref(out)))
    return out.value


# ---------------------------------------------------------------- marshalling helpers

def _dev_ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return C.c_void_p(x)
    if isinstance(x, C.Array):
        return C.cast(x, C.c_void_p)
    if hasattr(x, "data_ptr"):
        return C.c_void_p(x.data_ptr())
    return x


def _stream_ptr(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)          # torch.cuda.Stream


def layout_for(k, *, batch_dim: bool = True, workspace=None, tap=None, flags: int = 0) -> Layout:
    """Layout of a torch cache tensor shaped [layer, batch, head, token, dim] (any strides with
    unit dim stride); `workspace` / `tap` are torch CUDA tensors or None."""
    import torch
    if k.dim() != 5:
        raise ValueError("expected a [layer, batch, head, token, dim] tensor")
    if k.stride(4) != 1:
        raise ValueError("channel stride must be 1")
    dt = {torch.bfloat16: BF16, torch.float32: F32}[k.dtype]
    L = Layout()
    L.dtype = dt
    L.n_layers, L.batch = k.shape[0], k.shape[1]
    L.token_capacity = k.shape[3]
    L.stride_layer, L.stride_batch, L.stride_head, L.stride_token = k.stride(0), k.stride(1), k.stride(2), k.stride(3)
    L.pointer_table = 0
    L.flags = flags
    if workspace is not None:
        L.workspace = workspace.data_ptr()
        L.workspace_bytes = workspace.numel() * workspace.element_size()
    if tap is not None:
        L.tap_f32 = tap.data_ptr()
    return L
