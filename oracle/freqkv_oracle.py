"""FreqKV reference oracle -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
module; the product library never does.  All floating-point work is done in
fp64 by the plain C routines in ``freqkv_oracle.c`` (direct O(n^2) sums of the
paper's Appendix-A definitions); this file only marshals numpy arrays, applies
the cache bookkeeping of Sec. 3.4 and states the integer rules (retained
length, trigger schedule) of Sec. 4.1.

Parity pins live in ``tests/test_oracle_pins.py``.  Numeric values of
compressed K/V for real text are "parity unpinned": the paper prints none.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "freqkv_oracle.c")
_LIB = os.path.join(_HERE, "libfreqkv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc -O2 (no fast-math) and return the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        i = ctypes.c_int
        lib.freqkv_oracle_dct2.argtypes = [dp, i, i, i, dp]
        lib.freqkv_oracle_idct2.argtypes = [dp, i, i, dp]
        lib.freqkv_oracle_compress_span.argtypes = [dp, i, i, i, i, dp, dp]
        lib.freqkv_oracle_compress_head.argtypes = [dp, i, i, i, i, i, i, dp]
        for f in (lib.freqkv_oracle_dct2, lib.freqkv_oracle_idct2,
                  lib.freqkv_oracle_compress_span, lib.freqkv_oracle_compress_head):
            f.restype = i
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _as2d(x) -> np.ndarray:
    a = np.ascontiguousarray(x, dtype=np.float64)
    if a.ndim == 1:
        a = a[:, None]
    if a.ndim != 2:
        raise ValueError("expected [tokens] or [tokens, channels]")
    return a


# ---------------------------------------------------------------- integer rules

def retained_len(n: int, retain_ratio: float) -> int:
    """Lc = gamma * n (Sec. 3.3), floored to an integer and clamped to [1, n].

    The paper only uses ratios for which gamma*n is an integer (4092 -> 2046,
    Sec. 4.1); the small epsilon guards ratios such as 0.3 whose product lands
    a rounding error below an integer.
    """
    if not (0.0 < retain_ratio <= 1.0) or n < 1:
        raise ValueError("need 0 < retain_ratio <= 1 and n >= 1")
    return max(1, min(n, int(math.floor(retain_ratio * n + 1e-9))))


def new_len(cur_len: int, window: int, n_sink: int, retain_ratio: float) -> int:
    """Cache length after one trigger: sinks + retained rows + recent tail (Sec. 3.4)."""
    lc = retained_len(window - n_sink, retain_ratio)
    return n_sink + lc + (cur_len - window)


def trigger_count(total_tokens: int, window: int, n_sink: int, retain_ratio: float) -> int:
    """Number of compressions while `total_tokens` tokens stream through the cache.

    Sec. 3.4: the cache is compressed once it is full and further tokens arrive;
    each compression frees window - n_sink - Lc slots, which the next chunk fills.
    """
    lc = retained_len(window - n_sink, retain_ratio)
    freed = window - n_sink - lc
    if freed <= 0:
        raise ValueError("retain_ratio leaves no room for new tokens")
    count, filled = 0, window          # `filled` = tokens consumed when the cache is next full
    while filled < total_tokens:
        count += 1
        filled += freed
    return count


# ---------------------------------------------------------------- transforms

def dct2(x, n_out: int | None = None) -> np.ndarray:
    """Orthonormal DCT-II along axis 0 (Appendix A); first n_out coefficients."""
    a = _as2d(x)
    n, d = a.shape
    n_out = n if n_out is None else n_out
    z = np.empty((n_out, d), dtype=np.float64)
    if _load().freqkv_oracle_dct2(_p(a), n, d, n_out, _p(z)) != 0:
        raise RuntimeError("oracle dct2 failed")
    return z


def idct2(z) -> np.ndarray:
    """Inverse orthonormal DCT-II along axis 0 (Appendix A), length = z.shape[0]."""
    a = _as2d(z)
    L, d = a.shape
    y = np.empty((L, d), dtype=np.float64)
    if _load().freqkv_oracle_idct2(_p(a), L, d, _p(y)) != 0:
        raise RuntimeError("oracle idct2 failed")
    return y


def compress_span(x, lc: int, rescale: bool = True, return_coeffs: bool = False):
    """y = sqrt(Lc/n) * IDCT_Lc(DCT_n(x)[0:Lc])  (Sec. 3.3 Eq. 2-3)."""
    a = _as2d(x)
    n, d = a.shape
    y = np.empty((lc, d), dtype=np.float64)
    z = np.empty((lc, d), dtype=np.float64) if return_coeffs else None
    rc = _load().freqkv_oracle_compress_span(_p(a), n, lc, d, int(bool(rescale)), _p(y),
                                             _p(z) if z is not None else None)
    if rc != 0:
        raise RuntimeError("oracle compress_span failed")
    return (y, z) if return_coeffs else y


def compress_head(cache, cur_len: int, window: int, n_sink: int, retain_ratio: float,
                  rescale: bool = True) -> np.ndarray:
    """One trigger on one head-tensor [tokens, d]: returns the new rows [0, new_len)."""
    a = _as2d(cache)[:cur_len]
    a = np.ascontiguousarray(a)
    d = a.shape[1]
    lc = retained_len(window - n_sink, retain_ratio)
    out = np.empty((n_sink + lc + cur_len - window, d), dtype=np.float64)
    rc = _load().freqkv_oracle_compress_head(_p(a), cur_len, d, window, n_sink, lc,
                                             int(bool(rescale)), _p(out))
    if rc != 0:
        raise RuntimeError("oracle compress_head failed")
    return out


def compress_span_high(x, lc: int, rescale: bool = True, return_coeffs: bool = False):
    """The high-frequency variant of the ablation tables (Sec. 3.2 summarisation table, appendix table on
    retaining high frequencies): the Lc HIGHEST coefficients of the n-point DCT are kept instead of the
    lowest.  The paper does not say how the kept band becomes Lc cached rows; the reading taken is the
    only one that reuses its inverse unchanged: the kept band, in order, is the input of the Lc-point
    inverse DCT, with the same sqrt(Lc/n) factor:  y = sqrt(Lc/n) * IDCT_Lc(DCT_n(x)[n-Lc:n])."""
    a = _as2d(x)
    n = a.shape[0]
    z = dct2(a)[n - lc:]
    y = idct2(z)
    if rescale:
        y = y * math.sqrt(lc / n)
    return (y, z) if return_coeffs else y


def compress_head_high(cache, cur_len: int, window: int, n_sink: int, retain_ratio: float,
                       rescale: bool = True) -> np.ndarray:
    """compress_head with the high band retained: same sinks, retained size and tail rule (Sec. 3.4)."""
    a = _as2d(cache)[:cur_len]
    lc = retained_len(window - n_sink, retain_ratio)
    y = compress_span_high(a[n_sink:window], lc, rescale)
    return np.concatenate([a[:n_sink], y, a[window:cur_len]], axis=0)


def power_spectrum(x) -> np.ndarray:
    """Average power spectrum of key or value states (Sec. 3.1 and its figure; appendix on the head-wise
    analysis): x [samples, tokens, channels] (or [tokens, channels]) is taken to the frequency domain by the
    orthonormal DCT-II along the token axis, and the squared coefficients are averaged over samples and
    channels.  Returns P[t], t = 0 .. tokens-1."""
    a = np.asarray(x, dtype=np.float64)
    if a.ndim == 2:
        a = a[None]
    acc = np.zeros(a.shape[1])
    for sample in a:
        z = dct2(sample)
        acc += (z ** 2).sum(axis=1)
    return acc / (a.shape[0] * a.shape[2])


def drop_head(cache, cur_len: int, window: int, n_sink: int, retain_ratio: float) -> np.ndarray:
    """The "Dropping" variant (appendix on the compression overhead): no transform, the span keeps
    its Lc most recent rows; same sinks, retained size and tail rule as compress_head."""
    a = _as2d(cache)[:cur_len]
    lc = retained_len(window - n_sink, retain_ratio)
    return np.concatenate([a[:n_sink], a[window - lc:window], a[window:cur_len]], axis=0)


def compress_heads(heads, cur_len: int, window: int, n_sink: int, retain_ratio: float,
                   threads: int = 1) -> list:
    """compress_head over a list of head-tensors, optionally on several host threads."""
    fn = lambda h: compress_head(h, cur_len, window, n_sink, retain_ratio)
    if threads <= 1:
        return [fn(h) for h in heads]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(fn, heads))
