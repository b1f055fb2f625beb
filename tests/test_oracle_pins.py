"""Pins for the fp64 oracle: it is checked against things other than itself.

Each test names the passage of the paper (or the piece of mathematics) that
fixes the expected value.  A dropped term, a wrong normalisation, an index
off by one or a transposed operand in the oracle fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import scipy.fft

from oracle import freqkv_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_integers.txt")


def _rng(seed=0):
    return np.random.default_rng(seed)


def _dct_matrix(n):
    """Explicit orthonormal DCT-II matrix typed from Appendix A: C[t, j]."""
    C = np.zeros((n, n))
    for t in range(n):
        a = math.sqrt(1.0 / n) if t == 0 else math.sqrt(2.0 / n)
        for j in range(n):
            C[t, j] = a * math.cos(math.pi * t * (2 * j + 1) / (2 * n))
    return C


# -- P8: integers the paper prints ------------------------------------------------

def _golden():
    spans, counts = [], []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            p = line.split()
            if p[0] == "span":
                spans.append((int(p[1]), int(p[2]), float(p[3]), int(p[4]), int(p[5])))
            elif p[0] == "count":
                counts.append((int(p[1]), int(p[2])))
    return spans, counts


def test_paper_span_and_retained_length():
    spans, _ = _golden()
    assert spans
    for window, sink, ratio, n, lc in spans:
        assert window - sink == n
        assert orc.retained_len(n, ratio) == lc
    # LLaMA-3 window (Sec. 4.1): 8192 - 4 = 8188 -> 4094
    assert orc.retained_len(8188, 0.5) == 4094
    assert orc.retained_len(10, 1.0) == 10
    assert orc.retained_len(10, 0.3) == 3          # 0.3*10 = 2.9999999999999996 in binary
    assert orc.retained_len(7, 0.01) == 1          # clamps to one row


def test_paper_compression_counts():
    _, counts = _golden()
    assert len(counts) >= 8
    for total, expect in counts:
        assert orc.trigger_count(total, 4096, 4, 0.5) == expect, total
    # the 128K LLaMA-3 prefill of the benchmark workload (window 8192)
    assert orc.trigger_count(131072, 8192, 4, 0.5) == 31


# -- P4: brute force with explicit matrices on tiny sizes ------------------------

@pytest.mark.parametrize("n,lc,d", [(8, 4, 3), (9, 4, 2), (16, 16, 1), (13, 5, 4), (64, 32, 5), (30, 7, 2)])
def test_bruteforce_matrices(n, lc, d):
    x = _rng(n * 100 + lc).standard_normal((n, d))
    Cn, Cl = _dct_matrix(n), _dct_matrix(lc)
    assert np.allclose(Cn @ Cn.T, np.eye(n), atol=1e-13)
    z_ref = Cn @ x
    assert np.allclose(orc.dct2(x), z_ref, atol=1e-13)
    assert np.allclose(orc.dct2(x, lc), z_ref[:lc], atol=1e-13)
    assert np.allclose(orc.idct2(z_ref[:lc]), Cl.T @ z_ref[:lc], atol=1e-13)
    y_ref = math.sqrt(lc / n) * (Cl.T @ z_ref[:lc])
    y, z = orc.compress_span(x, lc, return_coeffs=True)
    assert np.allclose(y, y_ref, atol=1e-13)
    assert np.allclose(z, z_ref[:lc], atol=1e-13)
    y_nors = orc.compress_span(x, lc, rescale=False)
    assert np.allclose(y_nors, Cl.T @ z_ref[:lc], atol=1e-13)


# -- P1: ratio 1 is an exact round trip (the inverse recovers the signal, App. A) --

@pytest.mark.parametrize("n", [1, 2, 7, 254, 508])
def test_roundtrip_ratio_one(n):
    x = _rng(n).standard_normal((n, 3)) * 5.0
    y = orc.compress_span(x, n)
    assert np.max(np.abs(y - x)) < 1e-11
    assert np.max(np.abs(orc.idct2(orc.dct2(x)) - x)) < 1e-11


# -- P2: a constant sequence is reproduced exactly (rescaling restores the amplitude, Sec. 3.3) --

@pytest.mark.parametrize("n,lc", [(508, 254), (100, 37), (4092, 2046), (33, 1)])
def test_constant_preserved(n, lc):
    c = np.array([[3.25, -1.5, 1e-3]])
    x = np.repeat(c, n, axis=0)
    y, z = orc.compress_span(x, lc, return_coeffs=True)
    assert np.max(np.abs(y - np.repeat(c, lc, axis=0))) < 1e-11 * n
    assert lc == 1 or np.max(np.abs(z[1:])) < 1e-10 * n   # only the DC coefficient is non-zero
    assert np.allclose(z[0], c[0] * math.sqrt(n), rtol=1e-13)
    # without the rescale the amplitude grows by sqrt(n/lc) (rescaling ablation appendix)
    y2 = orc.compress_span(x, lc, rescale=False)
    assert np.allclose(y2, math.sqrt(n / lc) * np.repeat(c, lc, axis=0), rtol=1e-11)


# -- P3: Parseval for both transforms ---------------------------------------------

@pytest.mark.parametrize("n,lc", [(508, 254), (255, 100), (64, 64)])
def test_parseval(n, lc):
    x = _rng(7).standard_normal((n, 4))
    z_all = orc.dct2(x)
    assert np.allclose((z_all ** 2).sum(0), (x ** 2).sum(0), rtol=1e-12)
    y, z = orc.compress_span(x, lc, return_coeffs=True)
    assert np.allclose(z, z_all[:lc], atol=1e-13)
    assert np.allclose((y ** 2).sum(0), (lc / n) * (z ** 2).sum(0), rtol=1e-12)


# -- P5: a pure cosine below / above the cut ----------------------------------------

@pytest.mark.parametrize("n,lc", [(508, 254), (120, 45)])
def test_pure_cosine(n, lc):
    j = np.arange(n)
    m = np.arange(lc)
    for t0 in (0, 1, 2, lc // 2, lc - 1, lc, lc + 1, n - 1):
        x = np.cos(math.pi * t0 * (2 * j + 1) / (2 * n))
        y = orc.compress_span(x, lc)[:, 0]
        if t0 < lc:
            expect = np.cos(math.pi * t0 * (2 * m + 1) / (2 * lc))
        else:
            expect = np.zeros(lc)
        assert np.max(np.abs(y - expect)) < 1e-11, t0


# -- P6: closed form of the fused operator (Dirichlet kernel), row sums, M M^T, symmetry --

def _closed_form_M(n, lc):
    a = math.pi * (2 * np.arange(lc) + 1) / (2 * lc)
    b = math.pi * (2 * np.arange(n) + 1) / (2 * n)

    def D(theta):
        s = np.sin(theta / 2)
        small = np.abs(s) < 1e-14
        out = np.sin((lc - 0.5) * theta) / np.where(small, 1.0, s)
        return np.where(small, 2.0 * lc - 1.0, out)

    return (D(a[:, None] - b[None, :]) + D(a[:, None] + b[None, :])) / (2.0 * n)


@pytest.mark.parametrize("n,lc", [(508, 254), (61, 20), (96, 72), (12, 12)])
def test_closed_form_operator(n, lc):
    M = orc.compress_span(np.eye(n), lc)              # columns of M = images of unit vectors
    Mc = _closed_form_M(n, lc)
    assert np.max(np.abs(M - Mc)) < 1e-12
    assert np.allclose(M.sum(1), 1.0, atol=1e-12)                      # row sums
    assert np.allclose(M @ M.T, (lc / n) * np.eye(lc), atol=1e-12)     # scaled isometry on the kept band
    assert np.allclose(M[::-1, ::-1], M, atol=1e-12)                   # reversing x reverses y


# -- P7: library special case ---------------------------------------------------------

@pytest.mark.parametrize("n,lc,d", [(508, 254, 8), (4092, 2046, 2), (1000, 10, 3), (777, 776, 2)])
def test_against_scipy(n, lc, d):
    x = _rng(n + lc).standard_normal((n, d)) * 3.0 + 1.0
    z = scipy.fft.dct(x, type=2, norm="ortho", axis=0)
    y_ref = math.sqrt(lc / n) * scipy.fft.idct(z[:lc], type=2, norm="ortho", axis=0)
    y, zk = orc.compress_span(x, lc, return_coeffs=True)
    scale = np.abs(x).max()
    assert np.max(np.abs(zk - z[:lc])) < 1e-11 * scale * math.sqrt(n)
    assert np.max(np.abs(y - y_ref)) < 1e-11 * scale


# -- P9: amplitude over iterations (rescaling ablation appendix) ----------------------

def test_iterated_amplitude():
    rng = _rng(3)
    n, lc, d = 256, 128, 16
    # smooth signal: AR(1) with rho = 0.95
    e = rng.standard_normal((4 * n, d))
    a = np.zeros_like(e)
    a[0] = e[0] / math.sqrt(1 - 0.95 ** 2)
    for t in range(1, len(e)):
        a[t] = 0.95 * a[t - 1] + e[t]
    rms_in = math.sqrt((a ** 2).mean())
    with_rs = a[:n].copy()
    without = a[:n].copy()
    for it in range(3):
        yw = orc.compress_span(with_rs, lc, rescale=True)
        yo = orc.compress_span(without, lc, rescale=False)
        fresh = a[n + it * (n - lc): n + (it + 1) * (n - lc)]
        with_rs = np.concatenate([yw, fresh])
        without = np.concatenate([yo, fresh])
        # rescaled block keeps the signal's scale; un-rescaled grows by sqrt(n/lc) per pass
        assert 0.5 * rms_in < math.sqrt((yw ** 2).mean()) < 1.5 * rms_in
    ratio = math.sqrt((yo ** 2).mean()) / math.sqrt((yw ** 2).mean())
    assert ratio > 1.3 * math.sqrt(n / lc)      # amplified on every pass, compounding


# -- P10: sinks and tail are moved bit for bit; shapes follow Sec. 3.4 ------------------

@pytest.mark.parametrize("cur_len,window,sink,ratio", [(64, 64, 4, 0.5), (80, 64, 4, 0.5), (64, 64, 0, 0.25), (70, 50, 8, 1.0)])
def test_cache_bookkeeping(cur_len, window, sink, ratio):
    d = 6
    cache = _rng(cur_len).standard_normal((cur_len + 5, d))
    n = window - sink
    lc = orc.retained_len(n, ratio)
    out = orc.compress_head(cache, cur_len, window, sink, ratio)
    assert out.shape == (sink + lc + cur_len - window, d)
    assert out.shape[0] == orc.new_len(cur_len, window, sink, ratio)
    assert np.array_equal(out[:sink], cache[:sink])
    assert np.array_equal(out[sink + lc:], cache[window:cur_len])
    assert np.allclose(out[sink:sink + lc], orc.compress_span(cache[sink:window], lc), atol=0)
    if ratio == 1.0:
        assert np.max(np.abs(out - cache[:cur_len])) < 1e-12


def test_threads_give_same_result():
    heads = [_rng(i).standard_normal((40, 4)) for i in range(6)]
    a = orc.compress_heads(heads, 40, 40, 2, 0.5, threads=1)
    b = orc.compress_heads(heads, 40, 40, 2, 0.5, threads=4)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


# -- Dropping variant (appendix on the compression overhead): an index rule, checked on a literal example --

def test_dropping_literal_example():
    # 10 cached tokens, window 8, 2 sinks, ratio 0.5: span = tokens 2..7, Lc = 3 most recent of it = 5,6,7; tail 8,9
    cache = np.arange(10, dtype=np.float64)[:, None] * np.array([[1.0, 10.0]])
    out = orc.drop_head(cache, 10, 8, 2, 0.5)
    assert out[:, 0].tolist() == [0, 1, 5, 6, 7, 8, 9]
    assert out[:, 1].tolist() == [0, 10, 50, 60, 70, 80, 90]
    assert out.shape[0] == orc.new_len(10, 8, 2, 0.5)


# -- high-frequency retention (ablation tables): same transforms, the other end of the spectrum --------

@pytest.mark.parametrize("n,lc,d", [(8, 4, 3), (9, 4, 2), (13, 5, 4), (64, 32, 5), (30, 7, 2), (16, 15, 1)])
def test_high_band_bruteforce_matrices(n, lc, d):
    x = _rng(n * 7 + lc).standard_normal((n, d))
    Cn, Cl = _dct_matrix(n), _dct_matrix(lc)
    z_ref = (Cn @ x)[n - lc:]
    y, z = orc.compress_span_high(x, lc, return_coeffs=True)
    assert np.allclose(z, z_ref, atol=1e-13)
    assert np.allclose(y, math.sqrt(lc / n) * (Cl.T @ z_ref), atol=1e-13)
    assert np.allclose(orc.compress_span_high(x, lc, rescale=False), Cl.T @ z_ref, atol=1e-13)


@pytest.mark.parametrize("n,lc", [(508, 254), (120, 45)])
def test_high_band_pure_cosine_and_parseval(n, lc):
    j = np.arange(n)
    m = np.arange(lc)
    for t0 in (0, 1, n - lc - 1, n - lc, n - lc + 1, n - 2, n - 1):
        x = np.cos(math.pi * t0 * (2 * j + 1) / (2 * n))
        y = orc.compress_span_high(x, lc)[:, 0]
        if t0 >= n - lc:
            # basis function t0 of the n-point transform lands on index t0-(n-lc) of the Lc-point inverse;
            # index 0 of the inverse has the smaller normalisation, hence the factor sqrt(1/2) there
            s = t0 - (n - lc)
            expect = np.cos(math.pi * s * (2 * m + 1) / (2 * lc)) * (math.sqrt(0.5) if s == 0 else 1.0)
        else:
            expect = np.zeros(lc)
        assert np.max(np.abs(y - expect)) < 1e-11, t0
    x = _rng(5).standard_normal((n, 3))
    z_all = orc.dct2(x)
    y = orc.compress_span_high(x, lc)
    assert np.allclose((y ** 2).sum(0), (lc / n) * (z_all[n - lc:] ** 2).sum(0), rtol=1e-12)
    # the two bands of a half/half split carry the whole energy between them (Parseval)
    if n == 2 * lc:
        ylow = orc.compress_span(x, lc)
        assert np.allclose((y ** 2).sum(0) + (ylow ** 2).sum(0), 0.5 * (x ** 2).sum(0), rtol=1e-12)


def test_high_band_operator_properties_and_scipy():
    n, lc = 96, 40
    M = orc.compress_span_high(np.eye(n), lc)
    assert np.allclose(M @ M.T, (lc / n) * np.eye(lc), atol=1e-12)
    assert np.allclose(M[::-1, ::-1], (-1) ** (n - lc) * M, atol=1e-12)     # reversal symmetry up to a sign
    n, lc = 95, 40
    M = orc.compress_span_high(np.eye(n), lc)
    assert np.allclose(M[::-1, ::-1], -M, atol=1e-12)
    x = _rng(12).standard_normal((500, 4)) * 2.0
    z = scipy.fft.dct(x, type=2, norm="ortho", axis=0)
    ref = math.sqrt(200 / 500) * scipy.fft.idct(z[300:], type=2, norm="ortho", axis=0)
    assert np.max(np.abs(orc.compress_span_high(x, 200) - ref)) < 1e-11
    # a smooth sequence keeps almost nothing in the high band, an alternating one almost everything
    smooth = np.cos(np.linspace(0, 1, 400))[:, None]
    assert (orc.compress_span_high(smooth, 200) ** 2).sum() < 1e-6 * (smooth ** 2).sum()
    alt = ((-1.0) ** np.arange(400))[:, None]
    assert (orc.compress_span_high(alt, 200) ** 2).sum() > 0.49 * (alt ** 2).sum()


def test_high_band_cache_bookkeeping():
    cache = _rng(3).standard_normal((90, 6))
    out = orc.compress_head_high(cache, 80, 64, 4, 0.5)
    assert out.shape == (4 + 30 + 16, 6)
    assert np.array_equal(out[:4], cache[:4]) and np.array_equal(out[34:], cache[64:80])
    assert np.allclose(out[4:34], orc.compress_span_high(cache[4:64], 30), atol=0)


# -- power spectrum diagnostic (Sec. 3.1 figure; appendix on the head-wise analysis) ---------------------

def test_power_spectrum_closed_forms():
    n, d = 96, 5
    x = _rng(1).standard_normal((3, n, d))
    P = orc.power_spectrum(x)
    assert P.shape == (n,)
    # Parseval: the spectrum sums to the mean energy of a channel
    assert math.isclose(P.sum(), (x ** 2).sum() / (3 * d), rel_tol=1e-12)
    # explicit matrix
    Cn = _dct_matrix(n)
    ref = np.mean([((Cn @ x[b]) ** 2).mean(axis=1) for b in range(3)], axis=0)
    assert np.allclose(P, ref, rtol=1e-12, atol=1e-15)
    # a constant has only the DC line, n c^2; basis function t0 has a single line n/2 (n for t0 = 0)
    c = np.full((n, 2), 1.5)
    Pc = orc.power_spectrum(c)
    assert math.isclose(Pc[0], n * 1.5 ** 2, rel_tol=1e-12) and Pc[1:].max() < 1e-20
    j = np.arange(n)
    for t0 in (1, 7, n - 1):
        Pt = orc.power_spectrum(np.cos(math.pi * t0 * (2 * j + 1) / (2 * n))[:, None])
        assert math.isclose(Pt[t0], n / 2, rel_tol=1e-12)
        assert np.delete(Pt, t0).max() < 1e-20
    # scipy's transform
    assert np.allclose(P, (scipy.fft.dct(x, type=2, norm="ortho", axis=1) ** 2).mean(axis=(0, 2)), rtol=1e-11)


def test_power_spectrum_of_white_and_ar1_sequences():
    """White noise is flat at the variance; a stationary AR(1) sequence follows
    sigma_e^2 / (1 - 2 rho cos(w) + rho^2), w = pi t / n (low frequencies dominate, as Sec. 3.1 reports
    for KV states): statistical checks over many channels."""
    rng = _rng(9)
    n, d = 512, 2048
    P = orc.power_spectrum(rng.standard_normal((n, d)))
    assert abs(P.mean() - 1.0) < 0.01 and np.max(np.abs(P - 1.0)) < 0.2
    rho = 0.9
    e = rng.standard_normal((n, d))
    a = np.zeros_like(e)
    a[0] = e[0] / math.sqrt(1 - rho ** 2)
    for t in range(1, n):
        a[t] = rho * a[t - 1] + e[t]
    P = orc.power_spectrum(a)
    w = math.pi * np.arange(n) / n
    theory = 1.0 / (1 - 2 * rho * np.cos(w) + rho ** 2)
    rel = np.abs(P[4:] / theory[4:] - 1.0)            # the lowest few lines feel the finite length
    assert rel.max() < 0.2 and rel.mean() < 0.04
    assert P[: n // 2].sum() / P.sum() > 0.95          # energy kept by the lower half of the spectrum
