"""Pins for the attention oracle (attention over the compacted cache with the rotary embedding
applied at read time, Sec. 3.4 Eq. 5 and its closing paragraph).  Each check uses something other
than the oracle's own formula: complex arithmetic, library softmax / attention routines, closed
forms and special cases."""
import cmath
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import attend_oracle as att


def _rng(seed=0):
    return np.random.default_rng(seed)


def _case(seed, hq, hkv, t, d, scale=1.0):
    r = _rng(seed)
    return (r.standard_normal((hq, d)) * scale, r.standard_normal((hkv, t, d)), r.standard_normal((hkv, t, d)))


# -- the rotary embedding itself ---------------------------------------------------------------

def test_rope_literal_values():
    d, base = 8, 10000.0
    th = att.rope_frequencies(d, base)
    assert th[0] == 1.0
    assert math.isclose(th[-1], base ** (-(d - 2) / d), rel_tol=1e-15)
    assert math.isclose(th[1], 0.1, rel_tol=1e-15)                      # 10000**(-2/8)
    # unit vector on channel 0 at position 1: the pair (0, d/2) turns by exactly 1 radian
    x = np.zeros(d); x[0] = 1.0
    y = att.rope_rotate(x, 1, base)
    expect = np.zeros(d); expect[0] = math.cos(1.0); expect[d // 2] = math.sin(1.0)
    assert np.allclose(y, expect, atol=1e-16)
    # unit vector on channel d/2+1 at position 7: angle 7 * 0.1, partner is channel 1
    x = np.zeros(d); x[d // 2 + 1] = 2.0
    y = att.rope_rotate(x, 7, base)
    expect = np.zeros(d); expect[1] = -2.0 * math.sin(0.7); expect[d // 2 + 1] = 2.0 * math.cos(0.7)
    assert np.allclose(y, expect, atol=1e-15)
    # position 0 is the identity
    z = _rng(1).standard_normal((3, d))
    assert np.array_equal(att.rope_rotate(z, np.zeros(3), base), z)


@pytest.mark.parametrize("d,base", [(8, 10000.0), (64, 10000.0), (128, 500000.0)])
def test_rope_is_a_rotation_and_relative(d, base):
    r = _rng(d)
    q, k = r.standard_normal(d), r.standard_normal(d)
    for a, b, t in [(5, 2, 100), (8191, 0, 1), (17, 17, 4000), (3, 40, 123456)]:
        qa, kb = att.rope_rotate(q, a, base), att.rope_rotate(k, b, base)
        assert math.isclose(np.linalg.norm(qa), np.linalg.norm(q), rel_tol=1e-13)
        # the score depends on the position difference only
        s0 = qa @ kb
        s1 = att.rope_rotate(q, a + t, base) @ att.rope_rotate(k, b + t, base)
        assert abs(s0 - s1) < 1e-9 * (1 + abs(s0))
        # complex form: pairs (i, i+d/2) as complex numbers multiplied by exp(i pos theta_i)
        th = [base ** (-2.0 * i / d) for i in range(d // 2)]
        sc = sum((complex(q[i], q[i + d // 2]).conjugate() * complex(k[i], k[i + d // 2])
                  * cmath.exp(1j * (b - a) * th[i])).real for i in range(d // 2))
        assert abs(s0 - sc) < 1e-10 * (1 + abs(s0))


# -- attention: library routines ------------------------------------------------------------------

@pytest.mark.parametrize("hq,hkv,t,d,cur", [(4, 2, 50, 16, 50), (8, 8, 33, 64, 20), (6, 2, 300, 32, 257)])
def test_against_complex_scores_and_scipy_softmax(hq, hkv, t, d, cur):
    base = 10000.0
    q, k, v = _case(hq * 100 + t, hq, hkv, t, d, scale=3.0)
    out, lse = att.attend_decode(q, k, v, cur, base=base)
    g = hq // hkv
    th = base ** (-2.0 * np.arange(d // 2) / d)
    for h in range(hq):
        kk, vv = k[h // g, :cur], v[h // g, :cur]
        zq = q[h, :d // 2] + 1j * q[h, d // 2:]
        zk = kk[:, :d // 2] + 1j * kk[:, d // 2:]
        rel = (np.arange(cur) - (cur - 1))[:, None] * th[None, :]
        s = (np.conj(zq)[None, :] * zk * np.exp(1j * rel)).real.sum(1) / math.sqrt(d)
        w = scipy.special.softmax(s)
        assert np.allclose(out[h], w @ vv, atol=1e-12)
        assert math.isclose(lse[h], scipy.special.logsumexp(s), rel_tol=1e-12, abs_tol=1e-12)


def _rotate_half_torch(x, pos, base):
    d = x.shape[-1]
    inv = base ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
    ang = pos.to(torch.float64)[:, None] * inv[None, :]
    emb = torch.cat([ang, ang], dim=-1)
    xr = torch.cat([-x[..., d // 2:], x[..., :d // 2]], dim=-1)
    return x * emb.cos() + xr * emb.sin()


@pytest.mark.parametrize("rope", [False, True])
def test_against_torch_attention(rope):
    hq, hkv, t, d, cur, base = 8, 2, 120, 32, 97, 500000.0
    q, k, v = _case(11, hq, hkv, t, d, scale=2.0)
    out, _ = att.attend_decode(q, k, v, cur, base=base, rope=rope)
    tq = torch.from_numpy(q)[:, None, :]                                  # [Hq, 1, d]
    tk = torch.from_numpy(k[:, :cur]).repeat_interleave(hq // hkv, dim=0)  # [Hq, cur, d]
    tv = torch.from_numpy(v[:, :cur]).repeat_interleave(hq // hkv, dim=0)
    if rope:
        tq = _rotate_half_torch(tq, torch.tensor([cur - 1]), base)
        tk = _rotate_half_torch(tk, torch.arange(cur), base)
    ref = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None], tv[None])[0, :, 0]
    assert np.allclose(out, ref.numpy(), atol=1e-12)


# -- attention: closed forms and special cases ------------------------------------------------------

def test_zero_keys_give_the_mean_of_values():
    q, k, v = _case(3, 4, 2, 40, 16)
    k[:] = 0.0
    out, lse = att.attend_decode(q, k, v, 31)
    for h in range(4):
        assert np.allclose(out[h], v[h // 2, :31].mean(0), atol=1e-14)
        assert math.isclose(lse[h], math.log(31), rel_tol=1e-14)


def test_single_row_cache():
    q, k, v = _case(4, 2, 2, 5, 8)
    out, lse = att.attend_decode(q, k, v, 1)
    assert np.allclose(out, v[:, 0], atol=0)
    # position 0 for both: no rotation, the score is the plain scaled dot product
    assert np.allclose(lse, (q * k[:, 0]).sum(1) / math.sqrt(8), atol=1e-14)


def test_rows_beyond_cur_len_are_not_read():
    q, k, v = _case(5, 4, 4, 30, 16)
    k2, v2 = k.copy(), v.copy()
    k2[:, 19:] = np.nan
    v2[:, 19:] = np.nan
    a, la = att.attend_decode(q, k, v, 19)
    b, lb = att.attend_decode(q, k2, v2, 19)
    assert np.array_equal(a, b) and np.array_equal(la, lb)


def test_grouped_query_mapping():
    hq, hkv, t, d = 12, 3, 20, 8
    q, k, _ = _case(6, hq, hkv, t, d)
    v = np.zeros((hkv, t, d))
    for j in range(hkv):
        v[j] = j + 1.0                      # KV head j holds the constant j+1
    out, _ = att.attend_decode(q, k, v, t)
    for h in range(hq):
        assert np.allclose(out[h], h // 4 + 1.0, atol=1e-14)


def test_in_cache_positions_are_used():
    """A query aligned with the rotated key of row p* (and scaled up) retrieves v[p*]: this fails if keys
    are left unrotated, rotated with a wrong sign, or the query position is off by one."""
    d, t, base = 64, 200, 10000.0
    r = _rng(8)
    k = r.standard_normal((1, t, d))
    v = r.standard_normal((1, t, d))
    for p_star in (0, 57, 199):
        target = att.rope_rotate(k[0, p_star], p_star, base)           # rotated key of the wanted row
        # the query is rotated by position t-1 inside the oracle: undo that rotation beforehand
        zt = target[:d // 2] + 1j * target[d // 2:]
        th = base ** (-2.0 * np.arange(d // 2) / d)
        zq = zt * np.exp(-1j * (t - 1) * th)
        q = 40.0 * np.concatenate([zq.real, zq.imag])[None, :]
        out, _ = att.attend_decode(q, k, v, t, base=base)
        assert np.max(np.abs(out[0] - v[0, p_star])) < 1e-6


def test_explicit_query_position():
    q, k, v = _case(9, 2, 1, 64, 16)
    a, _ = att.attend_decode(q, k, v, 50)
    b, _ = att.attend_decode(q, k, v, 50, q_pos=49)
    c, _ = att.attend_decode(q, k, v, 50, q_pos=48)
    assert np.array_equal(a, b)
    assert np.max(np.abs(a - c)) > 1e-3


# -- chunk-wise (prefill) attention: causal inside the chunk, everything before it visible ------------

@pytest.mark.parametrize("rope", [False, True])
def test_prefill_against_torch_causal_attention(rope):
    hq, hkv, t, d, cur, qlen, base = 4, 2, 60, 16, 50, 20, 10000.0
    r = _rng(21)
    q = r.standard_normal((hq, qlen, d)) * 2.0
    k = r.standard_normal((hkv, t, d))
    v = r.standard_normal((hkv, t, d))
    out, lse = att.attend_prefill(q, k, v, cur, base=base, rope=rope)
    tq = torch.from_numpy(q)
    tk = torch.from_numpy(k[:, :cur]).repeat_interleave(hq // hkv, dim=0)
    tv = torch.from_numpy(v[:, :cur]).repeat_interleave(hq // hkv, dim=0)
    if rope:
        tq = _rotate_half_torch(tq, torch.arange(cur - qlen, cur), base)
        tk = _rotate_half_torch(tk, torch.arange(cur), base)
    # query i may see key j iff j <= cur - qlen + i
    mask = torch.arange(cur)[None, :] <= (torch.arange(qlen)[:, None] + cur - qlen)
    ref = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None], tv[None], attn_mask=mask)[0]
    assert np.allclose(out, ref.numpy(), atol=1e-12)
    s = (tq @ tk.transpose(1, 2)) / math.sqrt(d)
    s = s.masked_fill(~mask, float("-inf"))
    assert np.allclose(lse, torch.logsumexp(s, dim=-1).numpy(), atol=1e-12)


def test_prefill_special_cases():
    hq, hkv, t, d = 2, 1, 40, 8
    r = _rng(22)
    q = r.standard_normal((hq, 7, d))
    k = r.standard_normal((hkv, t, d))
    v = r.standard_normal((hkv, t, d))
    out, lse = att.attend_prefill(q, k, v, 30)
    # the last query of the chunk is the decode case
    dout, dlse = att.attend_decode(q[:, -1], k, v, 30)
    assert np.array_equal(out[:, -1], dout) and np.array_equal(lse[:, -1], dlse)
    # a chunk that is the whole cache: the first query sees only itself
    out2, _ = att.attend_prefill(q, k, v, 7)
    assert np.allclose(out2[:, 0], v[0, 0], atol=0)
    # later rows of the chunk never influence earlier queries
    k2, v2 = k.copy(), v.copy()
    k2[:, 27:] = 9.0
    v2[:, 27:] = -9.0
    out3, _ = att.attend_prefill(q, k2, v2, 30)
    assert np.array_equal(out3[:, :4], out[:, :4]) and not np.allclose(out3[:, 4:], out[:, 4:])
