"""Attention over the compacted cache, reference oracle -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
module; the product library never does.  Plain numpy in fp64, one query head at
a time, no blocking and no fusion.

What it computes (Sec. 3.3 Eq. 4, Sec. 3.4 Eq. 5 and the paragraph on RoPE that
closes Sec. 3.4; appendix "Compressing Key States with RoPE"):

  * the cache rows [0, cur_len) of one KV head are, in order, the sink tokens,
    the compressed rows and the tokens that came in since; the incoming token
    attends to all of them and to itself, i.e. its own key and value are the
    last row of the cache when attention runs;
  * keys are cached WITHOUT the rotary embedding; at attention time the key in
    cache row p is rotated with position p (an index inside the cache, not in
    the original sequence) and the query with its own in-cache position;
  * scores are q.k / sqrt(d), softmax over the rows, output = weights . V.

Readings where the paper is silent (stated again in the design notes):
  * rotary pairing and frequencies are those of the LLaMA models the paper
    evaluates: channel i pairs with channel i + d/2 and turns by
    pos * base**(-2 i / d)  (RoFormer, Sec. 3.2.2, with LLaMA's half-split pairing);
  * grouped-query attention maps query head h to KV head h // (Hq / Hkv).

Pins live in ``tests/test_attend_oracle_pins.py``.  Attention outputs on real
text are "parity unpinned": the paper prints none.
"""
from __future__ import annotations

import math

import numpy as np


def rope_frequencies(d: int, base: float) -> np.ndarray:
    """theta_i = base**(-2 i / d), i = 0 .. d/2 - 1."""
    if d % 2:
        raise ValueError("head_dim must be even")
    i = np.arange(d // 2, dtype=np.float64)
    return np.power(float(base), -2.0 * i / d)


def rope_rotate(x, pos, base: float) -> np.ndarray:
    """Rotate rows of x ([T, d] or [d]) by the rotary embedding at integer positions pos ([T] or scalar).

    Pair (x_i, x_{i+d/2}) turns by the angle pos * theta_i:
        out_i       = x_i cos - x_{i+d/2} sin
        out_{i+d/2} = x_{i+d/2} cos + x_i sin
    """
    x = np.asarray(x, dtype=np.float64)
    one = x.ndim == 1
    x2 = np.atleast_2d(x)
    p = np.atleast_1d(np.asarray(pos, dtype=np.float64))
    d = x2.shape[-1]
    h = d // 2
    ang = p[:, None] * rope_frequencies(d, base)[None, :]
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x2[:, :h], x2[:, h:]
    out = np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=1)
    return out[0] if one else out


def attend_decode_head(q, k, v, cur_len: int, q_pos: int | None = None, base: float = 10000.0,
                       rope: bool = True):
    """One query vector q [d] against cache rows [0, cur_len) of k, v [T, d].  Returns (out [d], lse).

    q_pos defaults to cur_len - 1: the query's own token is the last cached row.
    lse = log sum_p exp(score_p).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)[:cur_len]
    v = np.asarray(v, dtype=np.float64)[:cur_len]
    if cur_len < 1:
        raise ValueError("attention needs at least one cached row")
    d = q.shape[0]
    if q_pos is None:
        q_pos = cur_len - 1
    if rope:
        q = rope_rotate(q, q_pos, base)
        k = rope_rotate(k, np.arange(cur_len), base)
    s = (k @ q) / math.sqrt(d)
    m = s.max()
    e = np.exp(s - m)
    z = e.sum()
    out = (e / z) @ v
    return out, m + math.log(z)


def attend_decode(q, k, v, cur_len: int, q_pos: int | None = None, base: float = 10000.0,
                  rope: bool = True):
    """q [Hq, d]; k, v [Hkv, T, d] (pre-rotary keys).  Returns (out [Hq, d], lse [Hq])."""
    q = np.asarray(q, dtype=np.float64)
    hq, d = q.shape
    hkv = k.shape[0]
    if hq % hkv:
        raise ValueError("query heads must be a multiple of KV heads")
    group = hq // hkv
    out = np.zeros((hq, d))
    lse = np.zeros(hq)
    for h in range(hq):
        out[h], lse[h] = attend_decode_head(q[h], k[h // group], v[h // group], cur_len, q_pos, base, rope)
    return out, lse


def attend_prefill(q, k, v, cur_len: int, base: float = 10000.0, rope: bool = True):
    """Chunk-wise attention of Sec. 3.4 (Eq. 5): the last q_len cached rows are the tokens of the incoming
    chunk; query i sits at in-cache position p_i = cur_len - q_len + i and attends to rows [0, p_i]:
    sinks, compressed rows, the earlier tokens of its own chunk and itself.
    q [Hq, q_len, d]; k, v [Hkv, T, d] (pre-rotary keys).  Returns (out [Hq, q_len, d], lse [Hq, q_len])."""
    q = np.asarray(q, dtype=np.float64)
    hq, q_len, d = q.shape
    hkv = k.shape[0]
    if hq % hkv or q_len < 1 or q_len > cur_len:
        raise ValueError("bad shapes")
    group = hq // hkv
    out = np.zeros((hq, q_len, d))
    lse = np.zeros((hq, q_len))
    for h in range(hq):
        for i in range(q_len):
            p = cur_len - q_len + i
            out[h, i], lse[h, i] = attend_decode_head(q[h, i], k[h // group], v[h // group], p + 1, p, base, rope)
    return out, lse
