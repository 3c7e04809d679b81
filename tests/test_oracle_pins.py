"""Pins for the fp64 CPU oracle (no GPU).

The paper prints no worked numeric example and no tensor values for this path, so the oracle is
pinned to what the mathematics fixes: brute force in exact rational arithmetic on tiny inputs,
closed forms (one key, identical keys, zero query, two tokens = logistic, constant values),
invariances (key shift, partition choice, triple order), the library routines
scipy.special.softmax / logsumexp, and exact integer counts (bit-plane values).  Each test
names the mistake it is meant to catch.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle

RNG = np.random.RandomState


def _rand(rng, shape, dtype):
    return rng.standard_normal(shape).astype(dtype)


def _case(seed, B, Hq, Hkv, N, d, dtype=np.float32):
    rng = RNG(seed)
    q = _rand(rng, (B, Hq, d), dtype)
    k = _rand(rng, (B, Hkv, N, d), dtype)
    v = _rand(rng, (B, Hkv, N, d), dtype)
    return q, k, v


# ---- exact widening of fp16 --------------------------------------------------------------------


def test_fp16_bit_patterns_widen_exactly():
    """Every finite binary16 pattern must reach the arithmetic unchanged (catches a wrong
    exponent bias, subnormal or sign handling in the oracle's own decoder).  With d = 1,
    q = 1, scale = 1 and one-token ranges, m is the key itself and O is the value itself."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = bits.view(np.float16)
    keep = np.isfinite(vals)
    vals = vals[keep]
    n = vals.size
    q = np.ones((1, 1, 1), dtype=np.float16)
    k = vals.reshape(1, 1, n, 1).copy()
    v = vals[::-1].reshape(1, 1, n, 1).copy()
    ranges = [(0, j, j + 1) for j in range(n)]
    m, l, o = oracle.attn_partial(q, k, v, [n], 1.0, ranges)
    assert np.array_equal(m[:, 0], vals.astype(np.float64))
    assert np.array_equal(o[:, 0, 0], vals[::-1].astype(np.float64))
    assert np.all(l == 1.0)


def test_bf16_bit_patterns_widen_exactly():
    """The same for every finite bfloat16 pattern; the expected values come from numpy's own
    binary32 reading of the pattern shifted into the upper half (an independent decoder)."""
    bits = np.arange(65536, dtype=np.uint32)
    vals = (bits << 16).astype(np.uint32).view(np.float32)
    keep = np.isfinite(vals)
    bits16, vals = bits[keep].astype(np.uint16), vals[keep]
    n = vals.size
    one = np.array([0x3F80], dtype=np.uint16).reshape(1, 1, 1)  # 1.0
    k = bits16.reshape(1, 1, n, 1).copy()
    v = bits16[::-1].reshape(1, 1, n, 1).copy()
    ranges = [(0, j, j + 1) for j in range(n)]
    m, l, o = oracle.attn_partial(one, k, v, [n], 1.0, ranges)
    assert np.array_equal(m[:, 0], vals.astype(np.float64))
    assert np.array_equal(o[:, 0, 0], vals[::-1].astype(np.float64))
    assert np.all(l == 1.0)
    # and the torch library conversion agrees on the same patterns
    import torch
    t = torch.from_numpy(bits16.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(t, vals)


def test_bf16_matches_the_same_values_stored_as_fp32():
    """bfloat16 inputs are exactly representable in binary32, so the oracle must give bit-identical
    results for the bf16 patterns and for their fp32 widening (catches any bf16-specific path)."""
    rng = RNG(91)
    B, Hq, Hkv, N, d = 2, 4, 2, 37, 8
    def mk(shape):
        f = rng.standard_normal(shape).astype(np.float32)
        bits = (f.view(np.uint32) >> 16).astype(np.uint16)  # truncation is fine: any bf16 pattern will do
        return bits, (bits.astype(np.uint32) << 16).view(np.float32)
    qb, qf = mk((B, Hq, d))
    kb, kf = mk((B, Hkv, N, d))
    vb, vf = mk((B, Hkv, N, d))
    seq_lens = [37, 20]
    ranges = [(0, 0, 10), (0, 10, 37), (1, 0, 20), (1, 5, 5)]
    for a, b in zip(oracle.attn_partial(qb, kb, vb, seq_lens, 0.4, ranges), oracle.attn_partial(qf, kf, vf, seq_lens, 0.4, ranges)):
        assert np.array_equal(a, b)
    for a, b in zip(oracle.attn_full(qb, kb, vb, seq_lens, 0.4), oracle.attn_full(qf, kf, vf, seq_lens, 0.4)):
        assert np.array_equal(a, b)
    assert np.array_equal(oracle.attn_logits(qb, kb, vb, seq_lens, 0.4, ranges), oracle.attn_logits(qf, kf, vf, seq_lens, 0.4, ranges))


# ---- P1 brute force in rational arithmetic -----------------------------------------------------


def _brute(q, k, v, scale, tokens):
    """softmax(scale q.k) . v over the listed tokens for one head; dot products exact."""
    qf = [Fraction(float(x)) for x in q]
    s = []
    for t in tokens:
        dot = sum(a * Fraction(float(b)) for a, b in zip(qf, k[t]))
        s.append(float(Fraction(scale) * dot))
    mx = max(s)
    w = [math.exp(x - mx) for x in s]
    den = math.fsum(w)
    out = [math.fsum(w[i] * float(v[t][c]) for i, t in enumerate(tokens)) / den for c in range(len(v[0]))]
    return out, mx, den, mx + math.log(den)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_tiny(seed, dtype):
    """All four routines against the definition evaluated independently (N <= 8, d <= 4)."""
    B, Hq, Hkv, N, d = 2, 4, 2, 8, 4
    q, k, v = _case(seed, B, Hq, Hkv, N, d, dtype)
    seq_lens = [8, 5]
    scale = 0.5
    out, lse = oracle.attn_full(q, k, v, seq_lens, scale)
    ranges = [(0, 0, 3), (0, 3, 8), (1, 0, 1), (1, 1, 5), (1, 2, 2)]
    m, l, o = oracle.attn_partial(q, k, v, seq_lens, scale, ranges)
    mo, mlse = oracle.attn_merge(m, l, o, [0, 2, 5])
    co = oracle.attn_concat(q, k, v, seq_lens, scale, ranges)
    G = Hq // Hkv
    for b in range(B):
        for h in range(Hq):
            ref, _, _, rlse = _brute(q[b, h], k[b, h // G], v[b, h // G], scale, list(range(seq_lens[b])))
            assert np.allclose(out[b, h], ref, rtol=0, atol=1e-13)
            assert abs(lse[b, h] - rlse) < 1e-13
            assert np.allclose(mo[b, h], ref, rtol=0, atol=1e-13)
            assert abs(mlse[b, h] - rlse) < 1e-13
            assert np.allclose(co[b, h], ref, rtol=0, atol=1e-13)
    for r, (b, s, e) in enumerate(ranges):
        for h in range(Hq):
            if s == e:
                assert m[r, h] == -np.inf and l[r, h] == 0 and not o[r, h].any()
                continue
            ref, mx, den, _ = _brute(q[b, h], k[b, h // G], v[b, h // G], scale, list(range(s, e)))
            assert abs(m[r, h] - mx) < 1e-14
            assert abs(l[r, h] - den) < 1e-13
            assert np.allclose(o[r, h] / l[r, h], ref, rtol=0, atol=1e-13)


# ---- P2 / P3 / P4 / P8 closed forms ------------------------------------------------------------


def test_one_key_returns_its_value():
    q, k, v = _case(3, 2, 3, 3, 1, 8)
    out, lse = oracle.attn_full(q, k, v, [1, 1], 0.7)
    assert np.array_equal(out, v[:, :, 0, :].astype(np.float64))
    m, l, o = oracle.attn_partial(q, k, v, [1, 1], 0.7, [(0, 0, 1), (1, 0, 1)])
    s0 = 0.7 * np.einsum("bhd,bhd->bh", q.astype(np.float64), k[:, :, 0].astype(np.float64))
    assert np.allclose(m, s0, rtol=0, atol=1e-15)
    assert np.all(l == 1.0)
    assert np.array_equal(o, v[:, :, 0, :].astype(np.float64))
    assert np.allclose(lse, s0, rtol=0, atol=1e-15)


def test_identical_keys_give_mean_of_values():
    rng = RNG(4)
    N, d = 37, 16
    q = _rand(rng, (1, 2, d), np.float32)
    krow = _rand(rng, (1, 2, 1, d), np.float32)
    k = np.repeat(krow, N, axis=2)
    v = _rand(rng, (1, 2, N, d), np.float32)
    out, lse = oracle.attn_full(q, k, v, [N], 0.25)
    assert np.allclose(out[0], v[0].astype(np.float64).mean(axis=1), rtol=0, atol=1e-14)
    m, l, _ = oracle.attn_partial(q, k, v, [N], 0.25, [(0, 0, N)])
    s = 0.25 * (q[0].astype(np.float64) * krow[0, :, 0].astype(np.float64)).sum(-1)
    assert np.allclose(m[0], s, atol=1e-15) and np.all(l[0] == N)
    assert np.allclose(lse[0], s + math.log(N), atol=1e-14)


def test_zero_query_counts_tokens_exactly():
    """q = 0: every logit is 0, so m = 0 and l is the range length as an exact integer
    (catches an off-by-one in range membership)."""
    _, k, v = _case(5, 1, 2, 2, 200, 8)
    q = np.zeros((1, 2, 8), dtype=np.float32)
    ranges = [(0, 0, 200), (0, 17, 118), (0, 199, 200), (0, 50, 50)]
    m, l, o = oracle.attn_partial(q, k, v, [200], 1.0, ranges)
    for r, (_, s, e) in enumerate(ranges):
        if e > s:
            assert np.all(m[r] == 0.0) and np.all(l[r] == e - s)
            assert np.allclose(o[r], v[0, :, s:e].astype(np.float64).sum(axis=1), atol=1e-12)


def _bit_count(n, c):
    """#{j in [0, n): bit c of j set}, closed form."""
    period = 1 << (c + 1)
    return (n // period) * (1 << c) + max(0, n % period - (1 << c))


def test_bitplane_values_pin_range_membership():
    """V[j][c] = bit c of j and q = 0 make O_p[c] an integer count with a closed form; any token
    wrongly included or dropped changes at least one count."""
    N, d = 1500, 16
    rng = RNG(6)
    k = _rand(rng, (1, 1, N, d), np.float16)
    j = np.arange(N)[:, None]
    c = np.arange(d)[None, :]
    v = ((j >> c) & 1).astype(np.float16).reshape(1, 1, N, d)
    q = np.zeros((1, 1, d), dtype=np.float16)
    ranges = [(0, 0, N), (0, 1, 1024), (0, 1023, 1025), (0, 777, 778), (0, 512, 1500)]
    _, l, o = oracle.attn_partial(q, k, v, [N], 0.125, ranges)
    for r, (_, s, e) in enumerate(ranges):
        want = [_bit_count(e, cc) - _bit_count(s, cc) for cc in range(d)]
        assert o[r, 0].tolist() == [float(w) for w in want]
        assert l[r, 0] == e - s


def test_constant_values_pass_through():
    """V_j = c for all j gives out = c whatever K and q are (catches a missing 1/L)."""
    q, k, _ = _case(7, 2, 4, 2, 33, 8)
    cvec = RNG(8).standard_normal(8).astype(np.float32)
    v = np.broadcast_to(cvec, (2, 2, 33, 8)).copy()
    out, _ = oracle.attn_full(q, k, v, [33, 20], 0.3)
    assert np.allclose(out, cvec.astype(np.float64), rtol=0, atol=1e-14)


# ---- P6 spike at a range boundary --------------------------------------------------------------


def test_spike_belongs_to_exactly_one_side_of_a_cut():
    """One key aligned with q gives a logit far above the rest; m of the two ranges meeting at a
    cut shows which side owns the token (catches end-inclusive or begin-exclusive ranges)."""
    N, d = 64, 8
    q, k, v = _case(9, 1, 1, 1, N, d)
    k *= 0.01
    for spike in (30, 31):
        kk = k.copy()
        kk[0, 0, spike] = 100.0 * q[0, 0] / np.dot(q[0, 0], q[0, 0])  # q.k = 100
        m, _, _ = oracle.attn_partial(q, kk, v, [N], 1.0, [(0, 0, 31), (0, 31, N)])
        owner, other = (0, 1) if spike < 31 else (1, 0)
        assert abs(m[owner, 0] - 100.0) < 1e-4
        assert m[other, 0] < 1.0


# ---- P7 two tokens = logistic ------------------------------------------------------------------


def test_two_tokens_logistic():
    q, k, v = _case(10, 1, 3, 3, 2, 8)
    scale = 0.9
    out, _ = oracle.attn_full(q, k, v, [2], scale)
    q64, k64, v64 = (x.astype(np.float64) for x in (q, k, v))
    s = scale * np.einsum("hd,hnd->hn", q64[0], k64[0])
    sig = scipy.special.expit(s[:, 0] - s[:, 1])
    want = sig[:, None] * v64[0, :, 0] + (1 - sig)[:, None] * v64[0, :, 1]
    assert np.allclose(out[0], want, rtol=0, atol=1e-14)
    m, l, o = oracle.attn_partial(q, k, v, [2], scale, [(0, 0, 1), (0, 1, 2)])
    mo, _ = oracle.attn_merge(m, l, o, [0, 2])
    assert np.allclose(mo[0], want, rtol=0, atol=1e-14)


# ---- P9 key-shift invariance -------------------------------------------------------------------


def test_key_shift_invariance():
    """k_j <- k_j + u leaves the output unchanged and moves m by scale*q.u (catches a missing
    max subtraction or a max taken over the wrong quantity).  u is chosen so the shifted keys
    are exactly representable."""
    q, k, v = _case(11, 1, 2, 2, 50, 8)
    k = np.round(k * 64) / 64
    u = (np.round(RNG(12).standard_normal(8) * 4) / 4).astype(np.float32)
    k2 = (k + u).astype(np.float32)
    scale = 0.5
    o1, _ = oracle.attn_full(q, k, v, [50], scale)
    o2, _ = oracle.attn_full(q, k2, v, [50], scale)
    assert np.allclose(o1, o2, rtol=0, atol=1e-12)
    m1, _, _ = oracle.attn_partial(q, k, v, [50], scale, [(0, 0, 50)])
    m2, _, _ = oracle.attn_partial(q, k2, v, [50], scale, [(0, 0, 50)])
    shift = scale * q[0].astype(np.float64) @ u.astype(np.float64)
    assert np.allclose(m2[0] - m1[0], shift, rtol=0, atol=1e-12)


# ---- P10 / P11 partition invariance, concat == merge -------------------------------------------


@pytest.mark.parametrize("seed", range(6))
def test_partition_invariance_and_concat_equals_merge(seed):
    """Any table that tiles [0, N_b) once -- with empty and one-token ranges, up to 64 parts --
    merges to the unsplit result; the paper-literal concat route agrees as well."""
    rng = RNG(100 + seed)
    B, Hq, Hkv, N, d = 3, 4, 2, 257, 16
    q, k, v = _case(200 + seed, B, Hq, Hkv, N, d, np.float16 if seed % 2 else np.float32)
    seq_lens = [257, 100, 1]
    ranges, gp = [], [0]
    for b, n in enumerate(seq_lens):
        parts = int(rng.choice([1, 2, 3, 8, 64]))
        cuts = sorted(rng.randint(0, n + 1, size=parts - 1).tolist())
        bounds = [0] + cuts + [n]
        rs = [(b, bounds[i], bounds[i + 1]) for i in range(parts)]
        rng.shuffle(rs)  # order inside a group must not matter
        ranges += rs
        gp.append(len(ranges))
    full, flse = oracle.attn_full(q, k, v, seq_lens, 0.25)
    m, l, o = oracle.attn_partial(q, k, v, seq_lens, 0.25, ranges)
    mo, mlse = oracle.attn_merge(m, l, o, gp)
    co = oracle.attn_concat(q, k, v, seq_lens, 0.25, ranges)
    assert np.abs(mo - full).max() < 1e-12
    assert np.abs(mlse - flse).max() < 1e-12
    assert np.abs(co - full).max() < 1e-12


# ---- P12 merge algebra -------------------------------------------------------------------------


def test_merge_algebra():
    rng = RNG(13)
    T, Hq, d = 9, 3, 8
    m = rng.standard_normal((T, Hq)) * 5
    l = rng.uniform(0.5, 20, (T, Hq))
    o = rng.standard_normal((T, Hq, d)) * l[..., None]
    flat, flse = oracle.attn_merge(m, l, o, [0, T])
    # commutativity
    perm = rng.permutation(T)
    sh, shlse = oracle.attn_merge(m[perm], l[perm], o[perm], [0, T])
    assert np.abs(sh - flat).max() < 1e-13 and np.abs(shlse - flse).max() < 1e-13
    # identity element
    m2 = np.concatenate([m[:4], np.full((2, Hq), -np.inf), m[4:]])
    l2 = np.concatenate([l[:4], np.zeros((2, Hq)), l[4:]])
    o2 = np.concatenate([o[:4], np.zeros((2, Hq, d)), o[4:]])
    idn, _ = oracle.attn_merge(m2, l2, o2, [0, T + 2])
    assert np.abs(idn - flat).max() < 1e-13
    # single triple: out = O / l, lse = m + log l
    one, onelse = oracle.attn_merge(m[:1], l[:1], o[:1], [0, 1])
    assert np.allclose(one[0], o[0] / l[0][:, None], atol=1e-15)
    assert np.allclose(onelse[0], m[0] + np.log(l[0]), atol=1e-15)
    # associativity: merge sub-groups, rebuild their triples as (lse, 1, out), merge again
    sub, sublse = oracle.attn_merge(m, l, o, [0, 3, 7, T])
    again, againlse = oracle.attn_merge(sublse, np.ones_like(sublse), sub, [0, 3])
    assert np.abs(again - flat).max() < 1e-13 and np.abs(againlse - flse).max() < 1e-13
    # triple rescaling: (m, l, O) == (m - c, l e^c, O e^c)
    c = 1.75
    resc, _ = oracle.attn_merge(m - c, l * math.exp(c), o * math.exp(c), [0, T])
    assert np.abs(resc - flat).max() < 1e-12
    # all-empty group
    z, zlse = oracle.attn_merge(np.full((2, Hq), -np.inf), np.zeros((2, Hq)), np.zeros((2, Hq, d)), [0, 2, 2])
    assert not z.any() and np.all(zlse == -np.inf)


# ---- P13 stability -----------------------------------------------------------------------------


def test_large_logits_stay_finite():
    """Logits of magnitude 1e4: no overflow; two tokens still follow the logistic form and
    identical keys still average (catches exp taken before the max is subtracted)."""
    d = 4
    q = np.full((1, 1, d), 50.0, dtype=np.float32)
    k = np.zeros((1, 1, 2, d), dtype=np.float32)
    k[0, 0, 0] = 50.0
    k[0, 0, 1] = 50.0 - 0.005  # logits 1e4 and 1e4 - 1
    v = np.array([[[[1, 0, 0, 0], [0, 1, 0, 0]]]], dtype=np.float32)
    out, lse = oracle.attn_full(q, k, v, [2], 1.0)
    s0 = float(np.dot(q[0, 0].astype(np.float64), k[0, 0, 0].astype(np.float64)))
    s1 = float(np.dot(q[0, 0].astype(np.float64), k[0, 0, 1].astype(np.float64)))
    sig = 1.0 / (1.0 + math.exp(s1 - s0))
    assert np.all(np.isfinite(out)) and np.isfinite(lse).all()
    assert abs(out[0, 0, 0] - sig) < 1e-12 and abs(out[0, 0, 1] - (1 - sig)) < 1e-12
    m, l, o = oracle.attn_partial(q, k, v, [2], 1.0, [(0, 0, 1), (0, 1, 2)])
    mo, _ = oracle.attn_merge(m, l, o, [0, 2])
    assert np.abs(mo - out).max() < 1e-12
    kneg = -k  # logits about -1e4
    outn, _ = oracle.attn_full(q, kneg, v, [2], 1.0)
    assert np.all(np.isfinite(outn)) and abs(outn[0, 0, 1] - sig) < 1e-12


# ---- P14 grouped-query mapping -----------------------------------------------------------------


def test_gqa_equals_mha_with_repeated_kv():
    """Query head h reads KV head h // G (contiguous groups); h % G would fail here."""
    B, Hq, Hkv, N, d = 2, 8, 2, 40, 8
    q, k, v = _case(14, B, Hq, Hkv, N, d)
    G = Hq // Hkv
    krep = np.repeat(k, G, axis=1)
    vrep = np.repeat(v, G, axis=1)
    o1, l1 = oracle.attn_full(q, k, v, [40, 33], 0.4)
    o2, l2 = oracle.attn_full(q, krep, vrep, [40, 33], 0.4)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    rs = [(0, 0, 11), (1, 5, 33)]
    a = oracle.attn_partial(q, k, v, [40, 33], 0.4, rs)
    b = oracle.attn_partial(q, krep, vrep, [40, 33], 0.4, rs)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


# ---- P15 library softmax / logsumexp ------------------------------------------------------------


def test_against_scipy_softmax_and_logsumexp():
    q, k, v = _case(15, 2, 4, 4, 61, 16, np.float16)
    seq_lens = [61, 17]
    scale = 0.25
    out, lse = oracle.attn_full(q, k, v, seq_lens, scale)
    q64, k64, v64 = (x.astype(np.float64) for x in (q, k, v))
    for b, n in enumerate(seq_lens):
        s = scale * np.einsum("hd,hnd->hn", q64[b], k64[b, :, :n])
        p = scipy.special.softmax(s, axis=-1)
        assert np.allclose(out[b], np.einsum("hn,hnd->hd", p, v64[b, :, :n]), rtol=0, atol=1e-13)
        assert np.allclose(lse[b], scipy.special.logsumexp(s, axis=-1), rtol=0, atol=1e-13)


# ---- layout: strides and padding ---------------------------------------------------------------


def test_strided_layout_and_padding_rows_are_ignored():
    """A token-major [B, N, Hkv, d] cache viewed as [B, Hkv, N, d] must give the same result as
    its contiguous copy, and rows past seq_lens must never be read (they hold NaN here)."""
    B, Hq, Hkv, N, d = 2, 4, 2, 30, 8
    rng = RNG(16)
    q = _rand(rng, (B, Hq, d), np.float32)
    ks = _rand(rng, (B, N, Hkv, d), np.float32)
    vs = _rand(rng, (B, N, Hkv, d), np.float32)
    seq_lens = [30, 12]
    ks[1, 12:] = np.nan
    vs[1, 12:] = np.nan
    kview, vview = ks.transpose(0, 2, 1, 3), vs.transpose(0, 2, 1, 3)
    o1, l1 = oracle.attn_full(q, kview, vview, seq_lens, 0.35)
    o2, l2 = oracle.attn_full(q, np.ascontiguousarray(kview), np.ascontiguousarray(vview), seq_lens, 0.35)
    assert np.isfinite(o1).all() and np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_empty_cache_gives_zero_output():
    q, k, v = _case(17, 2, 2, 2, 4, 4)
    out, lse = oracle.attn_full(q, k, v, [0, 4], 1.0)
    assert not out[0].any() and np.all(lse[0] == -np.inf) and np.isfinite(lse[1]).all()


def test_bad_ranges_are_rejected():
    q, k, v = _case(18, 1, 1, 1, 4, 4)
    for bad in [(0, 3, 2), (0, 0, 5), (1, 0, 1), (0, -1, 2)]:
        with pytest.raises(ValueError):
            oracle.attn_partial(q, k, v, [4], 1.0, [bad])


# ---- raw logits (the paper's wire format) ------------------------------------------------------


def test_logits_match_exact_dot_products_and_rebuild_the_attention():
    """Every exported logit equals scale * q.k evaluated in rational arithmetic (catches a wrong
    column offset, head mapping or range order), and library softmax over the concatenated
    logits times the matching V rows reproduces the unsplit output (the paper's route)."""
    B, Hq, Hkv, N, d = 2, 4, 2, 12, 4
    q, k, v = _case(21, B, Hq, Hkv, N, d, np.float16)
    seq_lens = [12, 7]
    scale = 0.5
    ranges = [(1, 2, 7), (0, 0, 5), (0, 5, 5), (0, 5, 12), (1, 0, 2)]
    lg = oracle.attn_logits(q, k, v, seq_lens, scale, ranges)
    assert lg.shape == (Hq, 5 + 5 + 0 + 7 + 2)
    G = Hq // Hkv
    col = 0
    for (b, s, e) in ranges:
        for t in range(s, e):
            for h in range(Hq):
                dot = sum(Fraction(float(a)) * Fraction(float(c)) for a, c in zip(q[b, h], k[b, h // G, t]))
                assert lg[h, col] == float(Fraction(scale) * dot)
            col += 1
    full, _ = oracle.attn_full(q, k, v, seq_lens, scale)
    v64 = v.astype(np.float64)
    # sequence 0 is covered by ranges 1..3 (columns 5..16), sequence 1 by ranges 4 then 0
    for h in range(Hq):
        p0 = scipy.special.softmax(lg[h, 5:17])
        assert np.allclose(p0 @ v64[0, h // G, :12], full[0, h], rtol=0, atol=1e-13)
        s1 = np.concatenate([lg[h, 17:19], lg[h, 0:5]])
        p1 = scipy.special.softmax(s1)
        assert np.allclose(p1 @ v64[1, h // G, :7], full[1, h], rtol=0, atol=1e-13)


# ---- Post-QK^T selection -------------------------------------------------------------------------


def test_select_matches_python_sort_and_definition():
    """Top-k by Python's sort on (-value, column) -- an independent routine -- and the triple over
    the kept tokens written out with fsum.  Catches: wrong tie-break, wrong column->token map
    across ranges, selection over the wrong group, m not the kept maximum."""
    B, Hq, Hkv, N, d = 2, 4, 2, 40, 4
    q, k, v = _case(22, B, Hq, Hkv, N, d, np.float16)
    seq_lens = [40, 25]
    ranges = [(0, 5, 20), (0, 30, 40), (1, 0, 0), (1, 3, 25)]
    gp = [0, 2, 4]
    rng = RNG(23)
    ltok = 15 + 10 + 0 + 22
    lg = np.round(rng.standard_normal((Hq, ltok)) * 4).astype(np.float32) / 4  # many exact ties
    G = Hq // Hkv
    for top_k in (1, 3, 10, 100):
        sel, m, l, o = oracle.attn_select(q, k, v, seq_lens, 0.5, ranges, lg, gp, top_k)
        for g, (c0, c1, toks, b) in enumerate([(0, 25, list(range(5, 20)) + list(range(30, 40)), 0),
                                               (25, 47, list(range(3, 25)), 1)]):
            for h in range(Hq):
                order = sorted(range(c0, c1), key=lambda c: (-float(lg[h, c]), c))[:top_k]
                kept = sorted(order)
                want_tok = [toks[c - c0] for c in kept]
                got = [t for t in sel[g, h] if t >= 0]
                assert got == want_tok
                assert list(sel[g, h][len(got):]) == [-1] * (top_k - len(got))
                mx = max(float(lg[h, c]) for c in kept)
                w = [math.exp(float(lg[h, c]) - mx) for c in kept]
                assert m[g, h] == mx and abs(l[g, h] - math.fsum(w)) < 1e-13
                for cc in range(d):
                    ref = math.fsum(wi * float(v[b, h // G, t, cc]) for wi, t in zip(w, want_tok))
                    assert abs(o[g, h, cc] - ref) < 1e-13


def test_select_everything_equals_partial_and_select_one_is_argmax():
    """top_k >= group size keeps every token: with the oracle's own logits it reproduces the
    partial statistics of the group's ranges merged; top_k = 1 returns the V row of the argmax."""
    B, Hq, Hkv, N, d = 1, 2, 1, 30, 8
    q, k, v = _case(24, B, Hq, Hkv, N, d)
    ranges = [(0, 0, 12), (0, 12, 30)]
    lg64 = oracle.attn_logits(q, k, v, [30], 0.3, ranges)
    lg = lg64.astype(np.float32)
    sel, m, l, o = oracle.attn_select(q, k, v, [30], 0.3, ranges, lg, [0, 2], 64)
    full, lse = oracle.attn_full(q, k, v, [30], 0.3)
    assert [list(sel[0, h][:30]) for h in range(Hq)] == [list(range(30))] * Hq
    assert np.abs(o[0] / l[0][:, None] - full[0]).max() < 1e-6  # fp32 rounding of the logits
    assert np.abs(m[0] + np.log(l[0]) - lse[0]).max() < 1e-6
    sel1, m1, l1, o1 = oracle.attn_select(q, k, v, [30], 0.3, ranges, lg, [0, 2], 1)
    for h in range(Hq):
        j = int(np.argmax(lg[h]))
        assert sel1[0, h, 0] == j and l1[0, h] == 1.0 and m1[0, h] == float(lg[h, j])
        assert np.array_equal(o1[0, h], v[0, 0, j].astype(np.float64))


# ---- statistics over a listed token set --------------------------------------------------------


def _lists(rng, G, Hq, max_k, seq_len_of_group, pad_frac=0.3, dup=True):
    idx = np.full((G, Hq, max_k), -1, dtype=np.int32)
    for g in range(G):
        for h in range(Hq):
            n = seq_len_of_group[g]
            row = rng.randint(0, n, size=max_k) if dup else rng.permutation(n)[:max_k]
            row = np.asarray(row, dtype=np.int32)
            if row.size < max_k:
                row = np.concatenate([row, np.full(max_k - row.size, -1, np.int32)])
            row[rng.random_sample(max_k) < pad_frac] = -1 - rng.randint(0, 5)  # any negative value pads
            idx[g, h] = row
    return idx


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_gather_brute_force_with_duplicates_padding_and_gqa(dtype):
    """Listed-token statistics against the definition in rational arithmetic.  Catches: a list
    read for the wrong (group, head), the wrong sequence or KV head behind a group, padding that
    is counted, a duplicate that is dropped, m taken over the wrong set."""
    B, Hq, Hkv, N, d = 3, 4, 2, 9, 4
    q, k, v = _case(31, B, Hq, Hkv, N, d, dtype)
    seq_lens = [9, 4, 7]
    group_seq = [2, 0, 0, 1]
    rng = RNG(32)
    idx = _lists(rng, 4, Hq, 6, [seq_lens[b] for b in group_seq])
    idx[1, 2] = -1  # a list without tokens
    m, l, o = oracle.attn_gather(q, k, v, seq_lens, 0.5, group_seq, idx)
    G = Hq // Hkv
    for g, b in enumerate(group_seq):
        for h in range(Hq):
            toks = [int(t) for t in idx[g, h] if t >= 0]
            if not toks:
                assert m[g, h] == -np.inf and l[g, h] == 0 and not o[g, h].any()
                continue
            ref, mx, den, _ = _brute(q[b, h], k[b, h // G], v[b, h // G], 0.5, toks)
            assert abs(m[g, h] - mx) < 1e-14
            assert abs(l[g, h] - den) < 1e-13
            assert np.allclose(o[g, h] / l[g, h], ref, rtol=0, atol=1e-13)


def test_gather_zero_query_counts_listings_and_bitplanes_exactly():
    """q = 0: l is the number of listings (duplicates included) and, with V[t][c] = bit c of t,
    O[c] is the number of listed tokens whose bit c is set -- exact integers that pin which rows
    were read."""
    B, Hq, Hkv, N, d = 2, 2, 1, 300, 16
    q = np.zeros((B, Hq, d), np.float16)
    k = _rand(RNG(33), (B, Hkv, N, d), np.float16)
    t = np.arange(N)
    v = ((t[:, None] >> np.arange(d)[None, :]) & 1).astype(np.float16)
    v = np.broadcast_to(v, (B, Hkv, N, d)).copy()
    idx = _lists(RNG(34), 2, Hq, 50, [300, 200])
    m, l, o = oracle.attn_gather(q, k, v, [300, 200], 0.25, [0, 1], idx)
    for g in range(2):
        for h in range(Hq):
            toks = idx[g, h][idx[g, h] >= 0]
            assert m[g, h] == 0.0 and l[g, h] == toks.size
            want = ((toks[:, None] >> np.arange(d)[None, :]) & 1).sum(axis=0)
            assert np.array_equal(o[g, h], want.astype(np.float64))


def test_gather_of_a_whole_range_equals_partial_and_order_is_free():
    """The list [begin, end) in any order gives the range's statistics; one listed token gives
    (s, 1, V); listing every token twice doubles l and O and leaves m and O/l alone."""
    B, Hq, Hkv, N, d = 1, 4, 2, 64, 8
    q, k, v = _case(35, B, Hq, Hkv, N, d, np.float16)
    pm, pl, po = oracle.attn_partial(q, k, v, [64], 0.3, [(0, 10, 50)])
    rng = RNG(36)
    idx = np.stack([rng.permutation(np.arange(10, 50)) for _ in range(Hq)]).astype(np.int32)[None]
    m, l, o = oracle.attn_gather(q, k, v, [64], 0.3, [0], idx)
    assert np.array_equal(m, pm)
    assert np.abs(l - pl).max() < 1e-12 and np.abs(o - po).max() < 1e-12
    m2, l2, o2 = oracle.attn_gather(q, k, v, [64], 0.3, [0], np.concatenate([idx, idx[:, :, ::-1]], axis=2))
    assert np.array_equal(m2, pm)
    assert np.abs(l2 - 2 * pl).max() < 1e-12 and np.abs(o2 - 2 * po).max() < 1e-12
    one = np.full((1, Hq, 3), -1, np.int32)
    one[0, :, 1] = [7, 0, 63, 7]
    m1, l1, o1 = oracle.attn_gather(q, k, v, [64], 0.3, [0], one)
    lg = oracle.attn_logits(q, k, v, [64], 0.3, [(0, 0, 64)])
    for h in range(Hq):
        tkn = one[0, h, 1]
        assert m1[0, h] == lg[h, tkn] and l1[0, h] == 1.0
        assert np.array_equal(o1[0, h], v[0, h // 2, tkn].astype(np.float64))


def test_gather_over_a_selection_reproduces_the_selection_triple():
    """The kept-token list that the Post-QK^T selection writes, evaluated by the listed-token
    routine with the same query, gives the selection's own triple (up to the fp32 rounding of the
    logits the selection was handed)."""
    B, Hq, Hkv, N, d = 2, 4, 4, 80, 8
    q, k, v = _case(37, B, Hq, Hkv, N, d, np.float16)
    seq_lens = [80, 60]
    ranges = [(0, 0, 30), (0, 40, 80), (1, 5, 60)]
    gp = [0, 2, 3]
    lg = oracle.attn_logits(q, k, v, seq_lens, 0.35, ranges).astype(np.float32)
    sel, sm, sl, so = oracle.attn_select(q, k, v, seq_lens, 0.35, ranges, lg, gp, 12)
    m, l, o = oracle.attn_gather(q, k, v, seq_lens, 0.35, [0, 1], sel)
    assert np.abs(m - sm).max() < 1e-6
    assert np.abs(o / l[..., None] - so / sl[..., None]).max() < 1e-6
    assert np.abs(m + np.log(l) - sm - np.log(sl)).max() < 1e-6


def test_gather_rejects_tokens_past_the_sequence_end():
    q, k, v = _case(38, 2, 2, 2, 10, 4)
    idx = np.zeros((1, 2, 3), np.int32)
    idx[0, 1, 2] = 6
    with pytest.raises(ValueError):
        oracle.attn_gather(q, k, v, [10, 6], 1.0, [1], idx)
    oracle.attn_gather(q, k, v, [10, 6], 1.0, [0], idx)
    with pytest.raises(ValueError):
        oracle.attn_gather(q, k, v, [10, 6], 1.0, [2], idx)


def test_topk_is_the_definition_on_exactly_representable_logits():
    """Dyadic inputs and a power-of-two scale make every logit exact in fp32 and in fp64 alike,
    so the composed routine must keep exactly the k largest q.k (ties to the earlier token) found
    by integer arithmetic, and its triple is the listed-token routine over that set."""
    B, Hq, Hkv, N, d = 2, 4, 2, 50, 8
    rng = RNG(41)
    q = (rng.randint(-8, 9, size=(B, Hq, d)) / 4).astype(np.float16)
    k = (rng.randint(-8, 9, size=(B, Hkv, N, d)) / 4).astype(np.float16)
    v = _rand(rng, (B, Hkv, N, d), np.float16)
    seq_lens = [50, 30]
    ranges = [(0, 0, 20), (0, 25, 50), (1, 2, 30)]
    gp = [0, 2, 3]
    toks = [list(range(0, 20)) + list(range(25, 50)), list(range(2, 30))]
    for top_k in (1, 6, 40, 64):
        sel, m, l, o, lg = oracle.attn_topk(q, k, v, seq_lens, 0.25, ranges, gp, top_k)
        gm, gl, go = oracle.attn_gather(q, k, v, seq_lens, 0.25, [0, 1], sel)
        assert np.array_equal(m, gm) and np.abs(l - gl).max() < 1e-12 and np.abs(o - go).max() < 1e-12
        for g in range(2):
            for h in range(Hq):
                # integer dot products: 16 q.k, exact
                dots = [(int(np.round(16 * float(np.dot(q[g, h].astype(np.float64), k[g, h // 2, t].astype(np.float64))))), i)
                        for i, t in enumerate(toks[g])]
                best = sorted(dots, key=lambda x: (-x[0], x[1]))[:top_k]
                want = sorted(toks[g][i] for _, i in best)
                assert [t for t in sel[g, h] if t >= 0] == want
                assert m[g, h] == best[0][0] / 64.0  # scale 1/4 of (16 q.k)/16
