"""Pins of the oracle's arithmetic payload (Sec. 4.2 states the update as W_t = W_{t-1} + dW_t).

The oracle rounds through doubles; these tests fix it against things that do not:
  * exact rational arithmetic with a brute-force search for the nearest bf16 value,
  * torch's CPU bfloat16 addition and subtraction (a library routine),
  * hand-worked cases (tests/golden/arith_cases.txt),
  * the properties the variant exists for: applying an arithmetic bucket to the old weights
    gives the new ones bit for bit, whatever the patterns, and nearby values never escape.
"""
import bisect
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def frac(bits):
    """exact value of a finite bf16 pattern"""
    s, e, m = bits >> 15, (bits >> 7) & 0xFF, bits & 0x7F
    assert e != 0xFF
    v = Fraction(m, 128) * Fraction(2) ** -126 if e == 0 else (1 + Fraction(m, 128)) * Fraction(2) ** (e - 127)
    return -v if s else v


# non-negative finite values in pattern order, then 2^128 standing for infinity (IEEE: round as if
# the exponent range were unbounded, then anything that reaches 2^128 is infinite)
_MAGS = [frac(b) for b in range(0x7F80)] + [Fraction(2) ** 128]


def nearest_brute(x):
    """bf16 pattern nearest to the rational x, ties to the even pattern."""
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    hi = bisect.bisect_left(_MAGS, a)            # first pattern with value >= a
    if hi >= len(_MAGS):
        return sign | 0x7F80
    if _MAGS[hi] == a:
        return sign | hi
    lo = hi - 1
    dl, dh = a - _MAGS[lo], _MAGS[hi] - a
    if dl < dh:
        return sign | lo
    if dh < dl:
        return sign | hi
    return sign | (lo if lo % 2 == 0 else hi)


def finite(b):
    return (b & 0x7F80) != 0x7F80


def interesting_patterns(rng, n):
    pats = [0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080, 0x0081, 0x3F80, 0xBF80, 0x3F81, 0x3F7F, 0x7F7F, 0xFF7F,
            0x7F00, 0x4000, 0x3B00, 0x3FC0, 0x0100, 0x7F80, 0xFF80, 0x7FC0, 0xFFC1, 0x7F81]
    pats += [int(x) for x in rng.integers(0, 1 << 16, n)]
    return pats


def test_nearest_against_exact_rationals():
    rng = np.random.default_rng(5)
    pats = [p for p in interesting_patterns(rng, 300) if finite(p)]
    # values between neighbouring patterns: the midpoint (a tie) and points just off it
    for p in pats:
        if not finite(p + 1) and (p & 0x7FFF) != 0x7F7F:
            continue
        a = frac(p)
        b = frac(p + 1) if finite(p + 1) else (Fraction(2) ** 128) * (-1 if p & 0x8000 else 1)
        mid = (a + b) / 2
        eps = abs(b - a) / 1024
        for x in (mid, mid - eps, mid + eps, a + eps, b - eps):
            want = nearest_brute(x)
            got = oracle.bf16_nearest(float(x))          # all of these are exact doubles
            assert Fraction(float(x)) == x
            assert got == want, (hex(p), x, hex(got), hex(want))
    for p in pats:
        assert oracle.bf16_nearest(float(frac(p))) == p or (p == 0x8000 and oracle.bf16_nearest(-0.0) == 0x8000)
    assert oracle.bf16_nearest(float("inf")) == 0x7F80 and oracle.bf16_nearest(float("-inf")) == 0xFF80
    assert oracle.bf16_nearest(float("nan")) & 0x7FFF > 0x7F80
    assert oracle.bf16_nearest(-0.0) == 0x8000


def test_add_sub_against_exact_rationals():
    rng = np.random.default_rng(6)
    pats = [p for p in interesting_patterns(rng, 160) if finite(p)]
    # pairs of nearby magnitudes (cancellation), far apart magnitudes (absorption) and anything
    near = [(p, (p + int(k)) & 0xFFFF) for p in pats for k in (-3, -1, 1, 2, 130)]
    pairs = [(a, b) for a in pats[:60] for b in pats[:60]] + near
    for a, b in pairs:
        if not (finite(a) and finite(b)):
            continue
        s, d = frac(a) + frac(b), frac(a) - frac(b)
        ws, wd = nearest_brute(s), nearest_brute(d)
        gs, gd = oracle.bf16_add(a, b), oracle.bf16_sub(a, b)
        # an exact zero result takes IEEE's sign rule (+0 unless both operands are -0 / x - x = +0),
        # which the rational search cannot see
        if s == 0:
            ws = 0x8000 if (a == 0x8000 and b == 0x8000) else 0
        if d == 0:
            wd = 0x8000 if (a == 0x8000 and b == 0x0000) else 0
        assert gs == ws, ("add", hex(a), hex(b), hex(gs), hex(ws))
        assert gd == wd, ("sub", hex(a), hex(b), hex(gd), hex(wd))


def test_add_sub_against_torch_bfloat16():
    rng = np.random.default_rng(7)
    a = rng.integers(0, 1 << 16, 200000).astype(np.uint16)
    b = rng.integers(0, 1 << 16, 200000).astype(np.uint16)
    # half of the pairs close together, where differences are small and exact
    b[::2] = (a[::2].astype(np.int32) + rng.integers(-4, 5, a[::2].size)).astype(np.uint16)
    ta = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16)
    tb = torch.from_numpy(b.view(np.int16)).view(torch.bfloat16)
    ts = (ta + tb).view(torch.int16).numpy().view(np.uint16)
    td = (ta - tb).view(torch.int16).numpy().view(np.uint16)
    for i in range(0, a.size, 7):
        gs, gd = oracle.bf16_add(int(a[i]), int(b[i])), oracle.bf16_sub(int(a[i]), int(b[i]))
        for got, want in ((gs, int(ts[i])), (gd, int(td[i]))):
            if (want & 0x7FFF) > 0x7F80:                 # NaN: any NaN pattern
                assert (got & 0x7FFF) > 0x7F80
            else:
                assert got == want, (hex(int(a[i])), hex(int(b[i])), hex(got), hex(want))


def golden_cases():
    out = []
    with open(os.path.join(HERE, "golden", "arith_cases.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                o, n, e, v = line.split()
                out.append((int(o, 16), int(n, 16), int(e), int(v, 16)))
    return out


def test_hand_worked_cases():
    cases = golden_cases()
    assert len(cases) >= 12
    for o, n, e, v in cases:
        assert oracle.arith_payload(o, n) == (bool(e), v), (hex(o), hex(n))


def test_lossless_for_any_patterns():
    """apply(old, arithmetic entries) == new bit for bit; an escape exactly where adding fails."""
    rng = np.random.default_rng(8)
    n = 60000
    old = rng.integers(0, 1 << 16, n).astype(np.uint16)
    new = rng.integers(0, 1 << 16, n).astype(np.uint16)
    new[::3] = (old[::3].astype(np.int32) + rng.integers(-3, 4, old[::3].size)).astype(np.uint16)
    changed = np.flatnonzero(old != new).astype(np.int32)
    bucket = {"idx": changed, "val": new[changed], "seg_off": np.array([0, changed.size], dtype=np.int64)}
    ab = oracle.arith_bucket(bucket, [old])
    assert np.array_equal(ab["idx"] & 0x7FFFFFFF, changed)
    dst = old.copy()
    oracle.apply_bucket_arith(ab, [dst])
    assert np.array_equal(dst, new)
    esc = ab["idx"] < 0
    assert esc.any() and (~esc).any()
    assert np.array_equal(ab["val"][esc], new[changed][esc])
    # a non-escaped entry really is the rounded difference, and adding really reproduces new
    for k in np.flatnonzero(~esc)[::17]:
        o, w = int(old[changed[k]]), int(new[changed[k]])
        assert int(ab["val"][k]) == oracle.bf16_sub(w, o)
        assert oracle.bf16_add(o, int(ab["val"][k])) == w
    # an escaped one is a case where it does not
    for k in np.flatnonzero(esc)[::17]:
        o, w = int(old[changed[k]]), int(new[changed[k]])
        d = oracle.bf16_sub(w, o)
        assert (d & 0x7FFF) > 0x7F80 or oracle.bf16_add(o, d) != w


def test_nearby_values_never_escape():
    """Sterbenz: for y/2 <= x <= 2y (same sign, finite, non-zero) x - y is exact, so it is a bf16
    value and adding it back is exact too.  The entry then carries the true difference."""
    rng = np.random.default_rng(9)
    cnt = 0
    while cnt < 3000:
        o = int(rng.integers(0x0001, 0x7F80)) | (int(rng.integers(0, 2)) << 15)
        w = (o & 0x8000) | int(rng.integers(0x0001, 0x7F80))
        fo, fw = abs(frac(o)), abs(frac(w))
        if o == w or not (fo / 2 <= fw <= 2 * fo):
            continue
        esc, v = oracle.arith_payload(o, w)
        assert not esc
        assert frac(v) == frac(w) - frac(o)
        cnt += 1


def test_apply_arith_rejects_out_of_range():
    dst = np.zeros(4, dtype=np.uint16)
    with pytest.raises(oracle.OracleError):
        oracle.apply_segment_arith(np.array([4], np.int32), np.array([1], np.uint16), dst)
    with pytest.raises(oracle.OracleError):
        oracle.apply_segment_arith(np.array([4 - 2**31], np.int32), np.array([1], np.uint16), dst)
    oracle.apply_segment_arith(np.array([3 - 2**31], np.int32), np.array([0x1234], np.uint16), dst)
    assert dst[3] == 0x1234


def test_model_round_trip_with_shards():
    """encode_model -> arithmetic buckets -> apply on the receivers' sliced old copies == sliced new."""
    from workloads import models, synth
    tensors = models.decoder(layers=1, hidden=64, q_heads=4, kv_heads=2, head_dim=16, inter=96, vocab=128)
    recs = []
    for i, t, old, new in synth.model_pairs(tensors, "bernoulli", 3, p=0.2):
        recs.append(dict(t, old=old.view(torch.int16).numpy().view(np.uint16).copy(),
                         new=new.view(torch.int16).numpy().view(np.uint16).copy()))
    tp = 2
    buckets = oracle.encode_model(recs, tp)
    for d in range(tp):
        olds = [oracle.dense_shard(r["old"], r["rows"], r["cols"], r["rule"], r.get("sections"), tp, d) for r in recs]
        news = [oracle.dense_shard(r["new"], r["rows"], r["cols"], r["rule"], r.get("sections"), tp, d) for r in recs]
        ab = oracle.arith_bucket(buckets[d], olds)
        dst = [o.copy() for o in olds]
        oracle.apply_bucket_arith(ab, dst)
        for a, b in zip(dst, news):
            assert np.array_equal(a, b)
        # small steps of a few units in the last place: almost nothing escapes
        assert (ab["idx"] < 0).mean() < 0.05
