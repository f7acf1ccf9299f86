"""Pins for the oracle's fp32 -> bf16 round-to-nearest-even (optional fp32-master input of
the encode step).  Pinned against hand-worked IEEE 754 cases, against an exact-distance
formulation in Python integers / numpy, and against torch's CPU cast over ALL 2^32 patterns."""
import os

import numpy as np
import pytest
import torch

from oracle import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "rne_cases.txt")


def _cases():
    out = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, b = line.split()[:2]
        out.append((int(a, 16), int(b, 16)))
    return out


@pytest.mark.parametrize("u,want", _cases())
def test_hand_cases(u, want):
    assert oracle.rne_bf16(u) == want


def _nearest_even_by_distance(u):
    """Exact statement: among the two bf16 neighbours (as 32-bit patterns on the magnitude
    line) take the closer one, on a tie the one whose last kept bit is 0."""
    sign, mag = u & 0x80000000, u & 0x7FFFFFFF
    if mag > 0x7F800000:
        return None
    lo = mag & ~0xFFFF
    hi = lo + 0x10000
    dl, dh = mag - lo, hi - mag
    pick = lo if dl < dh else hi if dh < dl else (lo if ((lo >> 16) & 1) == 0 else hi)
    return ((sign | pick) >> 16) & 0xFFFF


def test_against_distance_definition_sampled():
    rng = np.random.default_rng(1)
    us = list(rng.integers(0, 1 << 32, size=20000, dtype=np.uint64))
    # every tie and near-tie around a few exponents, both signs
    for base in (0x00000000, 0x00800000, 0x3F800000, 0x3C000000, 0x7F000000, 0x7F7F0000):
        for k in range(0, 0x40000, 0x8000):
            for e in (-1, 0, 1):
                v = base + k + e
                if v >= 0:
                    us += [v, v | 0x80000000]
    for u in us:
        u = int(u) & 0xFFFFFFFF
        want = _nearest_even_by_distance(u)
        if want is not None:
            assert oracle.rne_bf16(u) == want, hex(u)


def test_against_torch_cast_all_patterns():
    """Library routine as pin: torch's CPU float32 -> bfloat16 conversion, every pattern.
    NaN inputs only need to stay NaN with the sign kept (payloads are library-specific)."""
    step = 1 << 26
    for start in range(0, 1 << 32, step):
        u = np.arange(start, start + step, dtype=np.uint32)
        got = oracle.rne_bf16(u)
        f = torch.from_numpy(u.view(np.int32)).view(torch.float32)
        ref = f.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        nan = (u & 0x7FFFFFFF) > 0x7F800000
        assert np.array_equal(got[~nan], ref[~nan]), hex(start)
        if nan.any():
            g = got[nan]
            assert ((g & 0x7FFF) > 0x7F80).all()
            assert np.array_equal(g & 0x8000, (u[nan] >> 16).astype(np.uint16) & 0x8000)


def test_nan_reading_quiet_bit():
    # reading: keep the top 16 bits, set the quiet bit
    assert oracle.rne_bf16(0x7F800001) == 0x7FC0
    assert oracle.rne_bf16(0x7FA00000) == 0x7FE0
    assert oracle.rne_bf16(0xFF812345) == 0xFFC1
