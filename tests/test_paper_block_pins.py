"""Pins for the oracle of the paper's self-contained 4x block (Section 3.2, Sections 4.2 / 4.3): the 8-bit float against
exact rationals, the block layout against an independent bit-level reader and writer in Python, clipping and outlier
padding against their statements.  No GPU, no HIP library."""
from __future__ import annotations

from fractions import Fraction

import numpy as np
import pytest

from helpers import half_to_fraction, py_canonical, round_fraction_to_half, stream_bits


@pytest.fixture(scope="module")
def pb():
    from oracle import paper_block as P
    return P


def _fp8_fraction(b: int) -> Fraction:
    e, mant = (b >> 3) & 15, b & 7
    mag = Fraction(mant, 512) if e == 0 else Fraction(8 + mant) * Fraction(2) ** (e - 10)
    return -mag if b & 0x80 else mag


def _fp8_nearest(v: Fraction) -> int:
    best = min(range(128), key=lambda c: (abs(_fp8_fraction(c) - abs(v)), c & 1, c))   # nearest; even code on a tie
    return best | (0x80 if v < 0 else 0)


def test_fp8_exhaustive_values_and_rounding(pb):
    vals = [_fp8_fraction(b) for b in range(256)]
    assert all(Fraction(pb.fp8_value(b)) == vals[b] for b in range(256))
    assert vals[0x7F] == 480 and vals[0x08] == Fraction(1, 64) and vals[0x01] == Fraction(1, 512) and vals[0x38] == 1
    assert all(vals[b] < vals[b + 1] for b in range(127))                     # the codes 0..127 are in increasing order
    for b in range(127):                                                      # every value, every midpoint, just off the midpoints
        lo, hi = vals[b], vals[b + 1]
        mid = (lo + hi) / 2
        assert pb.fp8_round(float(lo)) == b
        assert pb.fp8_round(float(mid)) == (b if b % 2 == 0 else b + 1)
        assert pb.fp8_round(float(mid) * (1 - 2.0 ** -40)) == b and pb.fp8_round(float(mid) * (1 + 2.0 ** -40)) == b + 1
        assert pb.fp8_round(-float(mid)) == 0x80 | (b if b % 2 == 0 else b + 1)
    assert pb.fp8_round(480.0) == 0x7F and pb.fp8_round(1e9) == 0x7F and pb.fp8_round(-70000.0) == 0xFF
    rng = np.random.default_rng(3)
    for v in rng.normal(0, 1, 300) * 10.0 ** rng.uniform(-4, 3, 300):
        assert pb.fp8_round(float(v)) == _fp8_nearest(Fraction(float(v)))


# ---------------------------------------------------------------------------------------------------------------
def _model(pb, S=3, texp=-6, seed=0, skew=2.4):
    rng = np.random.default_rng(seed)
    cent = np.sort(rng.uniform(-0.9, 0.9, (S, 15)), axis=1).astype(np.float16)
    lens = np.zeros((S, 4, 16), np.uint8)
    from oracle import oracle as O
    for p in range(S):
        for h in range(4):
            base = skew * (0.6 + 0.2 * h)
            counts = np.array([int(base ** k) + 1 for k in range(16)], np.uint64)[rng.permutation(16)]
            lens[p, h] = _lengths_2_to_8(counts)
    kp = np.array(O.limited_lengths(np.arange(1, S + 1, dtype=np.uint64) ** 2, 8), np.uint8) if S > 1 else np.array([1], np.uint8)
    m = pb.Model(cent.view(np.uint16), lens, kp, texp)
    assert pb.verify_model(m) == 0
    return m


def _lengths_2_to_8(counts):
    """Optimal code lengths in 2..8 for 16 symbols by exhaustive dynamic programming over sorted counts."""
    order = np.argsort(-counts.astype(np.int64), kind="stable")
    c = [int(counts[i]) for i in order]
    best = {}

    def go(i, last, budget):   # budget in units of 2^-8; lengths are non-decreasing along decreasing counts
        if i == 16:
            return (0, []) if budget == 0 else None
        key = (i, last, budget)
        if key in best:
            return best[key]
        res = None
        for l in range(last, 9):
            w = 1 << (8 - l)
            if w > budget:
                continue
            sub = go(i + 1, l, budget - w)
            if sub is not None:
                cost = c[i] * l + sub[0]
                if res is None or cost < res[0]:
                    res = (cost, [l] + sub[1])
        best[key] = res
        return res

    lens_sorted = go(0, 2, 256)[1]
    out = np.zeros(16, np.uint8)
    for rank, i in enumerate(order):
        out[i] = lens_sorted[rank]
    return out


def _py_decode(m, block):
    """Reads one block straight from the format statement: bit list, field by field."""
    bits = list(stream_bits(block)) + [0] * 64
    take = lambda pos, n: int("".join(str(b) for b in bits[pos:pos + n]), 2)
    s8 = take(0, 8)
    scale = _fp8_fraction(s8) * Fraction(2) ** m.texp
    h = take(8, 2)
    kp_codes = py_canonical([int(v) for v in m.kp_lens])
    p, pos = m.S - 1, 18
    for ln in range(1, 9):
        hit = [q for q in range(m.S) if m.kp_lens[q] == ln and kp_codes[q] == take(10, ln)]
        if hit:
            p, pos = hit[0], 10 + ln
            break
    lens = [int(v) for v in m.lens[p, h]]
    codes = py_canonical(lens)
    out = [Fraction(0)] * 128
    idx = []
    for i in range(128):
        sym = next(k for ln in range(2, 9) for k in range(16) if lens[k] == ln and codes[k] == take(pos, ln))
        if pos + lens[sym] > 512:
            break
        if sym == 15:
            out[i] = scale
        else:
            r = round_fraction_to_half(half_to_fraction(int(m.cent[p, sym])) * abs(scale))
            out[i] = half_to_fraction(r)
        idx.append(sym)
        pos += lens[sym]
    n_out = 0
    if len(idx) == 128:
        n_out = (512 - pos) // 15
        for j in range(n_out):
            out[take(pos, 7)] = _fp8_fraction(take(pos + 7, 8)) * Fraction(2) ** m.texp
            pos += 15
    return out, idx, n_out, p, h, s8


def _groups(seed, n, scale=0.02):
    rng = np.random.default_rng(seed)
    x = rng.normal(0, scale, (n, 128))
    x[rng.random((n, 128)) < 0.004] *= 9
    return x.astype(np.float16)


def test_decoder_against_bit_level_reader(pb):
    m = _model(pb, S=5, texp=-9, seed=1)
    x = _groups(2, 24)
    blocks = pb.encode(m, x.view(np.uint16))
    rng = np.random.default_rng(4)
    junk = rng.integers(0, 256, (24, 64), dtype=np.uint8)                       # arbitrary bytes decode the same way on both sides
    both = np.concatenate([blocks, junk])
    dec, n_coded, n_out = pb.decode(m, both)
    for g in range(both.shape[0]):
        want, idx, no, p, h, s8 = _py_decode(m, both[g])
        assert n_coded[g] == len(idx) and n_out[g] == no
        got = [half_to_fraction(int(v)) for v in dec[g]]
        assert got == want, g


def test_encoder_fields_and_decisions(pb):
    m = _model(pb, S=4, texp=-8, seed=5)
    x = _groups(6, 40)
    x[3] = 0                                        # all zero: scale byte 0, everything reconstructs to 0
    x[4, 17] = -0.75; x[4, 90] = 0.75               # the first of two equal magnitudes is the absolute maximum
    blocks = pb.encode(m, x.view(np.uint16))
    dec, n_coded, n_out = pb.decode(m, blocks)
    saw_clip = saw_pad = False
    for g in range(x.shape[0]):
        a, s8, p, h, idx = pb.quantize_group(m, x[g].view(np.uint16))
        mags = np.abs(x[g].astype(np.float64))
        assert a == int(np.argmax(mags)) and idx[a] == 15 and (np.delete(idx, a) < 15).all()
        exact_scale = Fraction(float(x[g, a])) / Fraction(2) ** m.texp
        assert s8 == _fp8_nearest(exact_scale) or (exact_scale == 0 and (s8 & 0x7F) == 0)
        out, didx, no, dp, dh, ds8 = _py_decode(m, blocks[g])
        assert (dp, dh, ds8) == (p, h, s8) and didx == list(idx[: len(didx)])
        # the codebook really is the shortest (lowest on ties)
        totals = [int(m.lens[p, k][idx].sum()) for k in range(4)]
        assert h == int(np.argmin(totals))
        # the pattern really has the least squared error over the 127 other values (exact arithmetic; clear margins only)
        sabs = abs(_fp8_fraction(s8)) * Fraction(2) ** m.texp
        sse = []
        for q in range(m.S):
            r = [half_to_fraction(round_fraction_to_half(half_to_fraction(int(c)) * sabs)) for c in m.cent[q]]
            tot = Fraction(0)
            for i in range(128):
                if i != a:
                    tot += min((Fraction(float(x[g, i])) - rk) ** 2 for rk in r)
            sse.append(tot)
        order = sorted(range(m.S), key=lambda q: sse[q])
        if sse[order[0]] == 0 or sse[order[1]] > sse[order[0]] * (1 + Fraction(1, 10 ** 5)):
            assert p == order[0]
        used = 10 + int(m.kp_lens[p]) + totals[h]
        if used > 512:
            saw_clip = True
            assert n_coded[g] < 128 and n_out[g] == 0 and not dec[g, n_coded[g]:].any()
        else:
            saw_pad = saw_pad or n_out[g] > 0
            assert n_coded[g] == 128 and n_out[g] == (512 - used) // 15
            # padded values: the largest remaining magnitudes, each stored as FP8 on the tensor scale
            rest = sorted((i for i in range(128) if i != a), key=lambda i: (-mags[i], i))[: n_out[g]]
            for i in rest:
                want = _fp8_fraction(_fp8_nearest(Fraction(float(x[g, i])) / Fraction(2) ** m.texp)) * Fraction(2) ** m.texp
                assert half_to_fraction(int(dec[g, i])) == want
            # the absolute maximum reconstructs to the FP8 scale with its sign
            assert half_to_fraction(int(dec[g, a])) == _fp8_fraction(s8) * Fraction(2) ** m.texp
    assert saw_clip and saw_pad
    assert not (dec[3] & 0x7FFF).any()                 # zeros (a negative centroid times a zero scale is -0)
    assert pb.quantize_group(m, x[4].view(np.uint16))[0] == 17


def test_clipping_is_literal_truncation(pb):
    """A model whose codes are all 8 bits except two: nothing fits; the block holds the first 512 bits of the stream."""
    cent = np.linspace(-0.9, 0.9, 15).astype(np.float16)[None]
    lens = np.full((1, 4, 16), 4, np.uint8)                                   # 10 + 1 + 512 bits: the last three values are cut
    m = pb.Model(cent.view(np.uint16), lens, np.array([1], np.uint8), -7)
    assert pb.verify_model(m) == 0
    x = _groups(9, 6)
    blocks = pb.encode(m, x.view(np.uint16))
    dec, n_coded, n_out = pb.decode(m, blocks)
    assert (n_coded == 125).all() and (n_out == 0).all() and not dec[:, 125:].any()
    for g in range(6):
        a, s8, p, h, idx = pb.quantize_group(m, x[g].view(np.uint16))
        bits = stream_bits(blocks[g])
        assert int("".join(map(str, bits[:8])), 2) == s8 and list(bits[8:11]) == [0, 0, 0]
        got = [int("".join(map(str, bits[11 + 4 * i: 15 + 4 * i])), 2) for i in range(125)]
        assert got == list(idx[:125])                                           # canonical code of index k with 16 four-bit codes is k
        assert list(bits[511:]) == [idx[125] >> 3]                              # the cut falls inside the next code: its first bit is there
    bad = pb.Model(cent.view(np.uint16), np.full((1, 4, 16), 4, np.uint8), np.array([1], np.uint8), 9)
    assert pb.verify_model(bad) == 2
    lens2 = lens.copy(); lens2[0, 1, 0] = 1
    assert pb.verify_model(pb.Model(cent.view(np.uint16), lens2, np.array([1], np.uint8), -7)) == 6
    lens2 = lens.copy(); lens2[0, 2, 0] = 5
    assert pb.verify_model(pb.Model(cent.view(np.uint16), lens2, np.array([1], np.uint8), -7)) == 7


def test_gemv_unit_vectors_pick_decoded_columns(pb):
    m = _model(pb, S=3, texp=-8, seed=7)
    rows, cols = 5, 384
    x = _groups(8, rows * 3).reshape(rows, cols)
    blocks = pb.encode(m, x.view(np.uint16))
    dec = pb.decode(m, blocks)[0].view(np.float16).reshape(rows, cols).astype(np.float64)
    for j in (0, 127, 128, 300, 383):
        e = np.zeros(cols, np.float16); e[j] = 1
        assert np.array_equal(pb.gemv(m, blocks, rows, cols, e.view(np.uint16)), dec[:, j])
    v = np.random.default_rng(1).normal(0, 1, cols).astype(np.float16)
    assert np.allclose(pb.gemv(m, blocks, rows, cols, v.view(np.uint16)), dec @ v.astype(np.float64), rtol=1e-12, atol=1e-15)
