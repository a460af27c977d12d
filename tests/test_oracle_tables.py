"""Pins for the oracle's table construction (normalise, spread, decode table, encode map).

Each check is against something fixed by the paper or by the mathematics of tANS, not
against the oracle's own formulas:
  * the spread against an exact-rational sort written with fractions.Fraction,
  * the decode table against the counting definition of the ANS sub-state,
  * the interval tiling that makes "newX + bits" a log2(l)-bit addition (Sec. II-A),
  * the zero-bit transitions that let tANS go below 1 bit/symbol (Sec. II-A),
  * the 3*l-byte table and the 192-byte example printed in Sec. II-A.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _freq_cases():
    rng = np.random.default_rng(20240623)
    cases = []
    for R in (2, 3, 4, 6, 8, 10, 12):
        L = 1 << R
        for trial in range(4):
            A = int(rng.integers(1, min(L, 40) + 1))
            cuts = np.sort(rng.choice(np.arange(1, L), size=A - 1, replace=False)) if A > 1 else np.array([], int)
            f = np.diff(np.concatenate(([0], cuts, [L]))).astype(np.uint32)
            syms = np.sort(rng.choice(256, size=A, replace=False))
            full = np.zeros(256, dtype=np.uint32)
            full[syms] = f
            cases.append((R, full))
        # heavily peaked and single-symbol cases
        full = np.zeros(256, dtype=np.uint32)
        full[5] = L
        cases.append((R, full))
        if L >= 4:
            full = np.zeros(256, dtype=np.uint32)
            full[0] = 1
            full[200] = L - 2
            full[255] = 1
            cases.append((R, full))
    return cases


CASES = _freq_cases()


@pytest.mark.parametrize("R,f", [c for c in CASES if c[0] <= 8])
def test_spread_matches_exact_rational_sort(orc, R, f):
    """State X holds the pair of rank X when (symbol, occurrence) pairs are ordered by the
    exact fraction (2i+1)/(2 f_s), ties to the smaller symbol."""
    pairs = [(Fraction(2 * i + 1, 2 * int(f[s])), s) for s in range(256) for i in range(int(f[s]))]
    pairs.sort()
    expected = np.array([s for _, s in pairs], dtype=np.uint8)
    assert np.array_equal(orc.spread(f, R), expected)


@pytest.mark.parametrize("R,f", CASES)
def test_spread_has_each_symbol_f_times(orc, R, f):
    sp = orc.spread(f, R)
    assert np.array_equal(np.bincount(sp, minlength=256), f)


@pytest.mark.parametrize("R,f", [c for c in CASES if c[0] <= 8])
def test_decode_table_matches_counting_definition(orc, R, f):
    """ANS sub-state by definition: x_s = f_s + #{states below x that carry the same symbol};
    the entry must renormalise x_s into [L, 2L) by appending nb bits."""
    L = 1 << R
    sym, nb, newX = orc.decode_table(f, R)
    sp = orc.spread(f, R)
    assert np.array_equal(sym, sp)
    for X in range(L):
        s = sp[X]
        xs = int(f[s]) + int(np.count_nonzero(sp[:X] == s))
        n = 0
        while (xs << n) < L:
            n += 1
        assert (xs << n) < 2 * L
        assert nb[X] == n
        assert newX[X] == (xs << n) - L


@pytest.mark.parametrize("R,f", CASES)
def test_intervals_tile_state_space(orc, R, f):
    """For every symbol the intervals [newX, newX + 2^nb) of its states tile [0, L) exactly,
    so the next state newX + bits never leaves [0, L): the adder is log2(l) bits wide
    (Sec. II-A: 6-bit adder for 64 states)."""
    L = 1 << R
    sym, nb, newX = orc.decode_table(f, R)
    assert int((newX.astype(np.int64) + (1 << nb.astype(np.int64)) - 1).max()) <= L - 1
    for s in np.nonzero(f)[0]:
        cover = np.zeros(L, dtype=np.int32)
        for X in np.nonzero(sym == s)[0]:
            cover[int(newX[X]):int(newX[X]) + (1 << int(nb[X]))] += 1
        assert np.all(cover == 1), f"symbol {s} intervals do not tile"
    # newX is a multiple of 2^nb, so the addition is also a bitwise OR
    assert np.all((newX.astype(np.int64) & ((1 << nb.astype(np.int64)) - 1)) == 0)


@pytest.mark.parametrize("R,f", CASES)
def test_zero_bit_transitions(orc, R, f):
    """Empty-label transitions (Sec. II-A) exist exactly for a symbol with f_s > L/2; along a
    chain of them the state strictly decreases (so chains end) unless f_s == L."""
    L = 1 << R
    sym, nb, newX = orc.decode_table(f, R)
    zero = nb == 0
    big = np.nonzero(f > L // 2)[0]
    if len(big) == 0:
        assert not zero.any()
        return
    s = big[0]
    assert zero.any()
    assert np.all(sym[zero] == s)
    assert int(zero.sum()) == 2 * int(f[s]) - L
    if f[s] < L:
        X = np.nonzero(zero)[0]
        assert np.all(newX[X] < X)
    else:
        assert np.array_equal(newX, np.arange(L))


@pytest.mark.parametrize("R,f", CASES)
def test_encode_map_inverts_decode_table(orc, R, f):
    """Every (state, symbol) pair: one encoder transition followed by one decoder transition
    returns to the same state and the same symbol, consuming exactly the emitted bits."""
    L = 1 << R
    sym, nb, newX = orc.decode_table(f, R)
    enc, base = orc.encode_map(f, R)
    for s in np.nonzero(f)[0]:
        fs = int(f[s])
        x = np.arange(L, 2 * L, dtype=np.int64)
        n = np.zeros(L, dtype=np.int64)
        for _ in range(R + 1):
            n = np.where((x >> n) >= 2 * fs, n + 1, n)
        assert np.all(((x >> n) >= fs) & ((x >> n) < 2 * fs))
        bits = x & ((1 << n) - 1)
        Xn = enc[base[s] + ((x >> n) - fs)].astype(np.int64)
        assert np.all(sym[Xn] == s)
        assert np.all(nb[Xn] == n)
        assert np.all(newX[Xn].astype(np.int64) + bits == x - L)


def test_lut_is_3l_bytes_and_paper_example(orc):
    """Sec. II-A: the LUT takes 3*l bytes; 64 states / 4-bit symbols / 6-bit adder -> 192 bytes."""
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "paper_sec2a_lut_bytes.txt"))
            if ln.strip() and not ln.startswith("#")]
    for states, symbol_bits, adder_bits, table_bytes in [[int(v) for v in r] for r in rows]:
        R = states.bit_length() - 1
        assert 1 << R == states and adder_bits == R
        A = 1 << symbol_bits
        counts = (np.arange(A, 0, -1) ** 2).astype(np.uint64)
        f = orc.normalize(counts, R)
        lut = orc.decode_table_bytes(f, R)
        assert len(lut) == table_bytes == 3 * states
        sym, nb, newX = orc.decode_table(f, R)
        assert np.array_equal(lut[0::3], sym) and np.array_equal(lut[1::3], nb)
        assert np.array_equal(lut[2::3], newX.astype(np.uint8))
        assert int(sym.max()) < A
        assert int((newX.astype(np.int64) + (1 << nb.astype(np.int64)) - 1).max()) < (1 << adder_bits)
    for R in (6, 7, 8):
        f = orc.normalize(np.array([900, 50, 30, 20], dtype=np.uint64), R)
        assert len(orc.decode_table_bytes(f, R)) == 3 << R


def test_normalize_properties(orc):
    rng = np.random.default_rng(7)
    for R in (4, 6, 8, 10, 12):
        L = 1 << R
        for _ in range(20):
            A = int(rng.integers(1, min(L, 256) + 1))
            counts = np.zeros(256, dtype=np.uint64)
            idx = rng.choice(256, size=A, replace=False)
            counts[idx] = rng.integers(1, 10 ** int(rng.integers(1, 8)), size=A).astype(np.uint64)
            f = orc.normalize(counts, R)
            assert int(f.sum()) == L
            assert np.array_equal(f > 0, counts > 0)
            # never above floor(c L / n) except for the bump to one and for the symbol that
            # takes the surplus; order of the counts is kept up to one unit
            n = int(counts.sum())
            fl = np.maximum((counts.astype(object) * L) // n, (counts > 0).astype(object)).astype(np.int64)
            surplus = L - int(fl.sum())
            if surplus >= 0:
                diff = f.astype(np.int64) - fl
                assert int(np.count_nonzero(diff)) <= 1 and int(diff.sum()) == surplus
                if surplus:
                    assert int(np.argmax(diff)) == int(np.argmax(fl))
            else:
                assert np.all(f.astype(np.int64) <= fl)
                cut = np.nonzero(f.astype(np.int64) < fl)[0]
                # only the largest ones were cut, and they end up level with each other
                assert int(f[cut].min()) >= int(np.delete(f, cut).max(initial=0)) - 1
    with pytest.raises(ValueError):
        orc.normalize(np.zeros(256, dtype=np.uint64), 8)
    with pytest.raises(ValueError):
        orc.normalize(np.ones(256, dtype=np.uint64), 6)      # 256 present symbols, 64 states


def test_bad_frequencies_rejected(orc):
    f = np.zeros(256, dtype=np.uint32)
    f[0] = 100
    with pytest.raises(ValueError):
        orc.spread(f, 8)
    with pytest.raises(ValueError):
        orc.decode_table(f, 8)
