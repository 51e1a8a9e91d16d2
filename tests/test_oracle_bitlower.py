"""Pins for the oracle's extraction-position rule and bit-lowering (paper Section 4.1).

Each check compares the C oracle with something that is not the oracle: the paper's two worked
examples, the set-theoretic definition evaluated by brute force over value sets, and a closed form
written here with numpy's floor division."""
import itertools
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bitlower_worked_examples.txt")


def _examples():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        v, lo, hi, s, code, err = line.split()
        rows.append((int(v), int(lo), int(hi), int(s), int(code), float(err)))
    return rows


def test_paper_worked_examples(oracle):
    rows = _examples()
    assert len(rows) == 2
    for v, lo, hi, s, code, err in rows:
        assert oracle.shift_for_range(lo, hi) == s
        assert oracle.bitlower(v, s) == code
        assert abs(v - code * 2 ** s) / abs(v) < err
    # the two examples use the same quantisation step (0.957/29 = 0.297/9)
    assert abs(0.957 / 29 - 0.297 / 9) < 1e-4
    # the "naive" top-four-bit conversion of the paper's first example loses far more than 4 %
    assert abs(29 - oracle.bitlower(29, 4) * 16) / 29 > 0.10 - 1e-9


def test_unused_bits_are_zero_to_four(oracle):
    # Fig. 12: between zero and four unused bits -> position 4 - unused in {0..4}
    seen = {oracle.shift_for_range(-a, a) for a in range(128)}
    assert seen == {0, 1, 2, 3, 4}
    assert oracle.shift_for_range(0, 0) == 0
    assert oracle.shift_for_range(-128, 127) == 4


def test_shift_rule_is_smallest_fitting_position_all_ranges(oracle):
    # definition by brute force: smallest s such that every value of the range survives
    # "shift right by s, keep four bits" without wrapping
    for lo in range(-128, 1):
        for hi in range(0, 128):
            want = next(s for s in range(5) if -8 <= (lo >> s) and (hi >> s) <= 7)
            assert oracle.shift_for_range(lo, hi) == want, (lo, hi)


def test_or_scan_equals_range_rule(oracle):
    # the dynamic variant (OR of magnitudes, highest set bit) must give the same position as the
    # range rule on the set's extremes; asymmetric two's complement: -16 fits s=1, +16 needs s=2
    assert oracle.shift_from_values(np.array([-16], np.int8)) == 1
    assert oracle.shift_from_values(np.array([16], np.int8)) == 2
    rng = np.random.default_rng(7)
    for _ in range(2000):
        n = int(rng.integers(1, 40))
        spread = int(rng.integers(1, 128))
        v = rng.integers(-spread - 1, spread + 1, size=n).astype(np.int8)
        assert oracle.shift_from_values(v) == oracle.shift_for_range(int(v.min()), int(v.max()))
    for x in range(-128, 128):
        v = np.array([x], np.int8)
        m = x if x >= 0 else ~x
        p = m.bit_length() - 1
        assert oracle.shift_from_values(v) == max(0, p - 2)


def test_bitlower_exhaustive_closed_form(oracle):
    # all 256 8-bit values x 5 positions against clamp(floor(q / 2^s), -8, 7)
    q = np.arange(-128, 128, dtype=np.int64)
    for s in range(5):
        want = np.clip(np.floor_divide(q, 2 ** s), -8, 7)
        got = np.array([oracle.bitlower(int(v), s) for v in q])
        assert (got == want).all(), s
        # python's >> on ints is an arithmetic shift: a third formulation
        assert all(int(g) == max(-8, min(7, int(v) >> s)) for g, v in zip(got, q))


def test_bitlower_in_range_is_truncation_without_clamp(oracle):
    # values inside the range a position was chosen for never touch the clamp, and the dropped part
    # is exactly the s low bits: 0 <= q - (L << s) < 2^s, and the kept bits are a subset of q's bits
    for s in range(5):
        lim = 8 * 2 ** s
        for q in range(-lim, lim):
            if q < -128 or q > 127:
                continue
            L = oracle.bitlower(q, s)
            assert -8 <= L <= 7
            assert 0 <= q - (L << s) < 2 ** s
            assert ((L << s) & 0xFF) == (q & 0xFF & ~(2 ** s - 1))


def test_bitlower_saturates_outside_range(oracle):
    for s in range(4):
        lim = 8 * 2 ** s
        for q in range(lim, 128):
            assert oracle.bitlower(q, s) == 7
        for q in range(-128, -lim):
            assert oracle.bitlower(q, s) == -8


def test_bitlower_pack_layout(oracle):
    rng = np.random.default_rng(3)
    src = rng.integers(-128, 128, size=(5, 64)).astype(np.int8)
    sh_g = np.array([1, 3], np.uint8)
    out = oracle.bitlower_pack(src, 32, sh_g, per_row=False)
    assert out.shape == (5, 32)
    for r, c in itertools.product(range(5), range(64)):
        nib = (int(out[r, c // 2]) >> (4 * (c % 2))) & 0xF
        val = nib - 16 if nib >= 8 else nib
        assert val == max(-8, min(7, int(src[r, c]) >> int(sh_g[c // 32])))
    sh_r = rng.integers(0, 5, size=(5, 2)).astype(np.uint8)
    out = oracle.bitlower_pack(src, 32, sh_r, per_row=True)
    for r, c in itertools.product(range(5), range(64)):
        nib = (int(out[r, c // 2]) >> (4 * (c % 2))) & 0xF
        val = nib - 16 if nib >= 8 else nib
        assert val == max(-8, min(7, int(src[r, c]) >> int(sh_r[r, c // 32])))


def test_round_half_up_variant_against_exact_rationals(oracle):
    """mode 1 rounds q / 2^s to the nearest integer, ties upwards, then saturates.  The paper prints no value for it, so it
    is pinned to the textbook definition floor(x + 1/2) evaluated in exact rational arithmetic (fractions.Fraction: no
    shifts, no integer division), exhaustively, and to what follows from that definition: ties go up, it never differs
    from truncation by more than one, and it is monotone in q."""
    from fractions import Fraction
    import math
    for s in range(0, 5):
        prev = -9
        for q in range(-128, 128):
            got = oracle.bitlower(q, s, 1)
            x = Fraction(q, 2 ** s)
            want = max(-8, min(7, math.floor(x + Fraction(1, 2))))
            assert got == want, (q, s)
            assert 0 <= got - oracle.bitlower(q, s, 0) <= 1      # truncation is the floor: rounding adds 0 or 1
            assert got >= prev
            prev = got
        if s > 0:   # a tie: q = k * 2^s + 2^(s-1) rounds to k + 1 (inside the range)
            for k in range(-8, 7):
                assert oracle.bitlower(k * 2 ** s + 2 ** (s - 1), s, 1) == k + 1
                assert oracle.bitlower(k * 2 ** s + 2 ** (s - 1) - 1, s, 1) == k


def test_dynamic_act_shifts_match_range_definition(oracle):
    # the OR scan over a group == the position of the group's (min, max) range (Section 4.1), group by group,
    # and only the first G4 groups are rescanned
    rng = np.random.default_rng(11)
    gs, G = 32, 6
    X = np.zeros((50, gs * G), np.int8)
    for g, amp in enumerate((3, 9, 20, 40, 100, 127)):
        X[:, g * gs:(g + 1) * gs] = rng.integers(-amp, amp + 1, size=(50, gs))
        X[0, g * gs] = -amp          # make sure the extreme is present
    static = np.full(G, 4, np.uint8)
    for G4 in (0, 1, 3, 6):
        got = oracle.dynamic_act_shifts(X, gs, G4, static)
        for g in range(G):
            blk = X[:, g * gs:(g + 1) * gs]
            want = oracle.shift_for_range(int(blk.min()), int(blk.max())) if g < G4 else 4
            assert got[g] == want
    assert list(oracle.dynamic_act_shifts(X, gs, 6, static)) == [0, 1, 2, 3, 4, 4]
