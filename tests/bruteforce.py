"""Exact-rational, per-block brute force of the DialectFP4 definitions.

A second, independent statement of the method used only to pin the oracle:
pure Python on fractions.Fraction, one block at a time, every choice made by
exhaustive search over candidates rather than by interval arithmetic.
It takes the formatbook as an argument and holds no table of its own.
"""
from fractions import Fraction


def exponent_by_search(amax):
    """Integer e with 4 <= amax / 2**e < 8, clamped to [-127, 127]; -127 for 0."""
    if amax == 0:
        return -127
    e = 0
    while amax / Fraction(2) ** e >= 8:
        e += 1
    while amax / Fraction(2) ** e < 4:
        e -= 1
    return max(-127, min(127, e))


def nearest_ties_up(s, values):
    """Position in `values` of the value nearest to s; equal distances -> larger value."""
    best = None
    for i, v in enumerate(values):
        d = abs(s - v)
        if best is None or d < best[0] or (d == best[0] and v > values[best[1]]):
            best = (d, i)
    return best[1]


def quantize_block(xs, book):
    """xs: 32 Fractions (signs given separately by the caller);
    book: 16 ascending lists of Fractions.  Returns (e, dialect, [index]*32)."""
    mags = [abs(x) for x in xs]
    e = exponent_by_search(max(mags))
    s = [m / Fraction(2) ** e for m in mags]
    smax = max(s)
    # stage 1: the pair whose shared largest value is nearest the block maximum
    pair_max = [book[2 * p][-1] for p in range(8)]
    p = nearest_ties_up(smax, pair_max)
    even, odd = book[2 * p], book[2 * p + 1]
    # stage 2: an element votes for a dialect when, among all values of the
    # pair, the nearest one is the value only that dialect has
    union = sorted(set(even) | set(odd))
    only_even = [v for v in even if v not in odd][0]
    only_odd = [v for v in odd if v not in even][0]
    votes_even = sum(1 for v in s if union[nearest_ties_up(v, union)] == only_even)
    votes_odd = sum(1 for v in s if union[nearest_ties_up(v, union)] == only_odd)
    d = 2 * p + (1 if votes_odd > votes_even else 0)
    idx = [nearest_ties_up(v, book[d]) for v in s]
    return e, d, idx


def mse_best_dialects(xs, book):
    """All dialects achieving the minimum squared error for the block (exhaustive)."""
    mags = [abs(x) for x in xs]
    e = exponent_by_search(max(mags))
    s = [m / Fraction(2) ** e for m in mags]
    errs = []
    for d in range(16):
        errs.append(sum((v - book[d][nearest_ties_up(v, book[d])]) ** 2 for v in s))
    best = min(errs)
    return [d for d in range(16) if errs[d] == best], errs


def gemm_integer_form(a_u, a_sign, a_e, w_u, w_sign, w_e):
    """Section 3.3 block MAC written with integers: for one output element,
    sum over blocks of 2**(ea+ew-2) * sum_k (+-ua)(+-uw).  Inputs are lists per
    block: half-unit magnitudes, sign bits, exponents.  Returns a Fraction."""
    total = Fraction(0)
    for ub, sb, eb, vb, tb, fb in zip(a_u, a_sign, a_e, w_u, w_sign, w_e):
        acc = 0
        for u, s, v, t in zip(ub, sb, vb, tb):
            acc += (-u if s else u) * (-v if t else v)
        total += Fraction(acc) * Fraction(2) ** (eb + fb - 2)
    return total


def e2m1_nearest_even(s, values):
    """Nearest E2M1 value; equal distances -> even position; saturating."""
    best = None
    for i, v in enumerate(values):
        d = abs(s - v)
        if best is None or d < best[0] or (d == best[0] and i % 2 == 0):
            best = (d, i)
    return best[1]
