"""Pins for the CPU oracle: paper text, closed forms, brute force, invariants.

None of these tests touches the GPU or the HIP library.  Each pins a part of
oracle/ to something other than itself, so that a dropped term, a wrong sign,
a wrong tie rule or a wrong table row fails at least one of them.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import dfp4_oracle as O
from oracle import mxfp4_oracle as MX
from tests import bruteforce as BF


def _golden(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return json.load(f)


def _bf16(x):
    """Round a float array to bf16 and return it as exact float64."""
    return torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


def _block(values, scale_log2=0):
    x = np.zeros((1, 32))
    x[0, :len(values)] = values
    return np.ldexp(x, scale_log2)


def _nibbles(codes):
    return O.unpack_codes(codes)


BOOK_FR = [[Fraction(int(u), 2) for u in row] for row in O.FORMATBOOK_HALF_UNITS]


# --------------------------------------------------------------------------
# formatbook: what the paper's text fixes
# --------------------------------------------------------------------------
def test_formatbook_rows_printed_in_the_paper(golden_dir):
    g = _golden(golden_dir, "paper_text_pins.json")
    assert list(O.FORMATBOOK[4]) == g["dialect4_values"]["values"]
    d = g["dialect5_differs"]
    only4 = set(O.FORMATBOOK[4]) - set(O.FORMATBOOK[5])
    only5 = set(O.FORMATBOOK[5]) - set(O.FORMATBOOK[4])
    assert only4 == {d["dialect4_only"]} and only5 == {d["dialect5_only"]}
    assert O.FORMATBOOK[4][-1] == O.FORMATBOOK[5][-1] == d["shared_max"]


def test_formatbook_structure(golden_dir):
    g = _golden(golden_dir, "paper_text_pins.json")
    hu = O.FORMATBOOK_HALF_UNITS
    assert hu.shape == (16, 8)
    assert (hu >= 0).all() and (hu <= 15).all()                 # 4-bit unsigned, unit 0.5
    assert (np.diff(hu, axis=1) > 0).all()                      # 8 distinct ascending magnitudes
    assert (hu[:, 0] == 0).all()
    maxima = sorted(set(O.FORMATBOOK[:, -1]))
    assert maxima == g["pair_maxima"]["values"]                 # every maximum in [4, 8) covered
    for p in range(8):
        e, o = set(hu[2 * p]), set(hu[2 * p + 1])
        assert hu[2 * p, -1] == hu[2 * p + 1, -1] == 15 - p     # pair shares max, descending
        assert len(e - o) == 1 and len(o - e) == 1              # differ in exactly one value
        assert max(e - o) > max(o - e)                          # even dialect: larger value (App. B)
    assert list(O.FORMATBOOK[7]) == g["fp4_e2m1"]["values"]     # base format is in the book
    base6 = g["fp4_e2m1"]["values"][:6]
    same = sum(list(O.FORMATBOOK[d][:6]) == base6 for d in range(16))
    assert same >= 15                                           # "most" small values follow FP4


def test_beneficial_range_printed_in_the_paper(golden_dir):
    g = _golden(golden_dir, "paper_text_pins.json")["dialect4_beneficial_range"]
    assert O.beneficial_range(4) == (g["lo"], g["hi"])
    # the partner's range ends where dialect 4's begins (midpoint of 4.0 and 5.0)
    assert O.beneficial_range(5) == (3.5, 4.5)


def test_beneficial_range_is_voronoi_cell_by_brute_force():
    # literal definition: s is inside iff its nearest value among all values
    # of the pair is the value only this dialect has
    for d in range(16):
        lo, hi = O.beneficial_range(d)
        even, odd = BOOK_FR[d & ~1], BOOK_FR[d | 1]
        union = sorted(set(even) | set(odd))
        mine = [v for v in BOOK_FR[d] if v not in BOOK_FR[d ^ 1]][0]
        for q in range(0, 8 * 16):                              # s on a 1/16 grid over [0, 8)
            s = Fraction(q, 16)
            inside = union[BF.nearest_ties_up(s, union)] == mine
            assert inside == (lo <= float(s) < hi), (d, s)


# --------------------------------------------------------------------------
# preprocessing
# --------------------------------------------------------------------------
def test_shared_exponent_closed_form(golden_dir):
    g = _golden(golden_dir, "paper_text_pins.json")["scaled_range"]
    for k in range(-120, 120):
        for m in (1.0, 1.0078125, 1.5, 1.9921875):            # bf16 mantissas incl. extremes
            amax = m * 2.0 ** k
            e = int(O.shared_exponent(amax))
            assert e == k - 2
            assert g["block_max_lo"] <= amax / 2.0 ** e < g["hi_exclusive"]
    assert int(O.shared_exponent(0.0)) == -127
    # clamp at the bottom: bf16 subnormals and the two smallest binades
    assert int(O.shared_exponent(2.0 ** -133)) == -127
    assert int(O.shared_exponent(2.0 ** -126)) == -127
    assert int(O.shared_exponent(2.0 ** -125)) == -127
    assert int(O.shared_exponent(2.0 ** -124)) == -126


def test_shared_exponent_vs_search():
    rng = np.random.default_rng(11)
    vals = _bf16(np.exp(rng.uniform(-80, 80, 500)))
    for v in vals:
        assert int(O.shared_exponent(v)) == BF.exponent_by_search(Fraction(v))


# --------------------------------------------------------------------------
# element rounding
# --------------------------------------------------------------------------
def test_element_example_printed_in_the_paper(golden_dir):
    g = _golden(golden_dir, "paper_text_pins.json")
    ex = g["element_example"]
    assert int(ex["mag_trunc_bits"], 2) / 4.0 == ex["scaled_value"]
    idx = O.nearest_index(np.array([[ex["scaled_value"]] * 32]), np.array([ex["dialect"]]))
    assert int(idx[0, 0]) == ex["index"]
    assert O.FORMATBOOK[ex["dialect"]][ex["index"]] == ex["quantized_value"]
    ri = g["rounding_interval"]
    t = np.arange(32)
    idx = O.nearest_index((t / 4.0)[None, :], np.array([ri["dialect"]]))[0]
    hit = O.FORMATBOOK[ri["dialect"]][idx] == ri["quantized_value"]
    assert list(np.nonzero(hit)[0]) == list(range(ri["t_first"], ri["t_last"] + 1))


def test_nearest_index_vs_exact_brute_force_all_dialects():
    # every dialect, s on a 1/32 grid (finer than the 5-bit magnitude, includes all ties)
    q = np.arange(0, 8 * 32)
    s = (q / 32.0).reshape(-1, 32)
    for d in range(16):
        got = O.nearest_index(s, np.full(s.shape[0], d)).reshape(-1)
        want = [BF.nearest_ties_up(Fraction(int(i), 32), BOOK_FR[d]) for i in q]
        assert list(got) == want, d


def test_five_bit_truncation_gives_the_same_index():
    # Section 3.2 preprocessing truncates to 2 fractional bits before rounding;
    # thresholds are multiples of 0.25, so truncation changes nothing, and the
    # index is the count of thresholds u[j-1]+u[j] (quarter-units) not above t
    rng = np.random.default_rng(5)
    s = _bf16(rng.uniform(0, 8, (64, 32)))
    s = np.minimum(s, 7.96875)
    for d in range(16):
        dd = np.full(s.shape[0], d)
        full = O.nearest_index(s, dd)
        trunc = O.nearest_index(np.floor(4 * s) / 4, dd)
        assert (full == trunc).all()
        hu = O.FORMATBOOK_HALF_UNITS[d]
        thr = hu[:-1] + hu[1:]
        count = (np.floor(4 * s)[:, :, None] >= thr).sum(axis=2)
        assert (full == count).all()


# --------------------------------------------------------------------------
# whole blocks
# --------------------------------------------------------------------------
def test_handworked_blocks(golden_dir):
    g = _golden(golden_dir, "handworked_blocks.json")
    for b in g["blocks"]:
        k = b.get("x_scale_log2", 0)
        x = _block(b["x"], k)
        codes, dialect, expo = O.dfp4_quantize(x)
        nib = _nibbles(codes)[0]
        n = len(b["codes"])
        assert int(expo[0, 0]) == b["exponent_byte"], b["name"]
        assert int(dialect[0, 0]) == b["dialect"], b["name"]
        assert list(nib[:n]) == b["codes"], b["name"]
        assert (nib[n:] == 0).all(), b["name"]
        deq = O.dfp4_dequantize(codes, dialect, expo)[0]
        assert list(deq[:n]) == list(np.ldexp(np.array(b["dequant"], dtype=np.float64), k)), b["name"]
        assert (deq[n:] == 0).all()


def test_handworked_gemm_and_mxfp4(golden_dir):
    g = _golden(golden_dir, "handworked_blocks.json")
    a = _block(g["blocks"][0]["x"])
    q = O.dfp4_quantize(a)
    assert O.dfp4_gemm(q, q)[0, 0] == g["gemm"]["value"]
    f = g["mxfp4"]
    codes, expo = MX.mxfp4_quantize(_block(f["x"]))
    n = len(f["codes"])
    assert int(expo[0, 0]) == f["exponent_byte"]
    assert list(_nibbles(codes)[0][:n]) == f["codes"]
    assert list(MX.mxfp4_dequantize(codes, expo)[0][:n]) == f["dequant"]


def _random_blocks(rng, n, kind):
    if kind == "gauss":
        x = rng.standard_normal((n, 32))
    elif kind == "t3":
        x = rng.standard_t(3, (n, 32))
    elif kind == "outlier":
        x = rng.standard_normal((n, 32))
        x[np.arange(n), rng.integers(0, 32, n)] *= 50
    elif kind == "wide":
        x = rng.standard_normal((n, 32)) * np.exp2(rng.integers(-100, 100, (n, 1)))
    elif kind == "grid":                      # many ties: multiples of 1/8 in [-8, 8)
        x = rng.integers(-64, 64, (n, 32)) / 8.0
    return _bf16(x)


@pytest.mark.parametrize("kind", ["gauss", "t3", "outlier", "wide", "grid"])
def test_quantize_vs_exact_brute_force(kind):
    rng = np.random.default_rng({"gauss": 1, "t3": 2, "outlier": 3, "wide": 4, "grid": 5}[kind])
    x = _random_blocks(rng, 96, kind)
    codes, dialect, expo = O.dfp4_quantize(x)
    nib = _nibbles(codes)
    for b in range(x.shape[0]):
        e, d, idx = BF.quantize_block([Fraction(v) for v in x[b]], BOOK_FR)
        assert int(expo[b, 0]) - 127 == e, (kind, b)
        assert int(dialect[b, 0]) == d, (kind, b)
        assert list(nib[b] & 7) == idx, (kind, b)
        assert list(nib[b] >> 3) == [int(np.signbit(v)) for v in x[b]]


def test_invariants():
    rng = np.random.default_rng(7)
    x = np.concatenate([_random_blocks(rng, 200, k) for k in ("gauss", "t3", "outlier", "grid")])
    x = x.reshape(-1, 128)                                      # 4 blocks per row
    codes, dialect, expo = O.dfp4_quantize(x)
    deq = O.dfp4_dequantize(codes, dialect, expo)
    e = expo.astype(np.int64) - 127
    s_hat = np.abs(deq).reshape(-1, 32) / np.exp2(e.reshape(-1, 1))
    d_flat = dialect.reshape(-1)
    # every dequantized magnitude is a value of the block's dialect
    for b in range(s_hat.shape[0]):
        assert set(s_hat[b]) <= set(O.FORMATBOOK[d_flat[b]])
    # sign is kept (zero keeps the sign of its input)
    assert (np.signbit(deq) == np.signbit(x)).all()
    # the quantized block maximum is the shared maximum of the selected pair,
    # i.e. the block maximum rounded to a multiple of 0.5 (capped at 7.5)
    smax = np.abs(x).reshape(-1, 32).max(axis=1) / np.exp2(e.reshape(-1))
    want = np.minimum(np.floor(2 * smax + 0.5) / 2, 7.5)
    assert (s_hat.max(axis=1) == want).all()
    assert (O.FORMATBOOK[d_flat][:, -1] == want).all()
    # error bound: half the largest gap of the dialect (plus the cap at 7.5)
    s = np.abs(x).reshape(-1, 32) / np.exp2(e.reshape(-1, 1))
    gap = np.diff(O.FORMATBOOK[d_flat], axis=1).max(axis=1)
    assert (np.abs(s - s_hat) <= np.maximum(gap / 2, 0.5)[:, None]).all()
    # power-of-two rescaling: same codes and dialect, exponent shifts
    for k in (-9, 3, 17):
        c2, d2, e2 = O.dfp4_quantize(np.ldexp(x, k))
        assert (c2 == codes).all() and (d2 == dialect).all()
        assert (e2.astype(np.int64) == expo.astype(np.int64) + k).all()
    # sign symmetry
    c3, d3, e3 = O.dfp4_quantize(-x)
    assert (c3 == (codes ^ 0x88)).all() and (d3 == dialect).all() and (e3 == expo).all()
    # permuting elements inside a block permutes the codes only
    perm = rng.permutation(32)
    xp = x.reshape(-1, 32)[:, perm].reshape(x.shape)
    c4, d4, e4 = O.dfp4_quantize(xp)
    assert (d4 == dialect).all() and (e4 == expo).all()
    assert (_nibbles(c4).reshape(-1, 32) == _nibbles(codes).reshape(-1, 32)[:, perm]).all()
    # quantizing the dequantized tensor changes nothing (blocks on the grid round-trip)
    c5, d5, e5 = O.dfp4_quantize(deq)
    assert (O.dfp4_dequantize(c5, d5, e5) == deq).all()


def test_on_grid_blocks_round_trip_exactly():
    rng = np.random.default_rng(3)
    for d in range(16):
        vals = O.FORMATBOOK[d]
        for trial in range(20):
            idx = rng.integers(0, 8, 32)
            idx[rng.integers(0, 32)] = 7                        # the pair maximum is present
            # make the vote unambiguous: use the differing value at least once
            differing = [i for i, v in enumerate(vals) if v not in O.FORMATBOOK[d ^ 1]][0]
            idx[rng.integers(0, 32)] = differing
            idx[np.argmax(idx == 7)] = 7
            sign = rng.integers(0, 2, 32)
            k = int(rng.integers(-20, 20))
            x = np.ldexp(np.where(sign == 1, -vals[idx], vals[idx]), k)[None, :]
            if not (idx == differing).any() or not (idx == 7).any():
                continue
            codes, dialect, expo = O.dfp4_quantize(x)
            assert (O.dfp4_dequantize(codes, dialect, expo) == x).all(), (d, trial)
            assert int(dialect[0, 0]) == d
            assert int(expo[0, 0]) == 127 + k


def test_elements_outside_both_ranges_do_not_depend_on_the_vote():
    # Section 3.2: the two dialects of a pair differ only inside their beneficial ranges
    for p in range(8):
        lo_e, hi_e = O.beneficial_range(2 * p)
        lo_o, hi_o = O.beneficial_range(2 * p + 1)
        t = np.arange(32) / 4.0
        outside = ~(((t >= lo_e) & (t < hi_e)) | ((t >= lo_o) & (t < hi_o)))
        ie = O.nearest_index(t[None, :], np.array([2 * p]))[0]
        io = O.nearest_index(t[None, :], np.array([2 * p + 1]))[0]
        assert (O.FORMATBOOK[2 * p][ie][outside] == O.FORMATBOOK[2 * p + 1][io][outside]).all()


def test_two_stage_choice_is_close_to_exhaustive_mse_search():
    # Table 2: the two-stage selection performs close to MSE-based selection.
    # Statistical, on synthetic blocks: the chosen dialect's squared error is
    # within a small factor of the best of all 16 on average.
    rng = np.random.default_rng(21)
    x = _random_blocks(rng, 150, "gauss")
    _, dialect, _ = O.dfp4_quantize(x)
    ratio, agree = [], 0
    for b in range(x.shape[0]):
        best, errs = BF.mse_best_dialects([Fraction(v) for v in x[b]], BOOK_FR)
        d = int(dialect[b, 0])
        agree += d in best
        ratio.append(float(errs[d] / min(errs)) if min(errs) > 0 else 1.0)
    assert np.mean(ratio) < 1.25
    assert agree / x.shape[0] > 0.25


def test_dialectfp4_beats_mxfp4_on_average():
    # direction of Table 1: lower quantization error than MXFP4 at block 32
    rng = np.random.default_rng(8)
    for kind in ("gauss", "t3", "outlier"):
        x = _random_blocks(rng, 400, kind)
        err_d = ((O.dfp4_dequantize(*O.dfp4_quantize(x)) - x) ** 2).sum()
        err_m = ((MX.mxfp4_dequantize(*MX.mxfp4_quantize(x)) - x) ** 2).sum()
        assert err_d < err_m, kind


# --------------------------------------------------------------------------
# dequantize, MAC, bit accounting
# --------------------------------------------------------------------------
def test_gemm_vs_integer_formulation():
    rng = np.random.default_rng(13)
    a = _random_blocks(rng, 3 * 4, "outlier").reshape(3, 128)
    w = _bf16(rng.standard_normal((5, 128)) * 0.02)
    aq, wq = O.dfp4_quantize(a), O.dfp4_quantize(w)
    out = O.dfp4_gemm(aq, wq)
    an, wn = _nibbles(aq[0]).reshape(3, 4, 32), _nibbles(wq[0]).reshape(5, 4, 32)
    hu = O.FORMATBOOK_HALF_UNITS
    for m in range(3):
        for n in range(5):
            au = [[int(hu[aq[1][m, b]][c & 7]) for c in an[m, b]] for b in range(4)]
            wu = [[int(hu[wq[1][n, b]][c & 7]) for c in wn[n, b]] for b in range(4)]
            asg = [[int(c >> 3) for c in an[m, b]] for b in range(4)]
            wsg = [[int(c >> 3) for c in wn[n, b]] for b in range(4)]
            ae = [int(aq[2][m, b]) - 127 for b in range(4)]
            we = [int(wq[2][n, b]) - 127 for b in range(4)]
            want = BF.gemm_integer_form(au, asg, ae, wu, wsg, we)
            assert Fraction(out[m, n]) == want
    # and against a different library routine on the same dequantized operands
    ad, wd = O.dfp4_dequantize(*aq), O.dfp4_dequantize(*wq)
    assert np.array_equal(out, np.einsum("mk,nk->mn", ad, wd))
    # transposed operands would not pass: shapes differ, values differ
    assert out.shape == (3, 5)


def test_effective_bits(golden_dir):
    g = _golden(golden_dir, "paper_text_pins.json")["effective_bits"]
    for bs, v in g["blockdialect"].items():
        assert round(O.effective_bits(int(bs)), 2) == v
    for bs, v in g["mxfp4"].items():
        assert round(MX.effective_bits(int(bs)), 2) == v
    # this build stores an 8-bit exponent (bf16 inputs): 4 + 12/32 and 4 + 8/32
    assert O.effective_bits(32, exponent_bits=8) == 4.375
    assert MX.effective_bits(32, exponent_bits=8) == 4.25


# --------------------------------------------------------------------------
# MXFP4 reading
# --------------------------------------------------------------------------
def test_mxfp4_vs_exact_brute_force():
    rng = np.random.default_rng(17)
    e2m1 = [Fraction(v) for v in MX.E2M1]
    for kind in ("gauss", "grid", "wide"):
        x = _random_blocks(rng, 64, kind)
        codes, expo = MX.mxfp4_quantize(x)
        nib = _nibbles(codes)
        for b in range(x.shape[0]):
            e = BF.exponent_by_search(Fraction(np.abs(x[b]).max()))
            assert int(expo[b, 0]) - 127 == e
            want = [BF.e2m1_nearest_even(abs(Fraction(v)) / Fraction(2) ** e, e2m1) for v in x[b]]
            assert list(nib[b] & 7) == want
        deq = MX.mxfp4_dequantize(codes, expo)
        assert (np.signbit(deq) == np.signbit(x)).all()
    # MXFP4 values are dialect 7's values: dequantizing MX codes through
    # dialect 7 of the DialectFP4 book gives the same numbers
    d7 = np.full(expo.shape, 7, dtype=np.uint8)
    assert np.array_equal(O.dfp4_dequantize(codes, d7, expo), deq)


# --------------------------------------------------------------------------
# the pins bite: planted mistakes in a copy of the oracle are caught
# --------------------------------------------------------------------------
def test_planted_mistakes_are_caught(monkeypatch, golden_dir):
    g = _golden(golden_dir, "handworked_blocks.json")

    def handworked_ok():
        try:
            test_handworked_blocks(golden_dir)
            return True
        except AssertionError:
            return False

    assert handworked_ok()
    # ties go down instead of up
    monkeypatch.setattr(O, "nearest_index",
                        lambda s, d: np.argmin(np.abs(s[:, :, None] - O.FORMATBOOK[d][:, None, :]), axis=2))
    with pytest.raises(AssertionError):
        test_element_example_printed_in_the_paper(golden_dir)
    monkeypatch.undo()
    # exponent off by one
    real = O.shared_exponent
    monkeypatch.setattr(O, "shared_exponent", lambda a: real(a) + 1)
    assert not handworked_ok()
    monkeypatch.undo()
    # vote inverted
    real_sel = O.select_dialect
    monkeypatch.setattr(O, "select_dialect", lambda s: real_sel(s) ^ 1)
    assert not handworked_ok()
    monkeypatch.undo()
    # a wrong row in the book
    book = O.FORMATBOOK.copy()
    book[4, 6] = 4.5
    monkeypatch.setattr(O, "FORMATBOOK", book)
    with pytest.raises(AssertionError):
        test_formatbook_rows_printed_in_the_paper(golden_dir)
    monkeypatch.undo()
    assert handworked_ok() and g


# --------------------------------------------------------------------------
# MSE-based dialect selection (Section 3.2: offline choice for weights)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("kind", ["gauss", "t3", "outlier", "wide", "grid"])
def test_mse_selection_vs_exact_brute_force(kind):
    # exhaustive search over the 16 dialects in exact rationals, all 32 terms included;
    # among equal errors the lowest id
    rng = np.random.default_rng({"gauss": 21, "t3": 22, "outlier": 23, "wide": 24, "grid": 25}[kind])
    x = _random_blocks(rng, 64, kind)
    codes, dialect, expo = O.dfp4_quantize_mse(x)
    nib = _nibbles(codes)
    for b in range(x.shape[0]):
        xs = [Fraction(v) for v in x[b]]
        best, _ = BF.mse_best_dialects(xs, BOOK_FR)
        d = int(dialect[b, 0])
        assert d == best[0], (kind, b, d, best)
        e = BF.exponent_by_search(max(abs(v) for v in xs))
        assert int(expo[b, 0]) - 127 == e
        s = [abs(v) / Fraction(2) ** e for v in xs]
        assert list(nib[b] & 7) == [BF.nearest_ties_up(v, BOOK_FR[d]) for v in s], (kind, b)


def test_mse_selection_never_worse_than_two_stage():
    rng = np.random.default_rng(26)
    for kind in ("gauss", "t3", "outlier"):
        x = _random_blocks(rng, 300, kind)
        err_mse = ((O.dfp4_dequantize(*O.dfp4_quantize_mse(x)) - x) ** 2).sum(axis=1)
        err_two = ((O.dfp4_dequantize(*O.dfp4_quantize(x)) - x) ** 2).sum(axis=1)
        assert (err_mse <= err_two * (1 + 1e-12)).all(), kind
        assert err_mse.sum() < err_two.sum(), kind


def test_mse_selection_on_grid_block_is_lossless():
    # a block made of dialect 11's own values (scaled by 2^3) is reproduced exactly, and
    # dialect 11 is the lowest id that holds all of them (3.5 occurs only in d11, d13, d14)
    vals = O.FORMATBOOK[11]
    x = np.tile(np.concatenate([vals, -vals]), 2).reshape(1, 32) * 8.0
    codes, dialect, expo = O.dfp4_quantize_mse(x)
    assert int(dialect[0, 0]) == 11 and int(expo[0, 0]) == 127 + 3
    assert np.array_equal(O.dfp4_dequantize(codes, dialect, expo), x)


def test_mse_selection_all_zero_block():
    codes, dialect, expo = O.dfp4_quantize_mse(np.zeros((1, 32)))
    assert int(dialect[0, 0]) == 0 and int(expo[0, 0]) == 0 and not codes.any()


# --------------------------------------------------------------------------
# requantized product
# --------------------------------------------------------------------------
def test_round_to_bf16_matches_library_rounding():
    import torch
    rng = np.random.default_rng(31)
    x = np.concatenate([rng.standard_normal(5000) * np.exp2(rng.integers(-60, 60, 5000)),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, -3.0e38, 2.0 ** -130])])
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    got = O.round_to_bf16(x)
    assert np.array_equal(got, want) and np.array_equal(np.signbit(got), np.signbit(want))


def test_gemm_requant_is_quantized_rounded_product():
    rng = np.random.default_rng(32)
    a = _random_blocks(rng, 3 * 2, "outlier").reshape(3, 64)
    w = _bf16(rng.standard_normal((32, 64)) * 0.02)
    aq, wq = O.dfp4_quantize(a), O.dfp4_quantize(w)
    codes, dialect, expo = O.dfp4_gemm_requant(aq, wq)
    prod = O.dfp4_dequantize(*aq) @ O.dfp4_dequantize(*wq).T
    deq = O.dfp4_dequantize(codes, dialect, expo)
    # one block of 32 per row; error bounded by the largest half-gap of any dialect (1.5 units)
    amax = np.abs(prod).max(axis=1, keepdims=True)
    assert (np.abs(deq - prod) <= amax * (1.5 / 4.0) + 1e-30).all()
    assert codes.shape == (3, 16) and dialect.shape == (3, 1)


def _requant_golden_case(golden_dir):
    g = _golden(golden_dir, "handworked_requant.json")
    a = np.zeros((1, 96))
    a[0, 0::32] = g["a_blocks"]
    w = np.zeros((32, 96))
    for j, row in enumerate(g["w_rows"]):
        w[j, 0::32] = row
    assert np.array_equal(_bf16(a), a) and np.array_equal(_bf16(w), w)      # all inputs are bf16 values
    return g, a, w


def test_handworked_requantized_product(golden_dir, monkeypatch):
    """Pins the precision chain of dfp4_gemm_requant (exact sum -> fp32 -> bf16 -> quantize) on a
    hand-worked block whose products sit on and just below a bf16 midpoint."""
    g, a, w = _requant_golden_case(golden_dir)
    aq, wq = O.dfp4_quantize(a), O.dfp4_quantize(w)
    # the operands dequantize to themselves (single elements on a pair's largest value)
    assert np.array_equal(O.dfp4_dequantize(*aq), a) and np.array_equal(O.dfp4_dequantize(*wq), w)
    prod = O.dfp4_gemm(aq, wq)
    assert prod[0, 1] == 16 - 2.0 ** -5 and prod[0, 2] == 16 - 2.0 ** -5 - 2.0 ** -22      # exact in float64
    assert list(O.round_to_bf16(prod)[0, :8]) == g["after_bf16"]
    codes, dialect, expo = O.dfp4_gemm_requant(aq, wq)
    n = len(g["codes"])
    assert int(expo[0, 0]) == g["exponent_byte"] and int(dialect[0, 0]) == g["dialect"]
    assert list(_nibbles(codes)[0][:n]) == g["codes"] and (_nibbles(codes)[0][n:] == 0).all()

    # the same block with the bf16 step dropped, and with a single rounding to bf16: both change a code
    monkeypatch.setattr(O, "round_to_bf16", lambda x: np.asarray(x, dtype=np.float64))
    assert list(_nibbles(O.dfp4_gemm_requant(aq, wq)[0])[0][:n]) == g["codes_if_bf16_step_skipped"]

    def one_step(x):
        u = np.asarray(x, dtype=np.float64).view(np.uint64)
        u = (u + np.uint64((1 << 44) - 1) + ((u >> np.uint64(45)) & np.uint64(1))) & ~np.uint64((1 << 45) - 1)
        return u.view(np.float64)
    monkeypatch.setattr(O, "round_to_bf16", one_step)
    assert list(_nibbles(O.dfp4_gemm_requant(aq, wq)[0])[0][:n]) == g["codes_if_rounded_to_bf16_in_one_step"]


# --------------------------------------------------------------------------
# blocks of 64
# --------------------------------------------------------------------------
@pytest.mark.parametrize("kind", ["gauss", "outlier", "wide", "grid"])
def test_block64_vs_exact_brute_force(kind):
    rng = np.random.default_rng({"gauss": 51, "outlier": 53, "wide": 54, "grid": 55}[kind])
    x = _random_blocks(rng, 96, kind).reshape(48, 64)
    codes, dialect, expo = O.dfp4_quantize_block64(x)
    nib = _nibbles(codes)
    for b in range(x.shape[0]):
        e, d, idx = BF.quantize_block([Fraction(v) for v in x[b]], BOOK_FR)     # exhaustive, any block length
        assert (int(expo[b, 0]) - 127, int(expo[b, 1]) - 127) == (e, e), (kind, b)
        assert (int(dialect[b, 0]), int(dialect[b, 1])) == (d, d), (kind, b)
        assert list(nib[b] & 7) == idx, (kind, b)


def test_block64_output_reads_as_the_32_element_format():
    # dequantizing through the ordinary (32-element) path gives values of the chosen dialect scaled by the
    # 64-element block's exponent; a block of 64 whose halves have very different maxima shows the difference
    x = np.zeros((1, 64))
    x[0, :32] = 6.5
    x[0, 32:] = 0.4
    codes, dialect, expo = O.dfp4_quantize_block64(x)
    assert int(expo[0, 0]) == int(expo[0, 1]) == 127 and int(dialect[0, 0]) == int(dialect[0, 1])
    deq = O.dfp4_dequantize(codes, dialect, expo)
    assert np.array_equal(deq[0, :32], np.full(32, 6.5)) and np.array_equal(deq[0, 32:], np.full(32, 0.5))
    c32, d32, e32 = O.dfp4_quantize(x)
    assert int(e32[0, 1]) < 127            # with blocks of 32 the second half gets its own, smaller exponent


# --------------------------------------------------------------------------
# blocks of 16
# --------------------------------------------------------------------------
@pytest.mark.parametrize("kind", ["gauss", "outlier", "wide", "grid"])
def test_block16_vs_exact_brute_force(kind):
    rng = np.random.default_rng({"gauss": 61, "outlier": 63, "wide": 64, "grid": 65}[kind])
    x = _random_blocks(rng, 48, kind).reshape(96, 16)               # 96 blocks of 16, one per row
    codes, dialect, expo = O.dfp4_quantize_block16(x)
    assert codes.shape == (96, 8) and dialect.shape == (96, 1) and expo.shape == (96, 1)
    nib = _nibbles(codes)
    for b in range(x.shape[0]):
        e, d, idx = BF.quantize_block([Fraction(v) for v in x[b]], BOOK_FR)     # exhaustive, any block length
        assert int(expo[b, 0]) - 127 == e and int(dialect[b, 0]) == d, (kind, b)
        assert [int(v) & 7 for v in nib[b]] == idx, (kind, b)
        assert [int(v) >> 3 for v in nib[b]] == [1 if np.signbit(v) else 0 for v in x[b]]


def test_block16_layout_dequantization_and_mixed_block_product():
    rng = np.random.default_rng(66)
    a = _random_blocks(rng, 3 * 4, "outlier").reshape(3, 128)
    w = _bf16(rng.standard_normal((5, 128)) * 0.02)
    a16, w32 = O.dfp4_quantize_block16(a), O.dfp4_quantize(w)
    assert a16[1].shape == (3, 8) and a16[2].shape == (3, 8)
    # a row quantized in blocks of 16 equals its 16-element pieces quantized one by one
    for r in range(3):
        for b in range(8):
            one = O.dfp4_quantize_block16(a[r:r + 1, 16 * b:16 * b + 16])
            assert np.array_equal(one[0][0], a16[0][r, 8 * b:8 * b + 8])
            assert one[1][0, 0] == a16[1][r, b] and one[2][0, 0] == a16[2][r, b]
    # dequantization: every value is in its own 16-block's dialect, scaled by that block's exponent
    deq = O.dfp4_dequantize_block(*a16, 16)
    for r in range(3):
        for b in range(8):
            vals = set(np.ldexp(O.FORMATBOOK[a16[1][r, b]], int(a16[2][r, b]) - 127))
            assert all(abs(v) in vals for v in deq[r, 16 * b:16 * b + 16])
    # smaller blocks never quantize worse than the blocks of 32 that contain them (same data, finer exponents)
    err16 = np.abs(deq - a).sum()
    err32 = np.abs(O.dfp4_dequantize(*O.dfp4_quantize(a)) - a).sum()
    assert err16 <= err32
    # the mixed-block product against exact rationals
    prod = O.dfp4_gemm_blocks(a16, 16, w32, 32)
    wd = O.dfp4_dequantize(*w32)
    for r in range(3):
        for c in range(5):
            exact = sum(Fraction(float(x)) * Fraction(float(y)) for x, y in zip(deq[r], wd[c]))
            assert Fraction(float(prod[r, c])) == exact
    assert np.array_equal(O.dfp4_dequantize_block(*w32, 32), wd)
