"""Pins of the CPU oracle against what the paper and the mathematics fix.

Every check here computes its expectation by a route other than the oracle:
closed forms in float64 numpy, brute-force sorting, Monte-Carlo means, the
known answers of the generator's authors, library routines (numpy half
conversion, torch's Adam).  None of them needs a GPU.
"""
import os

import numpy as np
import pytest

import fmt

HERE = os.path.dirname(os.path.abspath(__file__))
PE = 1024  # smallest legal partition


def rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- Philox
def test_philox_known_answers(orc):
    """Generator of the random-k / dithering draws == Philox4x32-10 (SC'11 known answers)."""
    n = 0
    for line in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(t, 16) for t in line.split()]
        assert len(w) == 10
        got = orc.philox4x32_10(w[0:4], w[4:6])
        assert [int(x) for x in got] == w[6:10]
        n += 1
    assert n == 3


def test_philox_is_a_bijection_of_the_counter(orc):
    """For a fixed key distinct counters give distinct blocks (Philox is a keyed permutation)."""
    outs = {tuple(int(x) for x in orc.philox4x32_10([c, 5, 9, 1], [123, 456])) for c in range(2000)}
    assert len(outs) == 2000


def test_half_widening_matches_numpy_for_all_65536_patterns(orc):
    h = np.arange(65536, dtype=np.uint16)
    ref = h.view(np.float16).astype(np.float32)
    got = np.array([orc.half_to_float(int(x)) for x in h], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


# ---------------------------------------------------------------- sizes
def test_k_rule_and_payload_sizes(orc):
    p = orc.make_params(orc.TOPK, 1 << 20, k_ratio=0.01)
    assert orc.partition_k(p, 1 << 20) == 10485          # floor(1% of 2^20)
    assert orc.partition_k(p, 391_208) == 3912           # ResNet-50 tail partition
    assert orc.partition_k(p, 50) == 1                   # never below one element
    assert orc.partition_stride(p) == 16 + 8 * fmt.ru4(10485)
    ps = orc.make_params(orc.SIGN, 1 << 20)
    assert orc.partition_stride(ps) == 16 + (1 << 20) // 8
    assert orc.payload_bytes(ps, 25_557_032) == 25 * orc.partition_stride(ps)
    pd = orc.make_params(orc.DITHER, 1 << 21, levels=4)
    assert orc.partition_stride(pd) == 16 + (1 << 21) // 2


def test_compression_rate_arithmetic_of_the_bert_experiment():
    """Section 5.2: k = 0.1 % with int32 indices gives 333x against 2-byte gradients, i.e. the
    paper's wire format spends 2 + 4 bytes per kept element; ours (f32 value) gives 250x."""
    d, k = 1_000_000, 1000
    assert round(2 * d / (k * (2 + 4))) == 333
    assert 2 * d / (k * (4 + 4)) == 250


# ---------------------------------------------------------------- scaled sign
@pytest.mark.parametrize("d", [1, 31, 32, 33, 1000, 1024])
def test_sign_closed_form(orc, d):
    """C(v) = ||v||_1/d * sign(v) (Section 3.3, the example after Definition 2)."""
    q = (rng(d).standard_normal(d) * 1e-3).astype(np.float32)
    p = orc.make_params(orc.SIGN, PE)
    rec = orc.encode_partition(p, 0, q)
    dec = orc.decode_partition(p, 0, rec, d)
    sigma = np.float32(np.abs(q.astype(np.float64)).sum() / d)
    assert np.array_equal(dec, np.where(q < 0, -sigma, sigma).astype(np.float32))
    s, bits, words = fmt.sign_bits(rec, d)
    assert s == sigma and np.array_equal(bits, q < 0)
    # bits past d are zero
    allbits = np.unpackbits(words.view(np.uint8), bitorder="little")
    assert not allbits[d:].any()
    # ||q - C(q)||^2 = ||q||_2^2 - ||q||_1^2/d  (expand the square), hence Definition 2 holds
    q64 = q.astype(np.float64)
    lhs = ((q64 - dec.astype(np.float64)) ** 2).sum()
    rhs = (q64 ** 2).sum() - np.abs(q64).sum() ** 2 / d
    assert lhs == pytest.approx(rhs, rel=1e-5, abs=1e-18)
    assert lhs <= (q64 ** 2).sum() * (1 + 1e-6)


def test_sign_of_zero_decodes_positive(orc):
    q = np.array([0.0, -0.0, 1.0, -1.0], dtype=np.float32)
    p = orc.make_params(orc.SIGN, PE)
    dec = orc.decode_partition(p, 0, orc.encode_partition(p, 0, q), 4)
    assert np.array_equal(dec, np.array([0.5, 0.5, 0.5, -0.5], dtype=np.float32))


# ---------------------------------------------------------------- top-k
def brute_topk(q, k):
    """k largest |q| by bit pattern, lowest index first among equals; ascending index order."""
    key = q.view(np.uint32) & np.uint32(0x7FFFFFFF)
    chosen = []
    taken = np.zeros(q.size, dtype=bool)
    for _ in range(k):                      # repeated arg-max, first index wins
        masked = np.where(taken, -1, key.astype(np.int64))
        j = int(np.argmax(masked))          # argmax returns the first maximum
        taken[j] = True
        chosen.append(j)
    return np.array(sorted(chosen), dtype=np.int32)


TOPK_CASES = {
    "gauss": lambda r, d: r.standard_normal(d).astype(np.float32),
    "all_equal": lambda r, d: np.full(d, 0.25, dtype=np.float32),
    "ties_at_threshold": lambda r, d: r.integers(-3, 4, d).astype(np.float32),
    "signed_zeros": lambda r, d: np.where(r.random(d) < 0.5, 0.0, -0.0).astype(np.float32),
    "two_values": lambda r, d: np.where(r.random(d) < 0.9, 1.0, -2.0).astype(np.float32),
}


@pytest.mark.parametrize("case", sorted(TOPK_CASES))
@pytest.mark.parametrize("d,ratio", [(1, 1.0), (7, 0.3), (64, 0.25), (257, 0.1), (1000, 0.01),
                                      (1024, 1.0), (513, 1e-9)])
def test_topk_against_brute_force(orc, case, d, ratio):
    q = TOPK_CASES[case](rng(d * 7 + len(case)), d)
    p = orc.make_params(orc.TOPK, PE, k_ratio=ratio)
    k = fmt.k_of(ratio, d)
    rec = orc.encode_partition(p, 0, q)
    kk, idx, val = fmt.topk_entries(rec, fmt.k_of(ratio, PE))
    assert kk == k
    ref = brute_topk(q, k)
    assert np.array_equal(idx, ref)
    assert np.array_equal(val.view(np.uint32), q[ref].view(np.uint32))
    dec = orc.decode_partition(p, 0, rec, d)
    exp = np.zeros(d, dtype=np.float32)
    exp[ref] = q[ref]
    assert np.array_equal(dec.view(np.uint32), exp.view(np.uint32))
    # Definition 2 with delta = k/d
    q64 = q.astype(np.float64)
    assert ((q64 - dec) ** 2).sum() <= (1 - k / d) * (q64 ** 2).sum() * (1 + 1e-12) + 1e-300


def test_topk_residual_is_q_with_selected_slots_zeroed(orc):
    """Section 4.2 (operator fusion): the residual equals q with the k sent slots set to zero."""
    D = 3000
    g = rng(1).standard_normal(D).astype(np.float32)
    e = rng(2).standard_normal(D).astype(np.float32) * np.float32(0.1)
    q = g + e
    p = orc.make_params(orc.TOPK, PE, k_ratio=0.05)
    res = e.copy()
    payload = orc.compress(p, g, res)
    strd = orc.partition_stride(p)
    exp = q.copy()
    for pi, d in enumerate(fmt.part_sizes(D, PE)):
        _, idx, _ = fmt.topk_entries(fmt.record(payload, pi, strd), fmt.k_of(0.05, PE))
        exp[pi * PE + idx] = 0.0
    assert np.array_equal(res.view(np.uint32), exp.view(np.uint32))


# ---------------------------------------------------------------- random-k
def test_randk_indices_follow_the_documented_draw_rule(orc):
    d, ratio, seed, stream, part_no = 1000, 0.05, 0xDEADBEEF12345678, (3 << 32) | 7, 5
    q = np.arange(d, dtype=np.float32)      # value == index, so values reveal the indices
    p = orc.make_params(orc.RANDK, PE, k_ratio=ratio, seed=seed, stream_id=stream)
    k, val = fmt.randk_values(orc.encode_partition(p, part_no, q))
    assert k == 50
    for t in range(k):
        blk = orc.philox4x32_10([t // 4, part_no, stream & 0xFFFFFFFF, stream >> 32],
                                [seed & 0xFFFFFFFF, seed >> 32])
        assert int(val[t]) == (int(blk[t % 4]) * d) >> 32


def test_randk_unbiased_with_d_over_k(orc):
    """Definition 1: E[C(x)] = x for random-k scaled by d/k (Monte-Carlo over seeds)."""
    d, ratio, trials = 64, 0.25, 12000
    x = rng(3).standard_normal(d).astype(np.float32)
    acc = np.zeros(d)
    acc2 = np.zeros(d)
    for s in range(trials):
        p = orc.make_params(orc.RANDK, PE, k_ratio=ratio, value_scale=-1.0, seed=1000 + s)
        dec = orc.decode_partition(p, 0, orc.encode_partition(p, 0, x), d).astype(np.float64)
        acc += dec
        acc2 += dec * dec
    mean = acc / trials
    se = np.sqrt(np.maximum(acc2 / trials - mean ** 2, 1e-30) / trials)
    assert np.all(np.abs(mean - x) <= 4.5 * se + 1e-7)


def test_randk_index_histogram_is_uniform(orc):
    d, k = 50, 1024
    counts = np.zeros(d)
    q = np.arange(1024, dtype=np.float32)[:d]
    n_draws = 0
    for s in range(40):
        p = orc.make_params(orc.RANDK, PE, k_ratio=1.0, seed=s, stream_id=s * 11)
        # k_ratio = 1 on d = 50 gives k = 50 draws per call
        kk, val = fmt.randk_values(orc.encode_partition(p, s, q))
        np.add.at(counts, val.astype(int), 1)
        n_draws += kk
    expected = n_draws / d
    chi2 = ((counts - expected) ** 2 / expected).sum()
    assert chi2 < 100.0          # 49 degrees of freedom: P(chi2 > 100) < 3e-5
    assert k == 1024


def test_randk_duplicates_add_up_in_decode(orc):
    d = 8
    x = (np.arange(d) + 1).astype(np.float32)
    p = orc.make_params(orc.RANDK, PE, k_ratio=1.0, value_scale=0.5, seed=77)
    rec = orc.encode_partition(p, 0, x)
    k, val = fmt.randk_values(rec)
    assert k == d
    idx = (val - 1).astype(int)
    assert len(set(idx.tolist())) < d       # 8 draws out of 8: a repeat is (almost) certain
    exp = np.zeros(d)
    np.add.at(exp, idx, 0.5 * val.astype(np.float64))
    assert np.array_equal(orc.decode_partition(p, 0, rec, d), exp.astype(np.float32))


# ---------------------------------------------------------------- dithering
@pytest.mark.parametrize("norm", ["l2", "linf"])
def test_dither_unbiased_and_bounded(orc, norm):
    d, s, trials = 48, 4, 12000
    x = rng(5).standard_normal(d).astype(np.float32)
    nm = orc.NORM_L2 if norm == "l2" else orc.NORM_LINF
    nu_ref = np.float32(np.sqrt((x.astype(np.float64) ** 2).sum())) if norm == "l2" else np.abs(x).max()
    acc = np.zeros(d)
    acc2 = np.zeros(d)
    for t in range(trials):
        p = orc.make_params(orc.DITHER, PE, levels=s, norm=nm, seed=t, stream_id=99)
        rec = orc.encode_partition(p, 0, x)
        nu, sgn, lvl, _ = fmt.dither_nibbles(rec, d)
        assert nu == nu_ref and lvl.max() <= s
        assert np.array_equal(sgn, x < 0)
        dec = orc.decode_partition(p, 0, rec, d).astype(np.float64)
        assert np.all(np.abs(dec) <= float(nu) * (1 + 1e-7))
        # the level is one of the two neighbours of s|x|/nu
        a = np.abs(x.astype(np.float64)) * s / float(nu)
        assert np.all((lvl >= np.floor(a) - 1e-6) & (lvl <= np.floor(a) + 1 + 1e-6))
        acc += dec
        acc2 += dec * dec
    mean = acc / trials
    se = np.sqrt(np.maximum(acc2 / trials - mean ** 2, 1e-30) / trials)
    assert np.all(np.abs(mean - x) <= 4.5 * se + 1e-6)


def test_dither_exact_on_grid_points_and_ternary_case(orc):
    """If s|q_j|/nu is an integer there is nothing to round; s = 1 with the max norm sends
    sign * {0, nu}."""
    s = 4
    lv = np.array([0, 1, 2, 3, 4, 4, 2, 0, 1, 3], dtype=np.float32)
    sg = np.array([1, -1, 1, -1, 1, -1, -1, 1, 1, -1], dtype=np.float32)
    x = sg * lv * np.float32(0.125)          # max |x| = 0.5, grid step 0.125
    for seed in range(20):
        p = orc.make_params(orc.DITHER, PE, levels=s, norm=orc.NORM_LINF, seed=seed)
        rec = orc.encode_partition(p, 0, x)
        nu, sgn, lvl, _ = fmt.dither_nibbles(rec, x.size)
        assert nu == 0.5 and np.array_equal(lvl, lv.astype(np.uint8))
        assert np.array_equal(orc.decode_partition(p, 0, rec, x.size), x)
    y = rng(9).standard_normal(200).astype(np.float32)
    p = orc.make_params(orc.DITHER, PE, levels=1, norm=orc.NORM_LINF, seed=4)
    dec = orc.decode_partition(p, 0, orc.encode_partition(p, 0, y), y.size)
    m = np.abs(y).max()
    assert set(np.unique(np.abs(dec)).tolist()) <= {0.0, float(m)}
    assert np.all((dec == 0) | (np.sign(dec) == np.sign(y)))


def test_dither_uses_one_draw_per_element_in_index_order(orc):
    """Element j consumes word j%4 of block j/4: recompute the levels from the draws."""
    d, s, seed, stream, part_no = 333, 4, 42, (9 << 32) | 1, 3
    x = rng(11).standard_normal(d).astype(np.float32)
    p = orc.make_params(orc.DITHER, PE, levels=s, seed=seed, stream_id=stream)
    rec = orc.encode_partition(p, part_no, x)
    nu, _, lvl, _ = fmt.dither_nibbles(rec, d)
    for j in range(d):
        blk = orc.philox4x32_10([j // 4, part_no, stream & 0xFFFFFFFF, stream >> 32], [seed, 0])
        u = np.float32(int(blk[j % 4]) >> 8) * np.float32(2.0 ** -24)
        a = np.float32(abs(x[j])) * (np.float32(s) / np.float32(nu))      # |x| * (s / nu), float32
        l = np.floor(a)
        exp = min(s, int(l) + int(u < np.float32(a - l)))
        assert lvl[j] == exp


@pytest.mark.parametrize("s", [15, 63, 20])
def test_dither_with_bit_planes_unbiased_bounded_and_sized(orc, s):
    """The 5- and 7-bit forms (and one in between): 4 + planes bits per element, levels up to s
    split over the nibble and the planes, the same two-neighbour rounding, unbiased."""
    d, trials = 40, 6000
    planes = {15: 1, 63: 3, 20: 2}[s]
    p0 = orc.make_params(orc.DITHER, PE, levels=s, norm=orc.NORM_LINF)
    assert orc.partition_stride(p0) == 16 + 4 * (fmt.ru4(PE // 8) + planes * fmt.ru4(PE // 32))
    assert orc.partition_stride(p0) == fmt.stride("dither", PE, levels=s)
    x = rng(50 + s).standard_normal(d).astype(np.float32)
    x[3] = np.abs(x).max() * np.float32(-1.5)      # the largest magnitude is negative: top level with the sign bit
    nu_ref = np.abs(x).max()
    acc = np.zeros(d)
    acc2 = np.zeros(d)
    seen_top = False
    for t in range(trials):
        p = orc.make_params(orc.DITHER, PE, levels=s, norm=orc.NORM_LINF, seed=t, stream_id=5)
        rec = orc.encode_partition(p, 0, x)
        nu, sgn, lvl = fmt.dither_levels(rec, d, PE, s)
        assert nu == nu_ref and lvl.max() <= s and np.array_equal(sgn, x < 0)
        assert lvl[3] == s
        a = np.abs(x.astype(np.float64)) * s / float(nu)
        assert np.all((lvl >= np.floor(a) - 1e-6) & (lvl <= np.floor(a) + 1 + 1e-6))
        dec = orc.decode_partition(p, 0, rec, d)
        # decode is (nu * level) / s, element by element
        exp = (np.float32(nu) * lvl.astype(np.float32)) / np.float32(s)
        assert np.array_equal(np.abs(dec), exp)
        acc += dec
        acc2 += dec.astype(np.float64) ** 2
    mean = acc / trials
    se = np.sqrt(np.maximum(acc2 / trials - mean ** 2, 1e-30) / trials)
    assert np.all(np.abs(mean - x) <= 4.5 * se + 1e-6)


def test_dither_bit_planes_take_the_high_level_bits_in_element_order(orc):
    """Grid points need no rounding, so the record is known bit for bit: nibble = sign and the
    low three level bits, plane t = bit 3 + t of each level, LSB first, planes at offsets fixed
    by the partition size."""
    s = 63
    lv = np.array([63, 0, 8, 7, 16, 32, 40, 21, 1, 62] * 4, dtype=np.uint32)      # 40 elements: two plane words
    sg = np.where(np.arange(lv.size) % 3 == 0, -1.0, 1.0).astype(np.float32)
    x = sg * lv.astype(np.float32) * np.float32(2.0 ** -6)
    x[0] = np.float32(-63 * 2.0 ** -6)
    p = orc.make_params(orc.DITHER, PE, levels=s, norm=orc.NORM_LINF, seed=1)
    rec = orc.encode_partition(p, 0, x)
    assert fmt.header_f32(rec) == np.float32(63 * 2.0 ** -6)
    nib_words = rec[16:16 + 4 * fmt.ru4((x.size + 7) // 8)].view(np.uint32)
    for j in range(x.size):
        nib = (int(nib_words[j // 8]) >> (4 * (j % 8))) & 15
        assert nib == (8 if x[j] < 0 else 0) | (int(lv[j]) & 7)
    off0 = 16 + 4 * fmt.ru4(PE // 8)
    for t in range(3):
        words = rec[off0 + t * 4 * fmt.ru4(PE // 32):][:8].view(np.uint32)
        for j in range(x.size):
            assert (int(words[j // 32]) >> (j % 32)) & 1 == (int(lv[j]) >> (3 + t)) & 1
    assert np.array_equal(orc.decode_partition(p, 0, rec, x.size), x)
    # with up to 7 levels there are no planes and the record is the nibble record as before
    p7 = orc.make_params(orc.DITHER, PE, levels=7)
    assert orc.partition_stride(p7) == 16 + 4 * fmt.ru4(PE // 8)


# ---------------------------------------------------------------- top-k with half-precision values
def test_topk16_keeps_the_same_slots_and_sends_halves(orc):
    """Same selection as top-k; values are the nearest halves; the residual of a kept slot is
    the rounding error; the message is 6 bytes per kept element, which against 2-byte
    (mixed-precision) gradients at k = 0.1 % is the compression rate of 333 the paper quotes
    (Section 5.2)."""
    d = PE - 97
    x = (rng(31).standard_normal(d) * np.float32(0.01)).astype(np.float32)
    p32 = orc.make_params(orc.TOPK, PE, k_ratio=0.02)
    p16 = orc.make_params(orc.TOPK16, PE, k_ratio=0.02)
    k_cap = fmt.k_of(0.02, PE)
    r32, r16 = orc.encode_partition(p32, 0, x), orc.encode_partition(p16, 0, x)
    k, idx, val = fmt.topk_entries(r32, k_cap)
    k2, idx2, val2 = fmt.topk16_entries(r16, k_cap)
    assert k == k2 == fmt.k_of(0.02, d) and np.array_equal(idx, idx2)
    assert np.array_equal(val2.view(np.uint16), val.astype(np.float16).view(np.uint16))
    assert orc.partition_stride(p16) == 16 + 4 * fmt.ru4(k_cap) + 4 * fmt.ru4((k_cap + 1) // 2) == fmt.stride("topk16", PE, 0.02)
    dec = orc.decode_partition(p16, 0, r16, d)
    want = np.zeros(d, np.float32)
    want[idx] = val.astype(np.float16).astype(np.float32)
    assert np.array_equal(dec, want)
    res = np.zeros(d, np.float32)
    orc.compress(p16, x, res)
    exp = x.copy()
    exp[idx] = x[idx] - want[idx]
    assert np.array_equal(res, exp)
    # bytes per kept element and the quoted rate
    pk = orc.make_params(orc.TOPK16, 1 << 20, k_ratio=0.001)
    kk = fmt.k_of(0.001, 1 << 20)
    payload_per_elem = (4 * kk + 2 * kk) / float(1 << 20)
    assert abs(2.0 / payload_per_elem - 333.3) < 1.0
    assert orc.partition_stride(pk) <= 16 + 6 * kk + 24


# ---------------------------------------------------------------- FP16 conversion
def test_float_to_half_matches_an_independent_conversion(orc):
    """Round to nearest even, overflow to infinity, subnormal halves, signed zeros: against
    numpy's float32 -> float16 cast on random bit patterns and on the boundary cases."""
    r = rng(123)
    bits = r.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    xs = bits.view(np.float32)
    xs = xs[np.isfinite(xs)]
    special = np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, -65520.0, 65536.0, 1e30, -1e30, np.inf, -np.inf,
                        2.0 ** -24, 2.0 ** -25, np.nextafter(np.float32(2.0 ** -25), np.float32(1)), 2.0 ** -26,
                        2.0 ** -14, np.nextafter(np.float32(2.0 ** -14), np.float32(0)), 1.0 + 2.0 ** -11,
                        1.0 + 2.0 ** -11 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -11, 1e-45, -1e-45, 0.1, 1 / 3],
                       dtype=np.float32)
    # halves around the binade boundaries and exact ties between neighbouring halves
    h = r.integers(0, 0x7bff, size=4000).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float32)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float32)
    ties = ((lo.astype(np.float64) + hi.astype(np.float64)) / 2).astype(np.float32)   # exact in float32
    allx = np.concatenate([xs[:60000], special, ties, -ties, np.nextafter(ties, np.float32(0)), np.nextafter(ties, np.float32(1e9))])
    with np.errstate(over="ignore"):
        want = allx.astype(np.float16).view(np.uint16)
    got = np.array([orc.float_to_half(float(v)) for v in allx], dtype=np.uint16)
    assert np.array_equal(got, want)
    assert orc.float_to_half(float("nan")) & 0x7c00 == 0x7c00 and orc.float_to_half(float("nan")) & 0x3ff != 0


def test_fp16_compressor_is_the_cast_and_its_residual_is_the_rounding_error(orc):
    d = 1001                                         # odd: the last half-word is padded
    x = (rng(4).standard_normal(d) * np.float32(3e-3)).astype(np.float32)
    x[:4] = [0.0, -0.0, 70000.0, -1e-8]
    p = orc.make_params(orc.FP16, PE)
    assert orc.partition_stride(p) == 16 + 2 * PE == fmt.stride("fp16", PE)
    rec = orc.encode_partition(p, 0, x)
    assert not rec[:16].any()
    with np.errstate(over="ignore"):
        want = x.astype(np.float16)
    assert np.array_equal(fmt.fp16_values(rec, d).view(np.uint16), want.view(np.uint16))
    assert not rec[16 + 2 * d:16 + 4 * fmt.ru4((d + 1) // 2)].any()
    dec = orc.decode_partition(p, 0, rec, d)
    assert np.array_equal(dec.view(np.uint32), want.astype(np.float32).view(np.uint32))
    # Definition 2 with a tiny 1 - delta: relative rounding error at most 2^-11 per normal element
    fin = np.isfinite(dec) & (np.abs(x) >= 2.0 ** -14)
    assert np.all(np.abs(dec[fin] - x[fin]) <= 2.0 ** -11 * np.abs(x[fin]))
    # error feedback: residual + decode = q where both are finite
    e = (rng(5).standard_normal(d) * np.float32(1e-4)).astype(np.float32)
    g = x.copy()
    g[2] = 1.0
    res = e.copy()
    pay = orc.compress(p, g, res)
    q = g + e
    assert np.array_equal(res, q - orc.decompress(p, pay, d))


def test_fp16_server_rounds_the_f32_mean_not_the_exact_one(orc):
    """Algorithm 4's Delta is an f32 vector and C rounds each of its elements to a half: with a
    number of workers that is no power of two the mean sum * (1/n) is rounded to f32 first and to
    a half then.  Against numpy's own two casts, on inputs where rounding the exact product to a
    half in one go (what a fused multiply-convert does) would give another half: such elements
    must be in the sample, else the pin would not tell the two readings apart."""
    n, d = 3, 64 * 4096
    r = rng(2024)
    # halves of mixed exponents: their sums carry up to 24 significant bits, and about one product
    # in 2^13 lies so close to the middle between two halves that the f32 rounding decides
    msgs = [(r.standard_normal(d) * 1e-3).astype(np.float16) for _ in range(n)]
    p = orc.make_params(orc.FP16, PE)
    pays = [orc.compress(p, m.astype(np.float32), None) for m in msgs]
    acc = np.zeros(d, np.float32)
    for m in msgs:
        acc = acc + m.astype(np.float32)
    two_step = (acc * np.float32(1.0 / n)).astype(np.float16)
    one_step = (acc.astype(np.float64) * np.float64(np.float32(1.0 / n))).astype(np.float16)   # the product, rounded once
    assert np.count_nonzero(one_step.view(np.uint16) != two_step.view(np.uint16)) > 0
    out = orc.server_aggregate([p] * n, pays, p, None, d)
    strd = orc.partition_stride(p)
    got = np.concatenate([fmt.fp16_values(fmt.record(out, k, strd), dk) for k, dk in enumerate(fmt.part_sizes(d, PE))])
    assert np.array_equal(got.view(np.uint16), two_step.view(np.uint16))


# ---------------------------------------------------------------- natural dithering
@pytest.mark.parametrize("norm", ["l2", "linf"])
def test_natural_dither_unbiased_on_power_of_two_levels(orc, norm):
    """Decoded magnitudes are 0 or nu * 2^(l-s); each element lands on one of the two levels
    that bracket it; the mean over many seeds is the input (Definition 1: E[C(x)] = x)."""
    d, s, trials = 48, 4, 12000
    x = rng(15).standard_normal(d).astype(np.float32)
    x[7] *= np.float32(0.01)                  # one element below the smallest level
    nm = orc.NORM_L2 if norm == "l2" else orc.NORM_LINF
    nu_ref = np.float32(np.sqrt((x.astype(np.float64) ** 2).sum())) if norm == "l2" else np.abs(x).max()
    grid = np.array([0.0] + [float(nu_ref) * 2.0 ** (l - s) for l in range(1, s + 1)])
    acc = np.zeros(d)
    acc2 = np.zeros(d)
    ax = np.abs(x.astype(np.float64))
    lo_ref = np.array([grid[grid <= a * (1 + 1e-7)].max() for a in ax])
    hi_ref = np.array([grid[grid >= a * (1 - 1e-7)].min() for a in ax])
    for t in range(trials):
        p = orc.make_params(orc.NATDITHER, PE, levels=s, norm=nm, seed=t, stream_id=77)
        rec = orc.encode_partition(p, 0, x)
        nu, sgn, lvl, _ = fmt.dither_nibbles(rec, d)
        assert nu == nu_ref and lvl.max() <= s
        assert np.array_equal(sgn, x < 0)
        dec = orc.decode_partition(p, 0, rec, d).astype(np.float64)
        mags = np.abs(dec)
        assert np.all(np.isin(mags, grid))                     # exact: scaling by powers of two
        assert np.all((mags == lo_ref) | (mags == hi_ref))
        acc += dec
        acc2 += dec * dec
    mean = acc / trials
    se = np.sqrt(np.maximum(acc2 / trials - mean ** 2, 1e-30) / trials)
    assert np.all(np.abs(mean - x) <= 4.5 * se + 1e-6)
    # both neighbours of an interior element do occur
    assert np.all((acc2 / trials - mean ** 2 > 0) | np.isin(ax, grid))


def test_natural_dither_exact_on_levels_and_equals_linear_for_one_level(orc):
    """Inputs that sit on a level are sent as they are; with s = 1 the levels are {0, nu} for
    both quantisers, so the two must produce the same bytes from the same draws."""
    s = 5
    lv = np.array([0, 1, 2, 3, 4, 5, 5, 3, 1, 0, 2], dtype=np.int64)
    sg = np.array([1, -1, 1, -1, 1, -1, 1, 1, -1, 1, -1], dtype=np.float32)
    mag = np.where(lv == 0, 0.0, 2.0 ** (lv - s)).astype(np.float32)       # nu = 1 (max norm)
    x = sg * mag
    for seed in range(20):
        p = orc.make_params(orc.NATDITHER, PE, levels=s, norm=orc.NORM_LINF, seed=seed)
        rec = orc.encode_partition(p, 0, x)
        nu, sgn, lvl, _ = fmt.dither_nibbles(rec, x.size)
        assert nu == 1.0 and np.array_equal(lvl, lv.astype(np.uint8))
        assert np.array_equal(orc.decode_partition(p, 0, rec, x.size), x)
    y = rng(19).standard_normal(500).astype(np.float32)
    for norm in (orc.NORM_L2, orc.NORM_LINF):
        pn = orc.make_params(orc.NATDITHER, PE, levels=1, norm=norm, seed=6, stream_id=3)
        pl = orc.make_params(orc.DITHER, PE, levels=1, norm=norm, seed=6, stream_id=3)
        rn, rl = orc.encode_partition(pn, 2, y), orc.encode_partition(pl, 2, y)
        assert np.array_equal(rn[:16 + 4 * ((y.size + 7) // 8)], rl[:16 + 4 * ((y.size + 7) // 8)])
        assert np.array_equal(orc.decode_partition(pn, 2, rn, y.size), orc.decode_partition(pl, 2, rl, y.size))


def test_natural_dither_probability_is_the_distance_to_the_lower_level(orc):
    """For y = |q| 2^(s-1)/nu between 2^e and 2^(e+1) the upper level is taken with probability
    (y - 2^e)/2^e; below the first level with probability y.  Checked as frequencies."""
    s = 3                                     # levels at y = 0, 1, 2, 4 with nu = 1
    ys = np.array([0.25, 0.8, 1.0, 1.5, 2.0, 3.0, 3.9], dtype=np.float64)
    p_up = np.array([0.25, 0.8, 0.0, 0.5, 0.0, 0.5, 0.95])
    lower = np.array([0, 0, 1, 1, 2, 2, 2])
    x = (ys / 4.0).astype(np.float32)
    x = np.concatenate([x, [np.float32(1.0)]])            # fixes the max norm at 1
    trials = 20000
    ups = np.zeros(ys.size)
    for t in range(trials):
        p = orc.make_params(orc.NATDITHER, PE, levels=s, norm=orc.NORM_LINF, seed=1000 + t, stream_id=5)
        _, _, lvl, _ = fmt.dither_nibbles(orc.encode_partition(p, 0, x), x.size)
        assert np.all((lvl[:-1] == lower) | (lvl[:-1] == lower + 1)) and lvl[-1] == s
        ups += lvl[:-1] == lower + 1
    freq = ups / trials
    assert np.all(np.abs(freq - p_up) <= 4.5 * np.sqrt(np.maximum(p_up * (1 - p_up), 1e-12) / trials) + 1e-12)


def test_given_scale_takes_the_place_of_the_reduction(orc):
    """A scale handed in (the hand-off the GPU tests use to decide packed bits on equal terms)
    is used exactly where the partition's own norm would be: the closed form of the scaled sign
    with sigma replaced, the draw-by-draw level rule with nu replaced, exact levels on the grid
    of the given nu, and -- handed the value the reduction itself finds -- the same bytes."""
    d, part_no = 777, 2
    q = rng(31).standard_normal(d).astype(np.float32)
    # scaled sign: bits do not depend on the scale; decode and residual use the given one
    p0 = orc.make_params(orc.SIGN, PE)
    own = fmt.header_f32(orc.encode_partition(p0, part_no, q))
    for given in (np.float32(own), np.float32(0.3), np.float32(own * 1.0000001)):
        rec = orc.encode_partition(p0, part_no, q, norm=given)
        sigma, bits, _ = fmt.sign_bits(rec, d)
        assert sigma == given and np.array_equal(bits, q < 0)
        assert np.array_equal(orc.decode_partition(p0, part_no, rec, d), np.where(q < 0, -given, given).astype(np.float32))
        res = np.zeros(d, np.float32)
        pay = orc.compress(orc.make_params(orc.SIGN, PE, norm_override=np.array([given], np.float32)), q, res)
        assert np.array_equal(pay[:rec.size], rec)
        assert np.array_equal(res, q - np.where(q < 0, -given, given).astype(np.float32))
    assert np.array_equal(orc.encode_partition(p0, part_no, q, norm=own), orc.encode_partition(p0, part_no, q))
    # linear dithering: every level recomputed from its draw with the given nu
    s, seed, stream = 4, 42, (9 << 32) | 1
    pd = orc.make_params(orc.DITHER, PE, levels=s, seed=seed, stream_id=stream)
    own = fmt.header_f32(orc.encode_partition(pd, part_no, q))
    assert np.array_equal(orc.encode_partition(pd, part_no, q, norm=own), orc.encode_partition(pd, part_no, q))
    given = np.float32(own * 1.37)
    rec = orc.encode_partition(pd, part_no, q, norm=given)
    nu, sgn, lvl, _ = fmt.dither_nibbles(rec, d)
    assert nu == given and np.array_equal(sgn, q < 0)
    for j in range(d):
        blk = orc.philox4x32_10([j // 4, part_no, stream & 0xFFFFFFFF, stream >> 32], [seed, 0])
        u = np.float32(int(blk[j % 4]) >> 8) * np.float32(2.0 ** -24)
        a = np.float32(abs(q[j])) * (np.float32(s) / given)
        l = np.floor(a)
        assert lvl[j] == min(s, int(l) + int(u < np.float32(a - l)))
    # grid points of a given nu that is not the vector's norm: nothing to round
    lv = np.array([0, 1, 2, 3, 4, 1, 2, 0], dtype=np.float32)
    sg = np.array([1, -1, 1, -1, 1, -1, -1, 1], dtype=np.float32)
    x = sg * lv * np.float32(0.25)                       # grid of nu = 1, while ||x||_2 = 1.5
    for kind, xs, levels in ((orc.DITHER, x, 4),
                             (orc.NATDITHER, sg * np.where(lv == 0, 0, 2.0 ** (lv - 4)).astype(np.float32), 4)):
        for seed in range(10):
            pk = orc.make_params(kind, PE, levels=levels, seed=seed)
            rec = orc.encode_partition(pk, 0, xs, norm=np.float32(1.0))
            nu, _, lvl, _ = fmt.dither_nibbles(rec, xs.size)
            assert nu == 1.0 and np.array_equal(lvl, lv.astype(np.uint8))
            assert np.array_equal(orc.decode_partition(pk, 0, rec, xs.size), xs)
            assert fmt.header_f32(orc.encode_partition(pk, 0, xs)) != 1.0     # (its own norm is another number)


def test_shared_short_scale_makes_the_sign_sum_exact(orc):
    """Aggregating scaled-sign messages by counting bits (the compressed-domain shortcut for the
    server) is the plain algorithm of Algorithm 4 whenever it is exact: if all n workers sent the
    same scale sigma and the low six bits of sigma's significand are clear, every partial sum of
    the n-term sum in worker order is an integer multiple m * sigma with |m| <= 64 and therefore
    representable, so the f32 sum equals sigma * (n - 2 c) (c = workers whose bit is set) to the
    bit.  Checked on the sum itself (float64 product against the sequential f32 sum; the same
    check fails for a scale with a full significand, which is why the condition is there) and on
    the oracle's server: its message and residual are those of compressing
    Delta = sigma (n - 2 c) / n + residual formed from the counts."""
    pe, D = PE, PE + 333
    short = np.uint32(0x3A83F1C0).view(np.float32)          # about 1.0e-3, 18 significant bits
    assert int(np.float32(short).view(np.uint32)) & 0x3F == 0 and int(np.float32(0.001).view(np.uint32)) & 0x3F != 0
    for n in (2, 4, 16, 64):
        gs = [(rng(90 + i).standard_normal(D) * 1e-3).astype(np.float32) for i in range(n)]
        neg = np.sum([g < 0 for g in gs], axis=0)
        for sigma, exact in ((np.float32(short), True), (np.float32(0.001), False)):
            acc = np.zeros(D, np.float32)
            for g in gs:                                     # the n-term sum as Algorithm 4 writes it
                acc = acc + np.where(g < 0, -sigma, sigma).astype(np.float32)
            product = np.float64(sigma) * (n - 2 * neg)      # exact in float64
            if exact:
                assert np.array_equal(acc.astype(np.float64), product), n
            elif n >= 4:
                assert not np.array_equal(acc.astype(np.float64), product), n
        sigma = np.float32(short)
        scales = np.full((D + pe - 1) // pe, sigma, np.float32)
        ins = [orc.make_params(orc.SIGN, pe, norm_override=scales) for _ in range(n)]
        pays = [orc.compress(ins[i], gs[i], None) for i in range(n)]
        out = orc.make_params(orc.SIGN, pe)
        et = (rng(7).standard_normal(D) * 2e-4).astype(np.float32)
        res = et.copy()
        p_out = orc.server_aggregate(ins, pays, out, res, D)
        delta = (np.float64(sigma) * (n - 2 * neg)).astype(np.float32) * (np.float32(1.0) / np.float32(n)) + et
        res2 = np.zeros(D, np.float32)                       # compress(delta, 0): q = delta + 0 = delta
        assert np.array_equal(p_out, orc.compress(out, delta, res2)) and np.array_equal(res, res2), n


@pytest.mark.parametrize("name", ["sign", "topk", "randk", "dither"])
def test_partitions_under_the_size_threshold_are_carried_as_they_are(orc, name):
    """Section 4.2: what is too small to be worth compressing is sent uncompressed.  With the
    partition as the unit: a bypassed partition's record is its values, its residual stays 0 on
    both sides, the server's result there is the plain average of Algorithm 1, and the update
    sees that average; every other partition's record, residual and draws (the Philox
    partition number) are exactly what a call without a mask gives."""
    kw = {"sign": {}, "topk": dict(k_ratio=0.05), "randk": dict(k_ratio=0.05, seed=4, stream_id=6),
          "dither": dict(levels=4, seed=9, stream_id=(1 << 32) | 2)}[name]
    kind = {"sign": orc.SIGN, "topk": orc.TOPK, "randk": orc.RANDK, "dither": orc.DITHER}[name]
    pe, n = PE, 3
    D = 5 * pe + 321
    mask = np.array([0, 1, 1, 0, 1, 0], dtype=np.uint8)
    prm = [orc.make_params(kind, pe, stream_id=kw.get("stream_id", 0) + i, **{k: v for k, v in kw.items() if k != "stream_id"})
           for i in range(n)]
    out = orc.make_params(kind, pe, stream_id=99, **{k: v for k, v in kw.items() if k != "stream_id"})
    gs = [(rng(40 + i).standard_normal(D) * 1e-3).astype(np.float32) for i in range(n)]
    es = [(rng(50 + i).standard_normal(D) * 1e-4).astype(np.float32) for i in range(n)]
    strd, ident = orc.partition_stride(prm[0]), 16 + 4 * pe
    sizes = orc.record_sizes_bypass(prm[0], mask, D)
    assert sizes == [ident if b else strd for b in mask]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    pays, plain = [], []
    for i in range(n):
        e_mask, e_plain = es[i].copy(), es[i].copy()
        pays.append(orc.compress_bypass(prm[i], mask, gs[i], e_mask))
        plain.append(orc.compress(prm[i], gs[i], e_plain))
        assert pays[i].size == offs[-1]
        for k in range(6):
            lo, hi = k * pe, min(D, (k + 1) * pe)
            rec = pays[i][offs[k]:offs[k + 1]]
            if mask[k]:
                q = gs[i][lo:hi] + es[i][lo:hi]
                assert not rec[:16].any() and np.array_equal(rec[16:16 + 4 * (hi - lo)].view(np.float32), q)
                assert not e_mask[lo:hi].any()
            else:
                assert np.array_equal(rec, plain[i][k * strd:(k + 1) * strd])
                assert np.array_equal(e_mask[lo:hi], e_plain[lo:hi])
        es[i] = e_mask
    sres = np.zeros(D, np.float32)
    p_out = orc.server_aggregate_bypass(prm, pays, out, mask, sres, D)
    dec = orc.decompress_bypass(out, mask, p_out, D)
    qs = [gs[i] + (rng(50 + i).standard_normal(D) * 1e-4).astype(np.float32) for i in range(n)]
    for k in range(6):
        lo, hi = k * pe, min(D, (k + 1) * pe)
        if mask[k]:
            acc = np.zeros(hi - lo, np.float32)
            for i in range(n):
                acc = acc + qs[i][lo:hi]
            mean = acc * np.float32(1.0 / n)
            assert np.array_equal(dec[lo:hi], mean) and not sres[lo:hi].any()
            assert np.allclose(dec[lo:hi], np.mean([q[lo:hi].astype(np.float64) for q in qs], axis=0), rtol=1e-6, atol=1e-9)
    # the update consumes the mixed message: same as updating with the decoded vector
    x = (rng(60).standard_normal(D) * 0.02).astype(np.float32)
    m, v = np.zeros(D, np.float32), np.zeros(D, np.float32)
    x2, m2, v2 = x.copy(), m.copy(), v.copy()
    opt = orc.make_opt(orc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, 1)
    orc.adaptive_update_bypass(out, mask, p_out, D, x, m, v, opt)
    ident_p = orc.make_params(orc.IDENTITY, pe)
    orc.adaptive_update(ident_p, orc.compress(ident_p, dec, None), D, x2, m2, v2, opt)
    assert np.array_equal(x, x2) and np.array_equal(m, m2) and np.array_equal(v, v2)


def test_zero_vector_encodes_to_zero(orc):
    z = np.zeros(100, dtype=np.float32)
    for kind in (orc.SIGN, orc.DITHER, orc.NATDITHER, orc.TOPK, orc.RANDK, orc.IDENTITY):
        p = orc.make_params(kind, PE, k_ratio=0.1, levels=4)
        dec = orc.decode_partition(p, 0, orc.encode_partition(p, 0, z), 100)
        assert not dec.any()


# ---------------------------------------------------------------- Algorithm 4 identities
KINDS = ["identity", "sign", "topk", "randk", "randk_scaled", "dither", "natdither", "fp16", "topk16"]


def params_for(orc, name, pe=PE, seed=1, stream=0):
    if name == "identity":
        return orc.make_params(orc.IDENTITY, pe)
    if name == "sign":
        return orc.make_params(orc.SIGN, pe)
    if name == "topk":
        return orc.make_params(orc.TOPK, pe, k_ratio=0.05)
    if name == "randk":
        return orc.make_params(orc.RANDK, pe, k_ratio=0.05, value_scale=1.0, seed=seed, stream_id=stream)
    if name == "randk_scaled":
        return orc.make_params(orc.RANDK, pe, k_ratio=0.05, value_scale=-1.0, seed=seed, stream_id=stream)
    if name == "dither":
        return orc.make_params(orc.DITHER, pe, levels=4, seed=seed, stream_id=stream)
    if name == "natdither":
        return orc.make_params(orc.NATDITHER, pe, levels=4, seed=seed, stream_id=stream)
    if name == "fp16":
        return orc.make_params(orc.FP16, pe)
    if name == "topk16":
        return orc.make_params(orc.TOPK16, pe, k_ratio=0.05)
    raise ValueError(name)


@pytest.mark.parametrize("name", KINDS)
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_error_feedback_identity_worker(orc, name, dtype):
    """Algorithm 4, worker: e' = q - C(q), hence e' + decode(delta) == q."""
    D = 2 * PE + 345
    g = (rng(21).standard_normal(D) * 1e-2).astype(dtype)
    e = (rng(22).standard_normal(D) * 1e-3).astype(np.float32)
    p = params_for(orc, name)
    res = e.copy()
    payload = orc.compress(p, g, res)
    dec = orc.decompress(p, payload, D)
    q = g.astype(np.float32) + e
    if name in ("identity", "topk"):
        assert np.array_equal(res + dec, q)
    else:
        tol = np.spacing(np.maximum(np.abs(q), np.abs(dec))) * (20 if name == "randk_scaled" else 1)
        assert np.all(np.abs((res.astype(np.float64) + dec) - q) <= tol)
    if name == "identity":
        assert not res.any()
    # without error feedback (Algorithm 3) the message is C(g) and nothing else changes
    payload0 = orc.compress(p, g, None)
    ez = np.zeros(D, dtype=np.float32)
    payload1 = orc.compress(p, g, ez)
    assert np.array_equal(payload0, payload1)


@pytest.mark.parametrize("name", KINDS)
def test_error_feedback_identity_server(orc, name):
    """Algorithm 4, server: Delta = mean(delta_i) + e~, p = C(Delta), e~' = Delta - p."""
    D, n = PE + 77, 4
    workers = [params_for(orc, name, seed=5, stream=i) for i in range(n)]
    outp = params_for(orc, name, seed=5, stream=1 << 16)
    payloads = []
    for i in range(n):
        g = (rng(100 + i).standard_normal(D) * 1e-2).astype(np.float32)
        payloads.append(orc.compress(workers[i], g, np.zeros(D, dtype=np.float32)))
    et = (rng(7).standard_normal(D) * 1e-3).astype(np.float32)
    acc = np.zeros(D, dtype=np.float32)
    for i in range(n):
        acc = acc + orc.decompress(workers[i], payloads[i], D)
    delta = acc * np.float32(1.0 / n) + et
    res = et.copy()
    p_msg = orc.server_aggregate(workers, payloads, outp, res, D)
    dec = orc.decompress(outp, p_msg, D)
    tol = np.spacing(np.maximum(np.abs(delta), np.abs(dec))) * (20 if name == "randk_scaled" else 1)
    assert np.all(np.abs((res.astype(np.float64) + dec) - delta) <= tol)
    # Algorithm 3: same with e~ = 0 and no residual written
    p3 = orc.server_aggregate(workers, payloads, outp, None, D)
    z = np.zeros(D, dtype=np.float32)
    p4 = orc.server_aggregate(workers, payloads, outp, z, D)
    assert np.array_equal(p3, p4)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_identity_compressor_recovers_plain_averaging(orc, dtype):
    """Section 3.1/3.2: with C = identity Algorithms 3 and 4 are Algorithm 1 and all residuals stay 0."""
    D, n, steps = 2 * PE + 10, 4, 3
    p = orc.make_params(orc.IDENTITY, PE)
    e = [np.zeros(D, dtype=np.float32) for _ in range(n)]
    et = np.zeros(D, dtype=np.float32)
    for t in range(steps):
        gs = [(rng(10 * t + i).standard_normal(D)).astype(dtype) for i in range(n)]
        payloads = [orc.compress(p, gs[i], e[i]) for i in range(n)]
        out = orc.decompress(p, orc.server_aggregate([p] * n, payloads, p, et, D), D)
        mean = np.zeros(D, dtype=np.float32)
        for g in gs:
            mean = mean + g.astype(np.float32)
        mean = mean * np.float32(1.0 / n)
        assert np.array_equal(out, mean)
        assert np.allclose(out, np.mean([g.astype(np.float64) for g in gs], axis=0), rtol=1e-6, atol=1e-7)
        assert not et.any() and not any(x.any() for x in e)


@pytest.mark.parametrize("name", ["sign", "topk"])
def test_residual_contraction_over_steps(orc, name):
    """Lemma 2, first step of its proof: ||e_{t+1}|| <= sqrt(1 - delta) ||g_t + e_t||, with
    delta = k/d for top-k and delta = ||q||_1^2 / (d ||q||_2^2) for the scaled sign."""
    D = PE
    p = params_for(orc, name)
    e = np.zeros(D, dtype=np.float32)
    for t in range(3):
        g = (rng(50 + t).standard_normal(D) * 1e-3).astype(np.float32)
        q = (g + e).astype(np.float64)
        orc.compress(p, g, e)
        if name == "topk":
            delta = fmt.k_of(0.05, D) / D
        else:
            delta = np.abs(q).sum() ** 2 / (D * (q ** 2).sum())
        assert np.linalg.norm(e.astype(np.float64)) <= np.sqrt(1 - delta) * np.linalg.norm(q) * (1 + 1e-6)


# ---------------------------------------------------------------- Algorithm 5 update
def run_update(orc, kind, steps, D=2 * PE + 100, wd=0.01, blocks=None, phi=(0.0, float("inf")), seed=0):
    r = rng(seed)
    x = (r.standard_normal(D) * 0.02).astype(np.float32)
    m = np.zeros(D, dtype=np.float32)
    v = np.zeros(D, dtype=np.float32)
    p = orc.make_params(orc.IDENTITY, PE)
    gs, xs = [], [x.copy()]
    for t in range(1, steps + 1):
        g = (r.standard_normal(D) * 1e-2).astype(np.float32)
        opt = orc.make_opt(kind, 1e-3, 0.9, 0.999, 1e-8, wd, t, phi_lo=phi[0], phi_hi=phi[1],
                           block_offsets=blocks)
        orc.adaptive_update(p, orc.compress(p, g, None), D, x, m, v, opt)
        gs.append(g)
        xs.append(x.copy())
    return gs, xs, m, v


def test_adam_mode_matches_textbook_adam(orc):
    """Algorithm 5 lines for m, v, bias correction and r, with x -= lr (r + wd x): Adam with
    L2 regularisation folded in after the ratio (decoupled form), checked in float64 and
    against torch.optim.AdamW-free hand formula."""
    steps = 5
    gs, xs, m, v = run_update(orc, orc.OPT_ADAM, steps, wd=0.01)
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.999))
    x = xs[0].astype(np.float64)
    mm = np.zeros_like(x)
    vv = np.zeros_like(x)
    for t in range(1, steps + 1):
        g = gs[t - 1].astype(np.float64)
        mm = b1 * mm + (1 - b1) * g
        vv = b2 * vv + (1 - b2) * g * g
        r = (mm / (1 - b1 ** t)) / (np.sqrt(vv / (1 - b2 ** t)) + 1e-8)
        x = x - 1e-3 * (r + 0.01 * x)
        assert np.allclose(xs[t], x, rtol=2e-6, atol=1e-9)
    # m mixes terms of size 1e-3 that cancel: absolute slack of a few float32 ulps of that size
    assert np.allclose(m, mm, rtol=1e-5, atol=1e-9) and np.allclose(v, vv, rtol=1e-5, atol=1e-12)


def test_adam_mode_matches_torch_adam_without_decay(orc):
    import torch

    steps = 4
    gs, xs, _, _ = run_update(orc, orc.OPT_ADAM, steps, wd=0.0)
    xt = torch.tensor(xs[0].astype(np.float64), requires_grad=True)
    opt = torch.optim.Adam([xt], lr=1e-3, betas=(float(np.float32(0.9)), float(np.float32(0.999))), eps=1e-8)
    for t in range(steps):
        xt.grad = torch.tensor(gs[t].astype(np.float64))
        opt.step()
        # torch divides sqrt(v) by sqrt(bias_corr2) and adds eps afterwards: same quantity
        assert np.allclose(xs[t + 1], xt.detach().numpy(), rtol=2e-6, atol=1e-9)


def test_lans_update_double_precision_rederivation_and_norm_bound(orc):
    """Algorithm 5, the d~ line, per block; and ||x_{t+1} - x_t|| <= lr * phi (appendix, the
    bound on the update norm)."""
    D = 2 * PE + 100
    blocks = np.array([0, 10, 700, PE + 3, D], dtype=np.uint64)
    for phi in [(0.0, float("inf")), (0.05, 0.4)]:
        steps = 3
        gs, xs, m, v = run_update(orc, orc.OPT_LANS, steps, D=D, blocks=blocks, phi=phi, seed=4)
        b1, b2 = float(np.float32(0.9)), float(np.float32(0.999))
        x = xs[0].astype(np.float64)
        mm = np.zeros_like(x)
        vv = np.zeros_like(x)
        mhat_prev = np.zeros_like(x)
        for t in range(1, steps + 1):
            g = gs[t - 1].astype(np.float64)
            mm = b1 * mm + (1 - b1) * g
            vv = b2 * vv + (1 - b2) * g * g
            mhat = mm / (1 - b1 ** t)
            # recursion of the bias-corrected first moment (appendix, proof of the first lemma)
            rec = b1 * (1 - b1 ** (t - 1)) / (1 - b1 ** t) * mhat_prev + (1 - b1) / (1 - b1 ** t) * g
            assert np.allclose(mhat, rec, rtol=1e-12, atol=1e-18)
            mhat_prev = mhat
            den = np.sqrt(vv / (1 - b2 ** t)) + 1e-8
            r, c = mhat / den, g / den
            xn = x.copy()
            for b in range(len(blocks) - 1):
                lo, hi = int(blocks[b]), int(blocks[b + 1])
                ur, uc = r[lo:hi] + 0.01 * x[lo:hi], c[lo:hi] + 0.01 * x[lo:hi]
                ph = min(max(np.linalg.norm(x[lo:hi]), phi[0]), phi[1])
                dd = ph * (b1 * ur / np.linalg.norm(ur) + (1 - b1) * uc / np.linalg.norm(uc))
                xn[lo:hi] = x[lo:hi] - 1e-3 * dd
                step_norm = np.linalg.norm(xs[t][lo:hi].astype(np.float64) - xs[t - 1][lo:hi])
                assert step_norm <= 1e-3 * ph * (1 + 1e-4) + 1e-9
            x = xn
            assert np.allclose(xs[t], x, rtol=3e-6, atol=2e-9)


def test_lans_default_blocks_are_the_partitions(orc):
    D = 2 * PE + 100
    a = run_update(orc, orc.OPT_LANS, 2, D=D, blocks=None, seed=8)[1][-1]
    b = run_update(orc, orc.OPT_LANS, 2, D=D, blocks=np.array([0, PE, 2 * PE, D], dtype=np.uint64), seed=8)[1][-1]
    assert np.array_equal(a, b)


def test_zero_norm_terms_contribute_nothing(orc):
    D = PE
    x = np.zeros(D, dtype=np.float32)
    m = np.zeros(D, dtype=np.float32)
    v = np.zeros(D, dtype=np.float32)
    p = orc.make_params(orc.IDENTITY, PE)
    opt = orc.make_opt(orc.OPT_LANS, 1e-3, 0.9, 0.999, 1e-8, 0.01, 1)
    orc.adaptive_update(p, orc.compress(p, np.zeros(D, dtype=np.float32), None), D, x, m, v, opt)
    assert not x.any() and np.isfinite(x).all()


def test_update_consumes_the_decoded_message(orc):
    """The update sees g~ = decode(p_t): feeding a sign message equals feeding its dense decode."""
    D = PE + 50
    g = (rng(31).standard_normal(D) * 1e-3).astype(np.float32)
    ps = orc.make_params(orc.SIGN, PE)
    pid = orc.make_params(orc.IDENTITY, PE)
    msg = orc.compress(ps, g, None)
    dense = orc.decompress(ps, msg, D)
    outs = []
    for prm, payload in ((ps, msg), (pid, orc.compress(pid, dense, None))):
        x = np.full(D, 0.5, dtype=np.float32)
        m = np.zeros(D, dtype=np.float32)
        v = np.zeros(D, dtype=np.float32)
        orc.adaptive_update(prm, payload, D, x, m, v, orc.make_opt(orc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1))
        outs.append((x, m, v))
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)
