"""The arithmetic behind the d = 64 bucket kernels, checked on the CPU: an fp32 number as a sum of bf16 pieces and an
fp32 product from the piece products that the kernels keep.  (No HIP code runs here: this pins the error bounds that
the kernels' header comments and the design notes state.)"""
import numpy as np

from paper_2410_03462_amd import synth


def bf16(x):
    """Nearest bf16 (ties to even) of fp32 numbers, as fp32."""
    return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32)))


def pieces(x, count):
    """x as `count` bf16 numbers: each the nearest bf16 of what the earlier ones leave (fp32 subtractions, exact)."""
    out, rest = [], np.asarray(x, dtype=np.float32)
    for _ in range(count):
        p = bf16(rest)
        out.append(p)
        rest = (rest - p).astype(np.float32)
    return out


def samples(seed, n=200000):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(n) * np.exp2(rng.integers(-20, 20, n))).astype(np.float32)


def test_three_pieces_hold_an_fp32_number_and_two_hold_it_to_2_pow_minus_16():
    x = samples(1)
    h, m, l = (p.astype(np.float64) for p in pieces(x, 3))
    assert np.array_equal(h + m + l, x.astype(np.float64))            # 3 x 8 significant bits >= the 24 of fp32
    hi, lo = (p.astype(np.float64) for p in pieces(x, 2))
    assert (np.abs(x - hi - lo) <= 2.0 ** -16 * np.abs(x)).all()      # a bf16 number has 8 significant bits
    # the remainders are exact in fp32 (what the kernels compute with one multiply-add each)
    assert np.array_equal((x - bf16(x)).astype(np.float64), x.astype(np.float64) - bf16(x).astype(np.float64))


def test_six_piece_products_give_an_fp32_grade_product():
    a, b = samples(2), samples(3)
    exact = a.astype(np.float64) * b.astype(np.float64)
    ah, am, al = (p.astype(np.float64) for p in pieces(a, 3))
    bh, bm, bl = (p.astype(np.float64) for p in pieces(b, 3))
    six = ah * bh + (ah * bm + am * bh) + (ah * bl + al * bh + am * bm)
    assert (np.abs(six - exact) <= 2.0 ** -23 * np.abs(exact)).all()      # what is dropped: a_m b_l + a_l b_m + a_l b_l
    # every piece product is exact in fp32 (8 x 8 significant bits), so only the fp32 accumulation rounds
    for p, q in ((ah, bh), (ah, bm), (am, bh), (ah, bl), (al, bh), (am, bm)):
        assert np.array_equal((p * q).astype(np.float32).astype(np.float64), p * q)
    a2 = [p.astype(np.float64) for p in pieces(a, 2)]
    b2 = [p.astype(np.float64) for p in pieces(b, 2)]
    three = a2[0] * b2[0] + a2[0] * b2[1] + a2[1] * b2[0]
    assert (np.abs(three - exact) <= 3 * 2.0 ** -16 * np.abs(exact)).all()      # two operand errors and a_l b_l
