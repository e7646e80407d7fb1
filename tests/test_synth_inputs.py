"""Pins for the seeded input generator and the storage casts both sides are handed.

The generator is pinned against published vectors of the algorithms it names (splitmix64, FNV-1a) and
against the transform written out with the math module; the bfloat16 cast against bit patterns worked
out by hand from the format (1 sign, 8 exponent, 7 fraction bits; spacing 2^-7 in [1, 2))."""
import math

import numpy as np

import synth_inputs as S


# -- generator ---------------------------------------------------------------------------------

def test_splitmix64_published_vectors():
    # first words of the sequence for states 0 and 1234567, as listed with the reference generator
    assert [int(v) for v in S._splitmix64_words(0, 3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert [int(v) for v in S._splitmix64_words(1234567, 5)] == [
        6457827717110365317, 3203168211198807973, 9817491932198370423, 4593380528125082431, 16408922859458223821]


def test_fnv1a_published_vectors():
    assert S.name_hash("") == 0xCBF29CE484222325
    assert S.name_hash("a") == 0xAF63DC4C8601EC8C
    assert S.name_hash("foobar") == 0x85944171F73967E8


def test_one_word_stepped_by_hand():
    # word 2 of a tensor's stream with unbounded Python integers, every step written out
    mask = (1 << 64) - 1
    seed = S.stream_seed("some/tensor", 99)
    z = (seed + 2 * 0x9E3779B97F4A7C15) & mask
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
    z = z ^ (z >> 31)
    assert int(S.raw_u64("some/tensor", 2, seed=99)[1]) == z
    # the stream's state is the doubly mixed (seed ^ name hash)
    assert seed == S._mix_scalar(S._mix_scalar(99) ^ S.name_hash("some/tensor"))
    # streams of different tensors and seeds differ, a stream does not depend on how much of it is asked for
    assert int(S.raw_u64("some/tensor", 1, seed=99)[0]) != int(S.raw_u64("some/tensor2", 1, seed=99)[0])
    assert int(S.raw_u64("some/tensor", 1, seed=99)[0]) != int(S.raw_u64("some/tensor", 1, seed=98)[0])
    assert np.array_equal(S.raw_u64("some/tensor", 7, seed=99)[:3], S.raw_u64("some/tensor", 3, seed=99))


def test_uniform_uses_top_53_bits():
    w = S.raw_u64("u", 4)
    u = S.uniform01("u", 4)
    for wi, ui in zip(w, u):
        assert ui == (int(wi) >> 11) / float(1 << 53)
        assert 0.0 <= ui < 1.0


def test_box_muller_pair_written_out():
    u = S.uniform01("pair", 2)
    r = math.sqrt(-2.0 * math.log(1.0 - u[0]))
    got = S.normal("pair", (2,))
    assert got[0] == r * math.cos(2.0 * math.pi * u[1])
    assert got[1] == r * math.sin(2.0 * math.pi * u[1])
    # an odd count takes the first value of the last pair; std scales; the radius identity holds
    assert np.array_equal(S.normal("pair", (3,))[:2], got)
    assert np.allclose(S.normal("pair", (2,), std=0.5), 0.5 * got, rtol=0, atol=0)
    assert abs(got[0] ** 2 + got[1] ** 2 - (-2.0 * math.log(1.0 - u[0]))) < 1e-12


def test_normal_moments_and_labels():
    x = S.normal("moments", (400, 500))
    n = x.size
    assert abs(x.mean()) < 4.0 / math.sqrt(n)
    assert abs(x.var() - 1.0) < 4.0 * math.sqrt(2.0 / n)
    assert abs((x ** 4).mean() - 3.0) < 0.1                      # kurtosis of a normal
    assert abs(np.mean(x[:, :-1] * x[:, 1:])) < 4.0 / math.sqrt(n)  # neighbours uncorrelated
    lab = S.labels("lab", 50000, 10)
    assert lab.dtype == np.int32 and lab.min() == 0 and lab.max() == 9
    counts = np.bincount(lab, minlength=10)
    assert np.all(np.abs(counts - 5000) < 5 * math.sqrt(5000 * 0.9))
    assert np.array_equal(lab[:4], (S.raw_u64("lab", 4) % np.uint64(10)).astype(np.int32))


# -- bfloat16 cast -----------------------------------------------------------------------------

def _bits(v):
    return int(S.bf16_bits(np.array([v], dtype=np.float64))[0])


def test_bf16_exact_values_and_signs():
    assert _bits(1.0) == 0x3F80
    assert _bits(-2.0) == 0xC000
    assert _bits(0.0) == 0x0000 and _bits(-0.0) == 0x8000
    assert _bits(1.0 + 2.0 ** -7) == 0x3F81                       # one step above 1
    assert _bits((2.0 - 2.0 ** -7) * 2.0 ** 127) == 0x7F7F        # largest finite value
    assert _bits(2.0 ** -133) == 0x0001                           # smallest subnormal
    assert _bits(float("inf")) == 0x7F80 and _bits(float("-inf")) == 0xFF80
    assert _bits(float("nan")) & 0x7FC0 == 0x7FC0                 # stays a quiet NaN


def test_bf16_ties_go_to_even():
    assert _bits(1.0 + 2.0 ** -8) == 0x3F80                       # halfway 0x3F80 / 0x3F81: even is below
    assert _bits(1.0 + 2.0 ** -7 + 2.0 ** -8) == 0x3F82           # halfway 0x3F81 / 0x3F82: even is above
    assert _bits(-(1.0 + 2.0 ** -7 + 2.0 ** -8)) == 0xBF82
    assert _bits(2.0 - 2.0 ** -8) == 0x4000                       # the carry runs into the exponent
    assert _bits(2.0 ** -134) == 0x0000                           # halfway between 0 and the smallest subnormal


def test_bf16_just_off_a_tie():
    assert _bits(1.0 + 2.0 ** -8 + 2.0 ** -30) == 0x3F81
    assert _bits(1.0 + 2.0 ** -8 - 2.0 ** -30) == 0x3F80
    assert _bits(2.0 ** -134 * (1.0 + 2.0 ** -20)) == 0x0001


def test_bf16_is_one_rounding_of_the_fp64_value():
    # Above a halfway point by less than fp32 resolves: rounding to fp32 first would land ON the tie and
    # then go to even (0x3F80); one rounding of the value itself goes up.
    assert _bits(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81
    assert _bits(-(1.0 + 2.0 ** -8 + 2.0 ** -40)) == 0xBF81
    assert _bits(1.0 + 2.0 ** -7 + 2.0 ** -8 - 2.0 ** -40) == 0x3F81   # just below a tie whose even side is above
    # fp32 inputs (what the GPU converts) take the same result as their fp64 widening
    f = np.float32(1.0 + 2.0 ** -8 + 2.0 ** -23)
    assert int(S.bf16_bits(np.array([f]))[0]) == 0x3F81


def test_bf16_overflow_threshold():
    half_above_max = (2.0 - 2.0 ** -8) * 2.0 ** 127                # halfway between the largest finite value and 2^128
    assert _bits(half_above_max) == 0x7F80                         # tie: the even neighbour is 2^128 = infinity
    assert _bits(half_above_max * (1.0 - 2.0 ** -40)) == 0x7F7F
    assert _bits(3.4028234663852886e38) == 0x7F80                  # largest fp32
    assert _bits(1e39) == 0x7F80 and _bits(-1e300) == 0xFF80       # beyond fp32's range


def test_bf16_round_trip_and_nearest():
    # every finite bfloat16 value survives; a random value lands on the nearer of its two neighbours
    bits = np.arange(0, 0x7F80, dtype=np.uint16)
    vals = S.bf16_bits_to_f64(bits)
    assert np.array_equal(S.bf16_bits(vals), bits)
    assert np.array_equal(S.bf16_bits(-vals), bits | np.uint16(0x8000))
    rng = np.random.default_rng(5)
    x = rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))
    r = S.round_bf16(x)
    b = S.bf16_bits(x).astype(np.int64)
    lo = S.bf16_bits_to_f64((b - 1).astype(np.uint16))
    hi = S.bf16_bits_to_f64((b + 1).astype(np.uint16))
    assert np.all(np.abs(r - x) <= np.abs(lo - x)) and np.all(np.abs(r - x) <= np.abs(hi - x))
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)          # half a step of 2^-7 relative, at most


def test_round_f32_is_ieee_single():
    x = np.array([1.0 + 2.0 ** -24, 1.0 + 2.0 ** -24 + 2.0 ** -50, 1.0 + 3 * 2.0 ** -24])
    assert np.array_equal(S.round_f32(x), np.array([1.0, 1.0 + 2.0 ** -23, 1.0 + 2.0 ** -22]))
