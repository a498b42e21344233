"""Pins of the epilogue oracle (bias add, rounding to fp16 / bf16).  CPU only."""
import numpy as np

from oracle import epilogue as E


def test_round_fp16_matches_numpy_conversion():
    """numpy converts float64 -> float16 with round-to-nearest-even: an independent routine."""
    g = np.random.default_rng(1)
    x = np.concatenate([g.normal(0, 1, 20000), g.normal(0, 300, 20000), g.normal(0, 1e-5, 20000),
                        g.uniform(-7e4, 7e4, 20000), [0.0, -0.0, 65504.0, 65519.9, 65520.0, -65520.0, 6e-8, 2.98e-8,
                                                      2.9802322387695312e-08, 6.103515625e-05, 1 + 2 ** -11, 1 + 3 * 2 ** -11]])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).astype(np.float64)
    got = E.round_to_16(x, E.F16)
    assert np.array_equal(got, want)
    assert np.array_equal(np.signbit(got), np.signbit(want))


def bf16_values_near(x):
    """All bf16 numbers within a few steps of x, from their bit patterns."""
    b = (np.float32(abs(x)).view(np.uint32) >> 16)
    cand = np.arange(max(0, int(b) - 3), int(b) + 4, dtype=np.uint32)
    cand = np.unique(np.concatenate([cand, cand | 0x8000]))
    return (cand.astype(np.uint32) << 16).view(np.float32).astype(np.float64), cand


def test_round_bf16_is_the_nearest_representable_value_ties_to_even():
    g = np.random.default_rng(2)
    xs = list(g.normal(0, 1, 300)) + list(g.normal(0, 1e4, 300)) + [1.0, 1 + 2 ** -8, 1 + 3 * 2 ** -8, 1 + 2 ** -9,
                                                                  -(1 + 2 ** -8), 255.5, 3.0e38, 1e-40]
    for x in xs:
        vals, bits = bf16_values_near(x)
        ok = np.isfinite(vals)
        d = np.abs(vals[ok] - x)
        best = d.min()
        winners = [(v, b) for v, b, dd in zip(vals[ok], bits[ok], d) if dd == best]
        got = float(E.round_to_16(np.array([x]), E.BF16)[0])
        if len(winners) == 1:
            assert got == winners[0][0], x
        else:                                   # a tie: the even bit pattern wins
            even = [v for v, b in winners if b % 2 == 0]
            assert got == even[0], x
    # exact for anything already representable; float32 -> upper 16 bits is the same map there
    v = (np.arange(0x3f00, 0x4100, dtype=np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(E.round_to_16(v, E.BF16), v)
    assert np.isinf(E.round_to_16(np.array([3.4e38]), E.BF16)[0])


def test_bias_is_added_per_output_column():
    C = np.arange(12, dtype=np.float64).reshape(2, 2, 3)
    b = np.array([0.5, -1.0, 2.0], dtype=np.float32)
    out = E.add_bias(C, b)
    for idx in np.ndindex(C.shape):
        assert out[idx] == C[idx] + float(b[idx[-1]])
