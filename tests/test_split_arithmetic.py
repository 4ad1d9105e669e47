"""The arithmetic fact behind the kernels that reach fp32 accuracy on bf16 matrix instructions
(three bf16 pieces per operand, products of order <= 2), checked on the CPU in numpy: the pieces
add up to the fp32 value exactly, every piece product is exact in fp32, and the six products
carry a * b to 2^-24 of |a||b| (the three products left out are smaller than that)."""
import numpy as np


def _bf16_rn(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 (returned as fp32 with the low 16 bits zero)."""
    u = x.astype(np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def _pieces(x: np.ndarray):
    p0 = _bf16_rn(x)
    r1 = (x - p0).astype(np.float32)
    p1 = _bf16_rn(r1)
    r2 = (r1 - p1).astype(np.float32)
    p2 = _bf16_rn(r2)
    return p0, p1, p2, r1, r2


def _samples(n, seed):
    rng = np.random.default_rng(seed)
    mant = rng.uniform(1.0, 2.0, size=n)
    expo = rng.integers(-20, 20, size=n)
    sign = rng.choice([-1.0, 1.0], size=n)
    return (sign * mant * np.exp2(expo)).astype(np.float32)


def test_three_pieces_reconstruct_the_value_exactly():
    x = _samples(200_000, 1)
    p0, p1, p2, r1, r2 = _pieces(x)
    # the leftovers are exact differences, and nothing is left after the third piece
    assert np.array_equal(r1.astype(np.float64), x.astype(np.float64) - p0.astype(np.float64))
    assert np.array_equal(r2.astype(np.float64), r1.astype(np.float64) - p1.astype(np.float64))
    assert np.array_equal(p2, r2)
    total = p0.astype(np.float64) + p1.astype(np.float64) + p2.astype(np.float64)
    assert np.array_equal(total, x.astype(np.float64))
    # piece sizes: 2^-8 and 2^-17 of the value at most (round to nearest: half a unit of 8 bits each time)
    ax = np.abs(x.astype(np.float64))
    assert np.all(np.abs(p1) <= ax * 2.0 ** -8) and np.all(np.abs(p2) <= ax * 2.0 ** -17)


def test_piece_products_are_exact_in_fp32_and_six_of_them_suffice():
    a, b = _samples(200_000, 2), _samples(200_000, 3)
    pa, pb = _pieces(a)[:3], _pieces(b)[:3]
    exact = a.astype(np.float64) * b.astype(np.float64)
    six = np.zeros_like(exact)
    dropped = np.zeros_like(exact)
    for i in range(3):
        for j in range(3):
            prod64 = pa[i].astype(np.float64) * pb[j].astype(np.float64)
            # 8 x 8 significant bits: the product fits fp32 without rounding
            assert np.array_equal((pa[i] * pb[j]).astype(np.float64), prod64)
            if i + j <= 2:
                six += prod64
            else:
                dropped += np.abs(prod64)
    scale = np.abs(exact)
    assert np.all(np.abs(six - exact) <= scale * 2.0 ** -24)
    assert np.all(dropped <= scale * 2.0 ** -24)
    # two pieces per operand (three products) would not do: 2^-16, far above fp32 rounding
    three = sum(pa[i].astype(np.float64) * pb[j].astype(np.float64) for i in range(2) for j in range(2) if i + j <= 1)
    assert np.max(np.abs(three - exact) / scale) > 2.0 ** -18


def test_byte_values_are_exact_in_one_piece():
    x = np.arange(256, dtype=np.float32)
    assert np.array_equal(_bf16_rn(x), x)
