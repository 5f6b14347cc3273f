"""Pins of the packing oracle (Sec. 5.2, symmetry-aware communication) against the paper's count, a library
routine, a hand-written example and the IEEE rounding rule."""
import numpy as np
import pytest

from oracle import pack


def test_count_is_n_times_n_plus_one_over_two():
    for n in (1, 2, 3, 64, 65, 577, 4609):
        X = np.zeros((n, n), dtype=np.float32)
        assert pack.pack_upper([X]).size == n * (n + 1) // 2 == pack.packed_elems([n])
    assert pack.packed_elems([3, 5, 1]) == 6 + 15 + 1


def test_hand_written_example():
    X = np.array([[1, 2, 3], [20, 4, 5], [30, 50, 6]], dtype=np.float32)     # lower triangle deliberately different
    Y = np.array([[7, 8], [80, 9]], dtype=np.float32)
    buf = pack.pack_upper([X, Y])
    assert buf.tolist() == [1, 2, 3, 4, 5, 6, 7, 8, 9]
    back = pack.unpack_upper(buf, [3, 2])
    assert back[0].tolist() == [[1, 2, 3], [2, 4, 5], [3, 5, 6]] and back[1].tolist() == [[7, 8], [8, 9]]


@pytest.mark.parametrize("n", [1, 2, 5, 33, 130])
def test_same_elements_as_numpy_triu_indices(n):
    rng = np.random.default_rng(n)
    X = rng.standard_normal((n, n)).astype(np.float32)
    iu = np.triu_indices(n)                                                  # row-major upper triangle
    assert np.array_equal(pack.pack_upper([X]), X[iu])
    S = (X + X.T).astype(np.float32)
    assert np.array_equal(pack.unpack_upper(pack.pack_upper([S]), [n])[0], S)   # no loss of information
    U = pack.unpack_upper(pack.pack_upper([X]), [n])[0]
    assert np.array_equal(U, U.T) and np.array_equal(np.triu(U), np.triu(X))


def test_bf16_rounding_rule():
    f = lambda bits: np.array([bits], dtype=np.uint32).view(np.float32)
    b = lambda x: int(pack.to_bf16_bits(x)[0])
    assert b(f(0x3F800000)) == 0x3F80                      # 1.0 is representable
    assert b(f(0x3F808000)) == 0x3F80                      # tie, even mantissa: stays
    assert b(f(0x3F818000)) == 0x3F82                      # tie, odd mantissa: up to even
    assert b(f(0x3F808001)) == 0x3F81                      # just above the tie: up
    assert b(f(0x3F807FFF)) == 0x3F80                      # just below: down
    assert b(f(0xBF818000)) == 0xBF82                      # sign is carried
    assert b(f(0x7F7FFFFF)) == 0x7F80                      # largest float rounds to infinity
    assert b(f(0x00000000)) == 0 and b(f(0x80000000)) == 0x8000
    assert b(f(0x7F800000)) == 0x7F80
    nan = pack.to_bf16_bits(np.array([np.nan], dtype=np.float32))[0]
    assert (nan & 0x7F80) == 0x7F80 and (nan & 0x7F) != 0
    # nearest: the rounded value is never further than half a unit in the last place, on random values
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(10000) * 10.0 ** rng.integers(-20, 20, 10000)).astype(np.float32)
    r = pack.from_bf16_bits(pack.to_bf16_bits(x)).astype(np.float64)
    ulp = np.abs(pack.from_bf16_bits(pack.to_bf16_bits(x) + np.uint16(1)).astype(np.float64) - r)
    assert np.all(np.abs(r - x.astype(np.float64)) <= 0.5 * ulp)
    # idempotent
    assert np.array_equal(pack.to_bf16_bits(pack.from_bf16_bits(pack.to_bf16_bits(x))), pack.to_bf16_bits(x))
