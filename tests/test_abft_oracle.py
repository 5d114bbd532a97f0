"""Pins of the checksum oracle: the identities of Section 2.3 (Eq. 3-6) and the location
encoding of Section 4.1 hold exactly on small-integer tiles; every element position and
every value-changing bit is located and corrected; Section 4.2's cost figure."""
import numpy as np
import pytest

from oracle import abft


def _tile(seed, m=8, k=6, n=5):
    rng = np.random.default_rng(seed)
    return (rng.integers(-8, 9, size=(m, k)).astype(np.float64),
            rng.integers(-8, 9, size=(k, n)).astype(np.float64))


def test_encoded_product_carries_row_and_column_sums():
    X, Y = _tile(0)
    Xp, Yp, Dp = abft.encode(X, Y)
    D = X @ Y
    assert Xp.shape == (9, 6) and Yp.shape == (6, 6)
    assert np.array_equal(Dp[:-1, :-1], D)
    assert np.array_equal(Dp[:-1, -1], D.sum(1))      # D e
    assert np.array_equal(Dp[-1, :-1], D.sum(0))      # e^T D


def test_relation_holds_after_every_outer_product_step():
    X, Y = _tile(1)
    steps = list(abft.online_outer_product(X, Y))
    assert len(steps) == X.shape[1]
    for s, acc in enumerate(steps):
        part = X[:, :s + 1] @ Y[:s + 1, :]
        assert np.array_equal(acc[:-1, :-1], part)
        assert np.array_equal(acc[:-1, -1], part.sum(1))
        assert np.array_equal(acc[-1, :-1], part.sum(0))
    assert np.array_equal(steps[-1], abft.encode(X, Y)[2])


def test_three_scalars_equal_weighted_sums_of_the_product():
    X, Y = _tile(2)
    assert abft.tile_checksums(X, Y) == abft.tile_sums(X @ Y)
    D = X @ Y
    w_r, w_c = np.arange(1, 9), np.arange(1, 6)
    assert abft.tile_sums(D) == (D.sum(), (D.sum(0) * w_c).sum(), (D.sum(1) * w_r).sum())


def test_every_position_is_located_and_corrected_exactly():
    X, Y = _tile(3)
    D = X @ Y
    carried = abft.tile_checksums(X, Y)
    clean, info = abft.locate_and_correct(D, carried, 0.5)
    assert info is None and np.array_equal(clean, D)
    for i in range(D.shape[0]):
        for j in range(D.shape[1]):
            for delta in (3.0, -17.0):
                bad = D.copy()
                bad[i, j] += delta
                fixed, info = abft.locate_and_correct(bad, carried, 0.5)
                assert info["ok"] and (info["row"], info["col"], info["delta"]) == (i, j, delta)
                assert np.array_equal(fixed, D)


@pytest.mark.parametrize("dtype,bits", [(np.float32, 32), (np.float64, 64)])
def test_every_value_changing_bit_flip_is_repaired(dtype, bits):
    """Fault model of Section 2.1: one flipped bit in one element of the output tile."""
    X, Y = _tile(4, 4, 3, 4)
    D = X @ Y
    D[D == 0] = 1.0                                      # avoid +0 / -0 sign flips
    carried = abft.tile_sums(D)
    for bit in range(bits):
        bad = D.copy()
        flipped = float(abft.flip_bit(dtype(D[2, 1]), bit, dtype))
        bad[2, 1] = flipped
        fixed, info = abft.locate_and_correct(bad, carried, 0.0)   # integer tile: any mismatch is a fault
        if np.isfinite(flipped) and abs(flipped - D[2, 1]) < 2.0 ** -40 * np.abs(D).sum():
            # below the resolution of a float64 sum over the tile: may go unseen, must not be
            # mis-corrected into a larger error
            assert np.allclose(fixed, D, rtol=0, atol=2.0 ** -39 * np.abs(D).sum())
        elif np.isfinite(flipped) and abs(flipped) < 2.0 ** 40:
            assert info is not None and info["ok"] and (info["row"], info["col"]) == (2, 1)
            assert np.allclose(fixed, D, rtol=0, atol=abs(flipped) * 2.0 ** -50)
        elif np.isfinite(flipped):
            # the error dwarfs the tile: it is detected; the location may no longer be decodable
            # in floating point, in which case the tile is left for recomputation
            assert info is not None
        else:
            assert info is not None and not info["ok"]   # Inf / NaN: detected, left for recompute


def test_row_form_locates_the_column_within_each_row():
    X, Y = _tile(5, 16, 8, 16)
    D = X @ Y
    carried = abft.row_checksums(X, Y)
    assert np.array_equal(carried[0], D.sum(1))
    assert np.array_equal(carried[1], D @ np.arange(1, 17))
    bad = D.copy()
    bad[3, 15] += 9.0
    bad[7, 0] -= 2.0                                     # one error per row is correctable
    fixed, found = abft.row_locate_and_correct(bad, carried, 0.5)
    assert [(f["row"], f["col"], f["delta"]) for f in found] == [(3, 15, 9.0), (7, 0, -2.0)]
    assert np.array_equal(fixed, D)


def test_two_errors_in_one_tile_are_not_silently_miscorrected():
    X, Y = _tile(6)
    D = X @ Y
    bad = D.copy()
    bad[0, 0] += 5.0
    bad[7, 4] += 5.0
    fixed, info = abft.locate_and_correct(bad, abft.tile_checksums(X, Y), 0.5)
    assert info is not None
    # two equal errors decode to the mid-point (row 4.5): must be rejected, tile unchanged
    assert not info["ok"] and np.array_equal(fixed, bad)


def test_flip_bit_touches_exactly_one_bit():
    v = np.float32(1.5)
    assert abft.flip_bit(v, 31, np.float32) == np.float32(-1.5)
    assert abft.flip_bit(v, 22, np.float32) == np.float32(1.0)
    assert abft.flip_bit(np.float64(1.0), 52, np.float64) == 0.5
    assert abft.flip_bit(abft.flip_bit(v, 7, np.float32), 7, np.float32) == v


def test_cost_model_value_quoted_in_section_4_2():
    assert abft.mma_overhead(4, 2) == 0.375
