"""Pins of the strided-ABFT linear-layer oracle against what the paper and the mathematics fix:
the definition of a matrix product (brute force), the checksum identity of eq. (15), (16) in
exact integer arithmetic, the location rule and the repair stated after eq. (16) for every
(class, fold), the stated limit (two errors spaced by a multiple of the stride), and the
two-word representation of the checksums.  CPU only."""
import numpy as np
import pytest

from oracle import ftgemm_oracle as orc


def small_ints(rng, shape, lo=-3, hi=4):
    return rng.integers(lo, hi, size=shape).astype(np.float64)


def test_linear_clean_is_the_definition():
    rng = np.random.default_rng(1)
    X, W = rng.standard_normal((5, 7)), rng.standard_normal((11, 7))
    Y = orc.linear_clean(X, W)
    assert Y.shape == (5, 11)
    for i in range(5):
        for j in range(11):
            assert abs(Y[i, j] - sum(X[i, k] * W[j, k] for k in range(7))) < 1e-12


def test_encode_w_against_loops():
    rng = np.random.default_rng(2)
    Wb = rng.standard_normal((32, 5))
    c1, c2 = orc.encode_w(Wb, 8)
    for c in range(8):
        for k in range(5):
            assert abs(c1[c, k] - sum(Wb[c + 8 * l, k] for l in range(4))) < 1e-12
            assert abs(c2[c, k] - sum((l + 1) * Wb[c + 8 * l, k] for l in range(4))) < 1e-12


def test_fault_free_residual_is_rounding_only():
    """The oracle rounds nowhere: on real-valued operands the fault-free statistic is float64
    rounding (orders of magnitude below the threshold), and a flipped bit is located and restored
    to the exact product."""
    rng = np.random.default_rng(34)
    X = rng.standard_normal((8, 256))
    W = rng.standard_normal((512, 256)) / 16
    prm = orc.Params()
    Yref = X @ W.T
    Y, ev, dg = orc.ftgemm(X, W, prm)
    assert ev == [] and dg["res_max"] < 1e-8
    Y, ev, _ = orc.ftgemm(X, W, prm, [(5, 300, 24)])
    assert ev == [(5, 300, 1)]
    assert np.max(np.abs(Y - Yref)) < 1e-12


def test_checksum_identity_is_exact_on_integers():
    """eq. (15): X check1^T equals the stride-8 fold of Y; with small integers every sum is exact,
    so the residual is exactly zero and nothing is flagged even at a zero threshold."""
    rng = np.random.default_rng(4)
    X, W = small_ints(rng, (6, 16)), small_ints(rng, (512, 16))
    prm = orc.Params(tau_rel=0.0, tau_abs=0.0)
    Y, ev, dg = orc.ftgemm(X, W, prm)
    assert ev == []
    assert np.array_equal(Y, X @ W.T)


@pytest.mark.parametrize("block_n", [64, 256])
def test_location_and_repair_for_every_class_and_fold(block_n):
    """A single wrong element in (class c, fold l) of block b is named as column
    n0 + c + 8 l (residual ratio l + 1) and restored exactly."""
    rng = np.random.default_rng(5)
    N = 2 * block_n
    X, W = small_ints(rng, (3, 8)), small_ints(rng, (N, 8))
    Yref = X @ W.T
    prm = orc.Params(block_n=block_n, tau_rel=0.0, tau_abs=0.25)
    for col in range(N):
        row = col % 3
        # bit 23 is the lowest exponent bit: the value doubles or halves, or a zero becomes 2^-126
        f = [(row, col, 23)]
        damaged = orc.bitflip32(Yref[row, col], 23)
        if abs(damaged - Yref[row, col]) <= 0.25:
            continue
        Y, ev, _ = orc.ftgemm(X, W, prm, f)
        assert ev == [(row, col, 1)], (col, ev)
        assert np.array_equal(Y, Yref)


def test_detect_only_leaves_the_damage():
    rng = np.random.default_rng(6)
    X, W = small_ints(rng, (4, 8), 1, 4), small_ints(rng, (256, 8), 1, 4)
    Yref = X @ W.T
    prm = orc.Params(tau_rel=0.0, tau_abs=0.25, correct=False)
    Y, ev, _ = orc.ftgemm(X, W, prm, [(2, 77, 23)])
    assert ev == [(2, 77, 0)]
    assert Y[2, 77] == orc.bitflip32(Yref[2, 77], 23) and Y[2, 77] != Yref[2, 77]
    Y[2, 77] = Yref[2, 77]
    assert np.array_equal(Y, Yref)


def test_errors_in_different_classes_of_a_row_are_all_repaired():
    rng = np.random.default_rng(7)
    X, W = small_ints(rng, (2, 8), 1, 4), small_ints(rng, (256, 8), 1, 4)
    Yref = X @ W.T
    prm = orc.Params(tau_rel=0.0, tau_abs=0.25)
    faults = [(1, 8 * l + c, 23) for c, l in ((0, 3), (1, 31), (5, 0), (7, 17))]
    Y, ev, _ = orc.ftgemm(X, W, prm, faults)
    assert sorted(e[1] for e in ev) == sorted(f[1] for f in faults)
    assert np.array_equal(Y, Yref)


def test_two_errors_spaced_by_the_stride_are_seen_but_not_repaired():
    """The limit stated after eq. (16): errors of one row whose columns differ by a multiple of 8
    share a checksum class; the class is flagged, the pair cannot be put right."""
    rng = np.random.default_rng(8)
    X, W = small_ints(rng, (2, 8), 1, 4), small_ints(rng, (256, 8), 1, 4)
    Yref = X @ W.T
    prm = orc.Params(tau_rel=0.0, tau_abs=0.25)
    Y, ev, _ = orc.ftgemm(X, W, prm, [(0, 3, 23), (0, 3 + 8 * 9, 23)])
    assert len(ev) == 1 and ev[0][0] == 0
    assert not np.array_equal(Y, Yref)


def test_non_finite_result_is_located_by_magnitude():
    X = np.array([[1.0, 0.5]])
    W = np.zeros((256, 2))
    W[:, 0] = 1.0          # every output is 1.0: exponent field 0x7F, bit 30 turns it into Inf
    prm = orc.Params()
    Y, ev, _ = orc.ftgemm(X, W, prm, [(0, 100, 30)])
    assert ev == [(0, 100, 1)]
    assert np.array_equal(Y, X @ W.T)


def test_ragged_last_block_counts_missing_columns_as_zero():
    rng = np.random.default_rng(9)
    N = 256 + 43
    X, W = small_ints(rng, (3, 8), 1, 4), small_ints(rng, (N, 8), 1, 4)
    Yref = X @ W.T
    prm = orc.Params(tau_rel=0.0, tau_abs=0.25)
    Y, ev, _ = orc.ftgemm(X, W, prm)
    assert ev == [] and np.array_equal(Y, Yref)
    Y, ev, _ = orc.ftgemm(X, W, prm, [(1, N - 1, 23)])
    assert ev == [(1, N - 1, 1)] and np.array_equal(Y, Yref)


def test_threshold_is_relative_to_the_summed_magnitude():
    rng = np.random.default_rng(10)
    X = rng.standard_normal((8, 64)).astype(np.float16).astype(np.float64)
    W = (rng.standard_normal((256, 64)) / 8).astype(np.float16).astype(np.float64)
    prm = orc.Params()
    Yref = X @ W.T
    Y, ev, dg = orc.ftgemm(X, W, prm)
    assert ev == [] and dg["res_max"] < 0.05        # fault-free residuals sit far below the threshold
    # a flip of mantissa bit 2 changes the element by about 2^-21 of its size: below the threshold
    Y, ev, _ = orc.ftgemm(X, W, prm, [(3, 10, 2)])
    assert ev == []
    # a flip of the top mantissa bit changes it by a quarter to a half of its size: flagged, repaired
    Y, ev, _ = orc.ftgemm(X, W, prm, [(3, 10, 22)])
    assert ev == [(3, 10, 1)]
    assert np.max(np.abs(Y - Yref)) < 1e-5


# ---------------------------------------------------------------- checksums over the tokens (fold_tokens)

def test_fold_tokens_identity_against_loops():
    """For every output feature the stride-8 fold of Y over the tokens of a block equals
    (fold of the token rows of X) W^T: checked with explicit loops on integers, where it is exact."""
    rng = np.random.default_rng(40)
    M, N, K = 64, 5, 8
    X, W = small_ints(rng, (M, K)), small_ints(rng, (N, K))
    Y = orc.linear_clean(X, W)
    for c in range(8):
        xc = sum(X[c + 8 * l] for l in range(M // 8))
        for n in range(N):
            assert sum(Y[c + 8 * l, n] for l in range(M // 8)) == float(xc @ W[n])
    prm = orc.Params(block_n=64, tau_rel=0.0, tau_abs=0.0, fold_tokens=True)
    Y2, ev, _ = orc.ftgemm(X, W, prm)
    assert ev == [] and np.array_equal(Y2, Y)


def test_fold_tokens_locates_along_the_token_axis():
    rng = np.random.default_rng(41)
    M, N, K = 512, 3, 8
    X, W = small_ints(rng, (M, K), 1, 4), small_ints(rng, (N, K), 1, 4)
    Yref = X @ W.T
    prm = orc.Params(tau_rel=0.0, tau_abs=0.25, fold_tokens=True)
    for row in (0, 7, 8, 255, 256, 300, 511):
        col = row % N
        Y, ev, _ = orc.ftgemm(X, W, prm, [(row, col, 23)])
        assert ev == [(row, col, 1)], (row, ev)
        assert np.array_equal(Y, Yref)


def test_fold_tokens_is_the_mirror_image_of_the_default():
    """Several errors in one token row are repaired (they lie in different output features, each
    with its own checksums); two errors of one feature 8 tokens apart are seen but not repaired.
    The default encoding behaves the other way round on the same faults."""
    rng = np.random.default_rng(42)
    M, N, K = 256, 256, 8
    X, W = small_ints(rng, (M, K), 1, 4), small_ints(rng, (N, K), 1, 4)
    Yref = X @ W.T
    tok = orc.Params(tau_rel=0.0, tau_abs=0.25, fold_tokens=True)
    feat = orc.Params(tau_rel=0.0, tau_abs=0.25)
    same_row = [(5, 3, 23), (5, 3 + 8 * 9, 23)]          # one token, features 72 apart
    Y, ev, _ = orc.ftgemm(X, W, tok, same_row)
    assert sorted(e[:2] for e in ev) == [(5, 3), (5, 75)] and np.array_equal(Y, Yref)
    Y, ev, _ = orc.ftgemm(X, W, feat, same_row)
    assert len(ev) == 1 and not np.array_equal(Y, Yref)
    same_col = [(5, 3, 23), (5 + 8 * 4, 3, 23)]          # one feature, tokens 32 apart
    Y, ev, _ = orc.ftgemm(X, W, tok, same_col)
    assert len(ev) == 1 and ev[0][1] == 3 and not np.array_equal(Y, Yref)
    Y, ev, _ = orc.ftgemm(X, W, feat, same_col)
    assert sorted(e[:2] for e in ev) == [(5, 3), (37, 3)] and np.array_equal(Y, Yref)


def test_fold_tokens_ragged_block_and_random_data():
    rng = np.random.default_rng(43)
    M, N, K = 256 + 43, 7, 64
    X = rng.standard_normal((M, K)).astype(np.float16).astype(np.float64)
    W = (rng.standard_normal((N, K)) / 8).astype(np.float16).astype(np.float64)
    prm = orc.Params(fold_tokens=True)
    Yref = X @ W.T
    Y, ev, dg = orc.ftgemm(X, W, prm)
    assert ev == [] and dg["res_max"] < 0.05 and np.array_equal(Y, Yref)
    Y, ev, _ = orc.ftgemm(X, W, prm, [(M - 1, 6, 22), (10, 0, 30)])
    assert [e[:2] for e in ev] == [(10, 0), (M - 1, 6)]
    assert np.max(np.abs(Y - Yref)) < 1e-5
