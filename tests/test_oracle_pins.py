"""Pins for the CPU oracle: everything here checks oracle/ against something
that is not oracle/ -- pure-Python brute force with exact rationals, numpy's
fp64 matmul for the all-keep case, numpy.packbits for the bit layout, algebraic
invariants, closed-form keep fractions and the one pattern example the paper
prints.  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.stats import norm

import mmm_synth as synth
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------
# independent helpers (numpy / pure Python only; nothing from oracle/)
# ----------------------------------------------------------------------------
def np_masks(w):
    """Boolean keep decisions and non-zero maps straight from the definitions."""
    X, Y = w.X, w.Y
    if w.pred == synth.PRED_GT:
        keep = X > np.float32(w.threshold)
    elif w.pred == synth.PRED_ABS_GT:
        keep = np.abs(X) > np.float32(w.threshold)
    else:
        keep = np.ones_like(X, dtype=bool)
    if w.keep_a is not None:
        keep &= synth.unpack_bits(w.keep_a, w.K)
    a_nz = keep & (X != 0)
    NB = w.N // w.bw
    kb = np.ones((w.K, NB), dtype=bool)
    if w.keep_rows is not None:
        kb &= synth.unpack_bits(w.keep_rows.reshape(1, -1), w.K)[0][:, None]
    if w.keep_blocks is not None:
        kb &= synth.unpack_bits(w.keep_blocks, NB)
    blk_any = (Y.reshape(w.K, NB, w.bw) != 0).any(axis=2)
    b_occ = kb & blk_any
    return a_nz, b_occ


def np_product64(w):
    a_nz, b_occ = np_masks(w)
    A = np.where(a_nz, w.X, 0).astype(np.float64)
    B = np.where(np.repeat(b_occ, w.bw, axis=1), w.Y, 0).astype(np.float64)
    return A @ B, np.abs(A) @ np.abs(B)


def brute_force_exact(w):
    """Pure-Python triple loop in exact rational arithmetic."""
    a_nz, b_occ = np_masks(w)
    C = np.zeros((w.M, w.N), dtype=w.X.dtype)       # float32, or float64 for double-precision workloads
    for i in range(w.M):
        for j in range(w.N):
            s = Fraction(0)
            for k in range(w.K):
                if a_nz[i, k] and b_occ[k, j // w.bw]:
                    s += Fraction(float(w.X[i, k])) * Fraction(float(w.Y[k, j]))
            C[i, j] = C.dtype.type(float(s))          # one rounding of the exact sum (float() rounds to nearest double)
    return C


def tiny(M, K, N, bw, pa, pb, seed, dist="uniform", p_rows=None):
    return synth.random_masked(M, K, N, bw, pa, pb, seed, dist=dist, p_rows=p_rows)


# ----------------------------------------------------------------------------
# C values
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("M,K,N,bw", [(1, 1, 1, 1), (3, 5, 4, 2), (7, 16, 12, 4), (12, 9, 16, 8),
                                       (5, 70, 24, 3), (4, 130, 6, 6), (9, 11, 10, 1)])
def test_brute_force_tiny(M, K, N, bw):
    for seed, (pa, pb) in enumerate([(0.5, 0.5), (0.2, 0.7), (1.0, 1.0), (0.9, 0.1)]):
        w = tiny(M, K, N, bw, pa, pb, 100 + seed, p_rows=0.8 if seed % 2 else None)
        ab, bb, C, mag = oracle.run_workload(w)
        np.testing.assert_array_equal(C, brute_force_exact(w))
        # the no-skipping dense definition on the materialised operands agrees too
        A = oracle.materialize_a(w.X, ab)
        B = oracle.materialize_b(w.Y, w.bw, bb)
        np.testing.assert_array_equal(C, oracle.dense_ref(A, B).astype(np.float32))


# ---- double-precision inputs: the same pins on the *_f64 functions -----------------------------
@pytest.mark.parametrize("M,K,N,bw", [(1, 1, 1, 1), (3, 5, 4, 2), (7, 16, 12, 4), (5, 70, 24, 3), (4, 130, 6, 6)])
def test_brute_force_tiny_f64(M, K, N, bw):
    """Exact rational sums rounded once to double: the long double accumulator may differ from that by its own
    rounding of partial sums, which is below half an ulp of double times the number of terms / 2048."""
    for seed, (pa, pb) in enumerate([(0.5, 0.5), (0.2, 0.7), (1.0, 1.0)]):
        w = synth.random_masked(M, K, N, bw, pa, pb, 300 + seed, dtype=synth.DT_F64, p_rows=0.8 if seed % 2 else None)
        assert w.X.dtype == np.float64 and w.Y.dtype == np.float64
        ab, bb, C, mag = oracle.run_workload(w)
        assert C.dtype == np.float64
        a_nz, b_occ = np_masks(w)
        np.testing.assert_array_equal(synth.unpack_bits(ab, w.K), a_nz)
        np.testing.assert_array_equal(synth.unpack_bits(bb, w.N // w.bw), b_occ)
        want = brute_force_exact(w)
        assert np.all(np.abs(C - want) <= np.spacing(np.abs(want)) + 2.0 ** -60 * mag)
        # integer inputs: exact
        wi = synth.random_masked(M, K, N, bw, pa, pb, 400 + seed, dtype=synth.DT_F64, dist="smallint")
        np.testing.assert_array_equal(oracle.run_workload(wi)[2], brute_force_exact(wi))


def test_f64_all_keep_identity_and_tiny_values():
    rng = np.random.default_rng(17)
    X = rng.uniform(0.5, 1.5, size=(21, 50))
    Y = rng.uniform(-1.5, -0.5, size=(50, 32))
    C, mag = oracle.mmm(X, Y, oracle.a_bits(X), oracle.b_bits(Y, 8), 8)
    ref = (X.astype(np.longdouble) @ Y.astype(np.longdouble))
    assert np.all(np.abs(C.astype(np.longdouble) - ref) <= np.abs(ref) * 2.0 ** -52)
    np.testing.assert_allclose(mag, np.abs(X) @ np.abs(Y), rtol=1e-14)
    eye = np.eye(32)
    kb = synth.pack_bits(rng.random((32, 4)) < 0.5)
    Y2 = rng.standard_normal((32, 32))
    C2, _ = oracle.mmm(eye, Y2, oracle.a_bits(eye), oracle.b_bits(Y2, 8, None, kb), 8)
    np.testing.assert_array_equal(C2, np.where(np.repeat(synth.unpack_bits(kb, 4), 8, axis=1), Y2, 0))   # C = N(Y)
    # values float cannot hold: 1e-310 (a double denormal) is non-zero, 1e300 passes > and |.| >
    X3 = np.array([[0.0, -0.0, 1e-310, -1e300, 2.5e-320, np.nan]])
    assert synth.unpack_bits(oracle.a_bits(X3), 6)[0].tolist() == [False, False, True, True, True, True]
    assert synth.unpack_bits(oracle.a_bits(X3, synth.PRED_GT, 0.0), 6)[0].tolist() == [False, False, True, False, True, False]
    assert synth.unpack_bits(oracle.a_bits(X3, synth.PRED_ABS_GT, 1.0), 6)[0].tolist() == [False, False, False, True, False, False]
    Y3 = np.zeros((1, 16))
    Y3[0, 9] = 4.9e-324
    assert synth.unpack_bits(oracle.b_bits(Y3, 8), 2)[0].tolist() == [False, True]


def test_all_keep_is_textbook_gemm():
    rng = np.random.default_rng(7)
    X = rng.uniform(0.5, 1.5, size=(33, 77)).astype(np.float32)   # no zeros anywhere
    Y = rng.uniform(-1.5, -0.5, size=(77, 48)).astype(np.float32)
    ab = oracle.a_bits(X)
    bb = oracle.b_bits(Y, 16)
    C, mag = oracle.mmm(X, Y, ab, bb, 16)
    ref = X.astype(np.float64) @ Y.astype(np.float64)
    np.testing.assert_allclose(C, ref, rtol=0, atol=1e-6 * np.abs(ref).max())
    assert np.all(np.abs(C.astype(np.float64) - ref) <= np.abs(ref) * 2.0 ** -23)
    np.testing.assert_allclose(mag, np.abs(X).astype(np.float64) @ np.abs(Y).astype(np.float64), rtol=1e-12)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_masked_equals_dense_of_materialised(seed):
    w = tiny(37, 150, 96, 8, 0.3, 0.4, seed, dist="normal", p_rows=0.7)
    ab, bb, C, mag = oracle.run_workload(w)
    ref, refmag = np_product64(w)
    assert np.all(np.abs(C - ref) <= np.abs(ref) * 2.0 ** -23 + 1e-30)
    np.testing.assert_allclose(mag, refmag, rtol=1e-12, atol=0)


def test_exact_integer_inputs_any_order():
    w = tiny(40, 200, 64, 16, 0.4, 0.5, 11, dist="smallint")
    ab, bb, C, mag = oracle.run_workload(w)
    ref, _ = np_product64(w)
    np.testing.assert_array_equal(C.astype(np.float64), ref)       # all sums are small exact integers
    # permuting k consistently on A's columns and B's rows changes nothing
    perm = np.random.default_rng(5).permutation(w.K)
    a_nz, b_occ = np_masks(w)
    Xp = np.where(a_nz, w.X, 0)[:, perm].astype(np.float32)
    Yp = np.where(np.repeat(b_occ, w.bw, axis=1), w.Y, 0)[perm, :].astype(np.float32)
    Cp, _ = oracle.mmm(Xp, Yp, oracle.a_bits(Xp), oracle.b_bits(Yp, w.bw), w.bw)
    np.testing.assert_array_equal(Cp, C)


def test_identity_left_and_right():
    rng = np.random.default_rng(3)
    n, bw = 48, 8
    Y = rng.standard_normal((n, n)).astype(np.float32)
    kb = synth.pack_bits(rng.random((n, n // bw)) < 0.5)
    eye = np.eye(n, dtype=np.float32)
    bb = oracle.b_bits(Y, bw, None, kb)
    C, _ = oracle.mmm(eye, Y, oracle.a_bits(eye), bb, bw)
    expect = np.where(np.repeat(synth.unpack_bits(kb, n // bw), bw, axis=1), Y, 0)
    np.testing.assert_array_equal(C, expect)                         # C = N(Y)
    X = rng.standard_normal((n, n)).astype(np.float32)
    ka = synth.pack_bits(rng.random((n, n)) < 0.3)
    ab = oracle.a_bits(X, synth.PRED_NONZERO, 0.0, ka)
    C2, _ = oracle.mmm(X, eye, ab, oracle.b_bits(eye, bw), bw)
    np.testing.assert_array_equal(C2, np.where(synth.unpack_bits(ka, n), X, 0))   # C = M(X)


def test_zero_masks_give_plus_zero():
    w = tiny(9, 40, 16, 8, 0.0, 0.5, 1)
    ab, bb, C, mag = oracle.run_workload(w)
    assert not ab.any() and np.all(C == 0) and not np.signbit(C).any() and np.all(mag == 0)
    assert oracle.counts(ab, bb, w.M, w.K, w.N, w.bw)[2] == 0
    w = tiny(9, 40, 16, 8, 0.5, 0.0, 2)
    ab, bb, C, mag = oracle.run_workload(w)
    assert not bb.any() and np.all(C == 0) and not np.signbit(C).any()
    assert oracle.counts(ab, bb, w.M, w.K, w.N, w.bw)[2] == 0


def test_skipped_operands_never_reach_the_sum_and_kept_infinity_follows_the_definition():
    """Skipping semantics pinned by a pure-Python loop that really skips (not by a dense product, where 0 x Inf would
    be NaN): junk at masked positions changes nothing, and an Inf inside an occupied block reaches exactly the rows
    whose element of A at that k is non-zero."""
    w = tiny(9, 24, 16, 4, 0.4, 0.5, 12, dist="smallint")
    a_nz, b_occ = np_masks(w)
    k, jb = [int(v[0]) for v in np.nonzero(b_occ)]
    j = jb * w.bw + 1
    w.Y[k, j] = np.inf
    w.X = np.where(synth.unpack_bits(w.keep_a, w.K), w.X, np.float32(np.nan))
    w.Y = np.where(np.repeat(synth.unpack_bits(w.keep_blocks, w.N // w.bw), w.bw, axis=1), w.Y, np.float32(-np.inf))
    want = np.zeros((w.M, w.N))
    for i in range(w.M):
        for jj in range(w.N):
            for kk in range(w.K):
                if a_nz[i, kk] and b_occ[kk, jj // w.bw]:
                    want[i, jj] += float(w.X[i, kk]) * float(w.Y[kk, jj])
    ab, bb, C, _ = oracle.run_workload(w)
    np.testing.assert_array_equal(synth.unpack_bits(ab, w.K), a_nz)
    np.testing.assert_array_equal(synth.unpack_bits(bb, w.N // w.bw), b_occ)
    np.testing.assert_array_equal(C, want.astype(np.float32))
    assert np.isinf(C[a_nz[:, k], j]).all() and np.isfinite(C[~a_nz[:, k], j]).all() and a_nz[:, k].any()
    assert np.isfinite(np.delete(C, j, axis=1)).all()


def test_accumulate_mode():
    w = tiny(10, 64, 32, 16, 0.5, 0.5, 9, dist="smallint")
    ab, bb, C, _ = oracle.run_workload(w)
    C2, _ = oracle.mmm(w.X, w.Y, ab, bb, w.bw, C_in=C)
    np.testing.assert_array_equal(C2, 2 * C)


def test_rows_subset_and_single_element():
    w = tiny(20, 90, 48, 16, 0.4, 0.4, 4, dist="normal")
    ab, bb, C, mag = oracle.run_workload(w)
    Cs, ms = oracle.mmm(w.X, w.Y, ab, bb, w.bw, rows=(5, 9))
    np.testing.assert_array_equal(Cs[5:9], C[5:9])
    assert np.all(Cs[:5] == 0) and np.all(Cs[9:] == 0)
    ref, refmag = np_product64(w)
    for (i, j) in [(0, 0), (19, 47), (7, 16), (13, 31)]:
        c, m = oracle.mmm_element(w.X, w.Y, ab, bb, w.bw, i, j)
        assert abs(c - ref[i, j]) <= 1e-12 * max(1.0, refmag[i, j])
        assert abs(m - refmag[i, j]) <= 1e-12 * max(1.0, refmag[i, j])


# ----------------------------------------------------------------------------
# map bits
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("M,K,N,bw", [(5, 64, 64, 8), (3, 65, 520, 8), (7, 127, 1040, 16), (2, 200, 4160, 32)])
def test_bits_match_packbits_definition(M, K, N, bw):
    w = tiny(M, K, N, bw, 0.3, 0.3, 42 + K, p_rows=0.6)
    w.X[0, 0] = 0.0      # a kept zero is not a non-zero
    ab = oracle.a_bits(w.X, w.pred, w.threshold, w.keep_a)
    bb = oracle.b_bits(w.Y, w.bw, w.keep_rows, w.keep_blocks)
    a_nz, b_occ = np_masks(w)
    np.testing.assert_array_equal(ab, synth.pack_bits(a_nz))
    np.testing.assert_array_equal(bb, synth.pack_bits(b_occ))
    # mask-count consistency, pad bits zero
    assert int(np.bitwise_count(ab).sum()) == int(a_nz.sum())
    assert int(np.bitwise_count(bb).sum()) == int(b_occ.sum())
    na, nb, macs = oracle.counts(ab, bb, M, K, N, bw)
    assert (na, nb) == (int(a_nz.sum()), int(b_occ.sum()))
    assert macs == int((a_nz.sum(axis=0).astype(np.int64) * b_occ.sum(axis=1).astype(np.int64)).sum()) * bw


def test_block_edges():
    K, N, bw = 70, 48, 16
    Y = np.zeros((K, N), dtype=np.float32)
    Y[0, 0] = 1.0            # first column of first block
    Y[1, 15] = 1.0           # last column of first block
    Y[2, 16] = 1.0           # first column of second block
    Y[3, N - 1] = 1.0        # very last column
    Y[K - 1, 31] = -2.0      # last row (K not a multiple of 64)
    bb = oracle.b_bits(Y, bw)
    assert bb.shape == (K, 1)
    assert [int(bb[r, 0]) for r in (0, 1, 2, 3, K - 1)] == [1, 1, 2, 4, 2]
    assert int(np.bitwise_count(bb).sum()) == 5
    X = np.zeros((2, K), dtype=np.float32)
    X[0, 63] = 1.0
    X[0, 64] = 1.0
    X[1, K - 1] = 3.0
    ab = oracle.a_bits(X)
    assert ab.shape == (2, 2)
    assert int(ab[0, 0]) == 1 << 63 and int(ab[0, 1]) == 1 and int(ab[1, 1]) == 1 << (K - 1 - 64)


def test_zero_semantics():
    X = np.array([[0.0, -0.0, 1e-45, -1e-40, np.nan, np.inf, -1.0, 2.0]], dtype=np.float32)
    assert int(oracle.a_bits(X)[0, 0]) == 0b11111100                 # +-0 are zero; denormal, NaN, Inf are not
    assert int(oracle.a_bits(X, synth.PRED_GT, 0.0)[0, 0]) == 0b10100100      # x > 0: denormal+, +Inf, 2
    assert int(oracle.a_bits(X, synth.PRED_ABS_GT, 0.5)[0, 0]) == 0b11100000  # |x| > .5: Inf, -1, 2
    Y = np.zeros((3, 16), dtype=np.float32)
    Y[0, 3] = -0.0
    Y[1, 9] = 1e-45
    Y[2, 12] = np.nan
    bb = oracle.b_bits(Y, 8)
    assert [int(v) for v in bb[:, 0]] == [0, 2, 2]


def test_keep_fraction_closed_forms():
    # Bernoulli keep: count within 5 sigma of p*n
    w = synth.random_masked(256, 512, 512, 16, 0.2, 0.1, 77)
    ab, bb = oracle.a_bits(w.X, w.pred, w.threshold, w.keep_a), oracle.b_bits(w.Y, 16, None, w.keep_blocks)
    for bits, n, p in [(ab, 256 * 512, 0.2), (bb, 512 * 32, 0.1)]:
        cnt = int(np.bitwise_count(bits).sum())
        assert abs(cnt - p * n) <= 5 * np.sqrt(n * p * (1 - p))
    # ReLU on N(mu,1): keep fraction Phi(mu)
    for mu, phi in [(-1.3, 0.0968), (-1.65, 0.0495)]:
        assert abs(norm.cdf(mu) - phi) < 5e-5
        wl = synth.relu_mlp(128, 2048, 64, 16, mu, None, 0.5, 5, "t")
        cnt = int(np.bitwise_count(oracle.a_bits(wl.X, wl.pred, wl.threshold)).sum())
        n = 128 * 2048
        assert abs(cnt - phi * n) <= 5 * np.sqrt(n * phi * (1 - phi)) + 5e-5 * n


def test_paper_pattern_example_and_our_bit_order():
    """The paper prints patterns first-vector-leftmost; our words are LSB-first."""
    kv = {}
    with open(os.path.join(GOLDEN, "paper_pattern_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, *vals = line.split()
                kv[key] = vals
    psize, vsize = int(kv["pattern_size"][0]), int(kv["vector_size"][0])
    printed = kv["pattern_as_printed"][0]
    vectors = [int(v) for v in kv["nonzero_vectors_one_based"]]
    assert [i + 1 for i, ch in enumerate(printed) if ch == "1"] == vectors
    Y = np.zeros((1, psize * vsize), dtype=np.float32)
    for v in vectors:
        Y[0, (v - 1) * vsize + 5] = 1.0
    word = int(oracle.b_bits(Y, vsize)[0, 0])
    ours_lsb_first = "".join("1" if (word >> i) & 1 else "0" for i in range(psize))
    assert ours_lsb_first == printed          # reading our word from bit 0 upward gives the printed string
    assert word == sum(1 << (v - 1) for v in vectors) == 0x0A


# ----------------------------------------------------------------------------
# generators and scaled configs
# ----------------------------------------------------------------------------
def test_generators_are_seeded_and_shaped():
    a, b = synth.config(2, scale=16), synth.config(2, scale=16)
    np.testing.assert_array_equal(a.X, b.X)
    np.testing.assert_array_equal(a.keep_blocks, b.keep_blocks)
    assert (a.M, a.K, a.N, a.bw) == (128, 128, 128, 16)
    w5 = synth.config(5, scale=16)
    assert w5.dtype == synth.DT_BF16 and w5.X_bits.dtype == np.uint16
    np.testing.assert_array_equal((w5.X_bits.astype(np.uint32) << 16).view(np.float32), w5.X)
    # bf16 rounding is nearest-even on the 16 dropped bits
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    _, v = synth.round_to_bf16(x)
    np.testing.assert_array_equal(v, np.array([1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7], dtype=np.float32))


def test_half_inputs_and_column_structured_generator():
    # IEEE half rounding is numpy's; the bit patterns and the widened values describe the same numbers
    w = synth.random_masked(24, 80, 48, 16, 0.4, 0.5, 9, dist="normal", dtype=synth.DT_F16)
    np.testing.assert_array_equal(w.X_bits.view(np.float16).astype(np.float32), w.X)
    np.testing.assert_array_equal(w.Y_bits.view(np.float16).astype(np.float32), w.Y)
    assert np.all(np.abs(w.X) < 65504)
    ab, bb, C, mag = oracle.run_workload(w)
    a_nz, b_occ = np_masks(w)
    np.testing.assert_array_equal(ab, synth.pack_bits(a_nz))
    ref, _ = np_product64(w)
    assert np.all(np.abs(C - ref) <= np.abs(ref) * 2.0 ** -23 + 1e-30)
    # column-structured A: the columns of A that are on and the rows of B that are on come from one set
    w = synth.column_sparse(40, 300, 96, 16, 0.2, 0.6, 0.7, 4)
    ab, bb, C, mag = oracle.run_workload(w)
    sel = synth.unpack_bits(w.keep_rows.reshape(1, -1), w.K)[0]
    assert 0.1 < sel.mean() < 0.3
    assert not (synth.unpack_bits(ab, w.K).any(axis=0) & ~sel).any()
    assert not (synth.unpack_bits(bb, w.N // w.bw).any(axis=1) & ~sel).any()
    ref, _ = np_product64(w)
    assert np.all(np.abs(C - ref) <= np.abs(ref) * 2.0 ** -23 + 1e-30)
    # only the selected k contribute: the product over the selected columns alone is the same
    A = np.where(synth.unpack_bits(ab, w.K), w.X, 0).astype(np.float64)
    B = np.where(np.repeat(synth.unpack_bits(bb, w.N // w.bw), w.bw, axis=1), w.Y, 0).astype(np.float64)
    np.testing.assert_allclose(A[:, sel] @ B[sel, :], ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_scaled_configs_run_and_agree_with_numpy(n):
    w = synth.config(n, scale=16)
    ab, bb, C, mag = oracle.run_workload(w)
    a_nz, b_occ = np_masks(w)
    np.testing.assert_array_equal(ab, synth.pack_bits(a_nz))
    np.testing.assert_array_equal(bb, synth.pack_bits(b_occ))
    ref, refmag = np_product64(w)
    assert np.all(np.abs(C - ref) <= np.abs(ref) * 2.0 ** -23 + 1e-30)
