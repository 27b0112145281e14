"""Pins for the CPU oracle (no GPU): the oracle is checked against what the
number formats and the mathematics fix, never against itself.

The paper (Evaluation section; Listing "Naive affine matmul") defines the
result as C = A B + C on row-major matrices and prints no numeric example, so
the pins are: the binary16/binary32 formats, closed forms, exact rational
arithmetic in a different loop order, numpy's float64 matmul on inputs where it
is exact, and algebraic invariants.
"""
import ctypes
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2108_13191_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ieee_binary16_values.txt")


def test_f16_decoder_all_patterns(oracle_mod):
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle_mod.f16_bits_to_f64(bits)
    want = bits.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def test_f16_decoder_golden_constants(oracle_mod):
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        h, v = line.split()
        got = oracle_mod.f16_bits_to_f64(np.array([int(h, 16)], dtype=np.uint16))[0]
        want = float(v)
        assert got == want and np.signbit(got) == np.signbit(want), (h, got, want)


def test_f32_c0_decoder(oracle_mod):
    # K = 0 makes the oracle return C0 decoded: compare with numpy's widening.
    rng = np.random.default_rng(3)
    bits = rng.integers(0, 2**32, size=(64, 257), dtype=np.uint64).astype(np.uint32)
    bits[0, :8] = [0, 0x80000000, 1, 0x007fffff, 0x00800000, 0x7f7fffff, 0x3f800000, 0x80000001]
    C0 = bits.view(np.float32)
    A = np.zeros((64, 0), dtype=np.float16)
    B = np.zeros((0, 257), dtype=np.float16)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    want = C0.astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(Cref), nan)
    assert np.array_equal(Cref[~nan], want[~nan])
    assert np.all(S == 0)


def _interesting_doubles(rng, n, lo_exp, hi_exp):
    e = rng.integers(lo_exp, hi_exp, size=n)
    m = rng.uniform(1.0, 2.0, size=n)
    s = rng.choice([-1.0, 1.0], size=n)
    return s * np.ldexp(m, e)


def test_encoder_f16_matches_numpy(oracle_mod):
    rng = np.random.default_rng(5)
    x = _interesting_doubles(rng, 200000, -30, 18)
    # every midpoint between neighbouring binary16 values, and its neighbours
    allh = np.arange(0, 0x7c00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mid = (allh[:-1] + allh[1:]) / 2
    x = np.concatenate([x, mid, -mid, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf),
                        allh, [65504.0, 65519.99, 65520.0, 65536.0, 1e6, -1e6, 0.0, -0.0,
                               2.0**-25, np.nextafter(2.0**-25, 1), 2.0**-26, np.inf, -np.inf]])
    got = oracle_mod.round_to_f16(x)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_encoder_f32_matches_numpy(oracle_mod):
    rng = np.random.default_rng(6)
    x = _interesting_doubles(rng, 200000, -160, 130)
    f = rng.integers(0, 0x7f800000 - 1, size=20000, dtype=np.int64).astype(np.uint32)
    lo = f.view(np.float32).astype(np.float64)
    hi = (f + 1).astype(np.uint32).view(np.float32).astype(np.float64)
    mid = (lo + hi) / 2
    x = np.concatenate([x, mid, -mid, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf), lo,
                        [0.0, -0.0, np.inf, -np.inf, 3.5e38, 1e-46, 2.0**-150]])
    got = oracle_mod.round_to_f32(x)
    with np.errstate(over="ignore"):
        want = x.astype(np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_identity_gives_b_plus_c0(oracle_mod):
    n = 96
    _, B, C0 = wl.make_inputs(n, 70, n, "uniform", "uniform", seed=1)
    A = np.eye(n, dtype=np.float16)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    assert np.array_equal(Cref, B.astype(np.float64) + C0.astype(np.float64))
    assert np.array_equal(S, np.abs(B.astype(np.float64)))


def test_permutation_moves_rows(oracle_mod):
    rng = np.random.default_rng(2)
    n = 77
    perm = rng.permutation(n)
    A = np.zeros((n, n), dtype=np.float16)
    A[np.arange(n), perm] = 1
    _, B, C0 = wl.make_inputs(n, 53, n, "uniform", "zeros", seed=4)
    Cref, _ = oracle_mod.gemm_f16(A, B, C0)
    assert np.array_equal(Cref, B.astype(np.float64)[perm])


def test_right_permutation_moves_columns(oracle_mod):
    rng = np.random.default_rng(8)
    n = 41
    perm = rng.permutation(n)
    B = np.zeros((n, n), dtype=np.float16)
    B[perm, np.arange(n)] = 1          # column j of A B is column perm[j] of A
    A, _, C0 = wl.make_inputs(29, n, n, "uniform", "zeros", seed=9)
    Cref, _ = oracle_mod.gemm_f16(A, B, C0)
    assert np.array_equal(Cref, A.astype(np.float64)[:, perm])


def test_all_ones_gives_k(oracle_mod):
    M, N, K = 13, 17, 1000
    A = np.ones((M, K), np.float16)
    B = np.ones((K, N), np.float16)
    C0 = np.full((M, N), 0.25, np.float32)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    assert np.all(Cref == K + 0.25)
    assert np.all(S == K)


def test_index_product_closed_form(oracle_mod):
    M, N, K = 40, 37, 19
    A = np.repeat(np.arange(M, dtype=np.float16)[:, None], K, axis=1)       # A[i,k] = i
    B = np.repeat(np.arange(N, dtype=np.float16)[None, :], K, axis=0)       # B[k,j] = j
    C0 = np.zeros((M, N), np.float32)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    want = K * np.outer(np.arange(M), np.arange(N)).astype(np.float64)
    assert np.array_equal(Cref, want) and np.array_equal(S, want)


def test_rank_one_outer_product(oracle_mod):
    A, B, C0 = wl.make_inputs(50, 60, 1, "uniform", "uniform", seed=11)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    a = A.astype(np.float64)
    b = B.astype(np.float64)
    assert np.array_equal(Cref, C0.astype(np.float64) + a * b)   # one exact product, one add
    assert np.array_equal(S, np.abs(a) * np.abs(b))


def test_asymmetric_operands_not_transposed(oracle_mod):
    # A = e_0 e_1^T (one entry), B = e_1 e_2^T: A B = e_0 e_2^T.  A swapped or
    # transposed operand puts the 1 elsewhere or gives 0.
    A = np.zeros((3, 4), np.float16); A[0, 1] = 3
    B = np.zeros((4, 5), np.float16); B[1, 2] = 5
    Cref, S = oracle_mod.gemm_f16(A, B, np.zeros((3, 5), np.float32))
    want = np.zeros((3, 5)); want[0, 2] = 15
    assert np.array_equal(Cref, want) and np.array_equal(S, want)


@pytest.mark.parametrize("M,N,K,seed", [(1, 1, 1, 0), (2, 3, 4, 1), (5, 4, 8, 2), (8, 8, 8, 3), (3, 7, 5, 4)])
@pytest.mark.parametrize("c_dtype", [np.float32, np.float16])
def test_exact_rational_brute_force(oracle_mod, M, N, K, seed, c_dtype):
    # inputs in [-1, 1]: every partial sum fits 53 bits, so the binary64 result
    # must equal the exact rational one.  Loop order here is i, j, k.
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=seed, c_dtype=c_dtype)
    if c_dtype == np.float32:
        C0 = (np.round(C0.astype(np.float64) * 2**24) / 2**24).astype(np.float32)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    for i in range(M):
        for j in range(N):
            acc = Fraction(float(C0[i, j]))
            mag = Fraction(0)
            for k in range(K):
                p = Fraction(float(A[i, k])) * Fraction(float(B[k, j]))
                acc += p
                mag += abs(p)
            assert Fraction(float(Cref[i, j])) == acc
            assert Fraction(float(S[i, j])) == mag


@pytest.mark.parametrize("M,N,K", [(33, 65, 129), (128, 96, 300), (7, 513, 64)])
def test_integer_inputs_equal_numpy_f64_matmul(oracle_mod, M, N, K):
    A, B, _ = wl.make_inputs(M, N, K, "int2", "zeros", seed=21)
    rng = np.random.default_rng(22)
    C0 = rng.integers(-8, 9, size=(M, N)).astype(np.float32)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    Ad, Bd = A.astype(np.float64), B.astype(np.float64)
    assert np.array_equal(Cref, Ad @ Bd + C0)
    assert np.array_equal(S, np.abs(Ad) @ np.abs(Bd))


def test_general_inputs_close_to_numpy_f64_matmul(oracle_mod):
    M, N, K = 64, 80, 777
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=23)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    Ad, Bd = A.astype(np.float64), B.astype(np.float64)
    want = Ad @ Bd + C0.astype(np.float64)
    bound = K * 2.0**-52 * (np.abs(Ad) @ np.abs(Bd) + np.abs(C0))
    assert np.all(np.abs(Cref - want) <= bound)
    assert np.all(np.abs(S - np.abs(Ad) @ np.abs(Bd)) <= bound)


def test_power_of_two_scaling_is_exact(oracle_mod):
    A, B, C0 = wl.make_inputs(31, 45, 200, "uniform", "zeros", seed=31)
    C1, S1 = oracle_mod.gemm_f16(A, B, C0)
    C4, S4 = oracle_mod.gemm_f16((A * np.float16(4)).astype(np.float16), B, C0)
    assert np.array_equal(C4, 4 * C1) and np.array_equal(S4, 4 * S1)


def test_transpose_identity_on_integers(oracle_mod):
    A, B, _ = wl.make_inputs(23, 35, 57, "int2", "zeros", seed=33)
    C0 = np.zeros((23, 35), np.float32)
    C1, _ = oracle_mod.gemm_f16(A, B, C0)
    C2, _ = oracle_mod.gemm_f16(np.ascontiguousarray(B.T), np.ascontiguousarray(A.T),
                                np.ascontiguousarray(C0.T))
    assert np.array_equal(C1.T, C2)


def test_magnitude_sum_dominates(oracle_mod):
    A, B, C0 = wl.make_inputs(40, 40, 333, "uniform", "uniform", seed=35)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    assert np.all(S >= np.abs(Cref - C0.astype(np.float64)) - 1e-12)
    # S is the same sum taken over absolute values
    Cabs, _ = oracle_mod.gemm_f16(np.abs(A), np.abs(B), np.zeros_like(C0))
    assert np.array_equal(S, Cabs)


def test_subnormal_inputs_are_honoured(oracle_mod):
    # A holds binary16 subnormals m * 2^-24, B powers of two: exact closed form.
    m = np.arange(1, 65, dtype=np.uint16)
    A = m.view(np.float16).reshape(8, 8)
    B = np.diag(np.array([1, 2, 4, 8, 16, 32, 64, 128], dtype=np.float16))
    Cref, _ = oracle_mod.gemm_f16(A, B, np.zeros((8, 8), np.float32))
    want = m.reshape(8, 8).astype(np.float64) * 2.0**-24 * np.array([1, 2, 4, 8, 16, 32, 64, 128.0])
    assert np.array_equal(Cref, want)


def test_leading_dimensions_and_nan_padding(oracle_mod):
    M, N, K = 19, 23, 29
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=41)
    Ap, Bp, Cp = wl.make_inputs(M, N, K, "uniform", "uniform", seed=41, lda=K + 3, ldb=N + 8, ldc=N + 1)
    assert np.array_equal(A, Ap) and Ap.strides[0] == (K + 3) * 2
    C1, S1 = oracle_mod.gemm_f16(A, B, C0)
    C2, S2 = oracle_mod.gemm_f16(Ap, Bp, Cp)
    assert np.array_equal(C1, C2) and np.array_equal(S1, S2)
    assert not np.isnan(C2).any()


def test_row_subset_equals_full(oracle_mod):
    A, B, C0 = wl.make_inputs(100, 64, 50, "uniform", "uniform", seed=43)
    Cf, Sf = oracle_mod.gemm_f16(A, B, C0)
    rows = wl.sample_rows(100, 12, 32, seed=1)
    assert rows[0] == 0 and rows[-1] == 99 and len(set(rows.tolist())) == len(rows)
    Cs, Ss = oracle_mod.gemm_f16(A, B, C0, rows=rows)
    assert np.array_equal(Cs, Cf[rows]) and np.array_equal(Ss, Sf[rows])


def test_f16_c0_path(oracle_mod):
    A, B, C0 = wl.make_inputs(16, 16, 16, "int2", "uniform", seed=45, c_dtype=np.float16)
    Cref, _ = oracle_mod.gemm_f16(A, B, C0)
    assert np.array_equal(Cref, A.astype(np.float64) @ B.astype(np.float64) + C0.astype(np.float64))


def test_empty_problems(oracle_mod):
    for M, N, K in [(0, 5, 3), (5, 0, 3), (0, 0, 0)]:
        Cref, S = oracle_mod.gemm_f16(np.zeros((M, K), np.float16), np.zeros((K, N), np.float16),
                                      np.zeros((M, N), np.float32))
        assert Cref.shape == (M, N) and S.shape == (M, N)


def test_error_codes(oracle_mod):
    lib = ctypes.CDLL(oracle_mod.build())
    i64, vp = ctypes.c_int64, ctypes.c_void_p
    f = lib.oracle_gemm_f16
    f.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, ctypes.c_int, vp, vp]
    f.restype = ctypes.c_int
    buf = np.zeros(64, np.float64)
    p = buf.ctypes.data
    assert f(-1, 2, 2, p, 2, p, 2, p, 2, 0, p, p) == -1
    assert f(2, 2, 2, p, 1, p, 2, p, 2, 0, p, p) == -2
    assert f(2, 2, 2, p, 2, p, 1, p, 2, 0, p, p) == -2
    assert f(2, 2, 2, p, 2, p, 2, p, 1, 0, p, p) == -2
    assert f(2, 2, 2, None, 2, p, 2, p, 2, 0, p, p) == -3
    assert f(2, 2, 2, p, 2, p, 2, p, 2, 0, p, p) == 0


# ---- the fused epilogue step (bias per column, ReLU) ----------------------------
def test_bias_act_closed_forms(oracle_mod):
    """Pins that do not retype the formula: hand-written values, exact rational
    arithmetic element by element, and special values."""
    C = np.array([[1.5, -2.0, 0.25], [-0.5, 4.0, -8.0]])
    bias = np.array([-1.0, 0.5, 8.0], dtype=np.float32)
    assert np.array_equal(oracle_mod.bias_act(C, bias, False), [[0.5, -1.5, 8.25], [-1.5, 4.5, 0.0]])
    assert np.array_equal(oracle_mod.bias_act(C, bias, True), [[0.5, 0.0, 8.25], [0.0, 4.5, 0.0]])
    assert np.array_equal(oracle_mod.bias_act(C, None, True), [[1.5, 0.0, 0.25], [0.0, 4.0, 0.0]])
    assert np.array_equal(oracle_mod.bias_act(C, None, False), C)
    # the bias belongs to the column, not the row: a transposed-operand slip fails here
    wide = oracle_mod.bias_act(np.zeros((3, 4)), np.array([1.0, 2.0, 3.0, 4.0]), False)
    assert np.array_equal(wide, np.tile([1.0, 2.0, 3.0, 4.0], (3, 1)))
    # exact rationals, other loop order
    rng = np.random.default_rng(4)
    Cr = rng.integers(-64, 65, size=(5, 7)) / 8.0
    b16 = (rng.integers(-64, 65, size=7) / 16.0).astype(np.float16)
    got = oracle_mod.bias_act(Cr, b16, True)
    for j in range(7):
        for i in range(5):
            v = Fraction(float(Cr[i, j])) + Fraction(float(b16[j]))
            assert Fraction(float(got[i, j])) == (v if v >= 0 else 0)
    # NaN and -0 pass through ReLU, +/-inf behave as numbers
    s = oracle_mod.bias_act(np.array([[np.nan, -0.0, np.inf, -np.inf]]), None, True)
    assert np.isnan(s[0, 0]) and s[0, 1] == 0 and np.signbit(s[0, 1]) and s[0, 2] == np.inf and s[0, 3] == 0
    # input is not modified
    assert C[0, 1] == -2.0


def test_bias_act_composes_with_gemm(oracle_mod):
    """relu(C0 + A B + bias) on integer inputs against numpy's exact float64 matmul."""
    A, B, C0 = wl.make_inputs(24, 40, 16, "int2", "zeros", seed=11)
    C0[:] = np.arange(24 * 40).reshape(24, 40) % 5 - 2
    bias = (np.arange(40) % 7 - 3).astype(np.float32)
    Cref, _ = oracle_mod.gemm_f16(A, B, C0)
    want = np.maximum(A.astype(np.float64) @ B.astype(np.float64) + C0 + bias[None, :], 0.0)
    assert np.array_equal(oracle_mod.bias_act(Cref, bias, True), want)


# ---- the literal binary16-accumulating reading (a numerical comparison, not the parity reference) ----

def test_rounding_every_slice_closed_forms(oracle_mod):
    rng = np.random.default_rng(21)
    A = rng.integers(-2, 3, (24, 96)).astype(np.float16)
    B = rng.integers(-2, 3, (96, 40)).astype(np.float16)
    C0 = rng.integers(-4, 5, (24, 40)).astype(np.float16)
    # small integers: every partial sum is a binary16 value, so no rounding happens at any slice width
    exact = A.astype(np.int64) @ B.astype(np.int64) + C0.astype(np.int64)
    for w in (1, 16, 32, 96):
        assert np.array_equal(oracle_mod.gemm_f16_rounding_every_slice(A, B, C0, w), exact.astype(np.float64))
    # one slice over the whole k range = one rounding of the exact result
    A = rng.uniform(-1, 1, (16, 80)).astype(np.float16)
    B = rng.uniform(-1, 1, (80, 24)).astype(np.float16)
    C0 = rng.uniform(-1, 1, (16, 24)).astype(np.float16)
    Cref, _ = oracle_mod.gemm_f16(A, B, C0)
    assert np.array_equal(oracle_mod.gemm_f16_rounding_every_slice(A, B, C0, 80), oracle_mod.round_to_f16(Cref).astype(np.float64))
    # 2049 ones: 2048 + 1 is a tie in binary16 and goes to even (2048) when every product is rounded in
    ones = np.ones((1, 2049), np.float16)
    assert oracle_mod.gemm_f16_rounding_every_slice(ones, ones.T.copy(), np.zeros((1, 1), np.float16), 1)[0, 0] == 2048.0
    assert oracle_mod.round_to_f16(oracle_mod.gemm_f16(ones, ones.T.copy(), np.zeros((1, 1), np.float16))[0])[0, 0] == 2048.0  # 2049 -> tie -> 2048
    ones = np.ones((1, 2051), np.float16)           # 2051 rounds to 2052 in one rounding; one at a time it never leaves 2048
    assert oracle_mod.round_to_f16(oracle_mod.gemm_f16(ones, ones.T.copy(), np.zeros((1, 1), np.float16))[0])[0, 0] == 2052.0
    assert oracle_mod.gemm_f16_rounding_every_slice(ones, ones.T.copy(), np.zeros((1, 1), np.float16), 1)[0, 0] == 2048.0


def test_round_on_store_is_the_more_accurate_reading(oracle_mod):
    """Both readings of the half-precision mode stay inside 4e-3 * sum|a||b| on the
    headline's data; rounding at every 16-deep slice loses about ten times more."""
    K = 4096
    A, B, C0 = wl.make_inputs(40, 48, K, "normal_rsqrtk", "zeros", seed=2, c_dtype=np.float16)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    once = np.abs(oracle_mod.round_to_f16(Cref).astype(np.float64) - Cref) / S
    sliced = np.abs(oracle_mod.gemm_f16_rounding_every_slice(A, B, C0, 16) - Cref) / S
    assert once.max() <= 2.0 ** -11 and sliced.max() <= 4e-3
    assert sliced.max() > 3 * once.max() and sliced.mean() > 3 * once.mean()
