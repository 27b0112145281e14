"""GPU parity: the HIP library (through its C ABI) against the CPU oracle,
element by element on the same seeded inputs.

Bars: bit-exact on integer-valued inputs; otherwise
|C - C_ref| <= 1e-5 * sum_k|a||b| (f32 accumulate) and <= 4e-3 * sum_k|a||b|
(f16 accumulate), elementwise.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2108_13191_amd import binding, workloads as wl   # noqa: E402
from gpu_util import run_gemm, assert_close, config_id, TOL   # noqa: E402

CDT = {"f32": np.float32, "f16": np.float16}
ALL_CONFIGS = list(range(binding.num_configs()))


@pytest.fixture(autouse=True)
def _auto_config():
    binding.force_config(-1)
    yield
    binding.force_config(-1)


def _check(oracle_mod, A, B, C0, mode, literal=False, exact=False, what="", **kw):
    got = run_gemm(A, B, C0, mode, **kw)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    if exact:
        want = oracle_mod.round_to_f32(Cref) if mode == "f32" else oracle_mod.round_to_f16(Cref)
        assert np.array_equal(got.view(np.uint16 if mode == "f16" else np.uint32),
                              want.view(np.uint16 if mode == "f16" else np.uint32)), f"{what}: not bit-exact"
        return 0.0
    return assert_close(got, Cref, S, C0, mode, literal=literal, what=what)


# ---- the named small workloads ---------------------------------------------

def test_sq256_uniform_f32(oracle_mod):
    A, B, C0 = wl.workload_inputs("sq256_uniform", "f32")
    _check(oracle_mod, A, B, C0, "f32", literal=True, what="256^3 uniform")


@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_sq256_integers_bit_exact(oracle_mod, mode):
    A, B, C0 = wl.workload_inputs("sq256_int", mode)
    _check(oracle_mod, A, B, C0, mode, exact=True, what="256^3 integers")


@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_sq1024_uniform_nonzero_c(oracle_mod, mode):
    A, B, C0 = wl.workload_inputs("sq1024_uniform", mode)
    r = _check(oracle_mod, A, B, C0, mode, literal=True, what="1024^3 uniform")
    print(f"1024^3 {mode}: max err/bound {r:.3f}")


# ---- every kernel configuration on shapes with several tiles and ragged edges

SHAPES = [(64, 64, 64), (300, 264, 200), (520, 776, 136), (257, 8, 8), (1, 520, 72), (130, 136, 1000),
          (513, 264, 64), (256, 256, 8)]


@pytest.mark.parametrize("cfg", ALL_CONFIGS)
@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_each_config_tolerance(oracle_mod, cfg, mode):
    assert binding.force_config(cfg) == 0
    for idx, (M, N, K) in enumerate(SHAPES):
        A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=100 + idx, c_dtype=CDT[mode])
        used = binding.query_config(mode == "f16", M, N, K, 16, K, 16, N, 16, N)["id"]
        assert used == cfg
        _check(oracle_mod, A, B, C0, mode, what=f"cfg {cfg} shape {(M, N, K)}")


@pytest.mark.parametrize("cfg", ALL_CONFIGS)
@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_each_config_integers_bit_exact(oracle_mod, cfg, mode):
    assert binding.force_config(cfg) == 0
    for idx, (M, N, K) in enumerate([(300, 264, 200), (512, 512, 256), (96, 1032, 448)]):
        A, B, _ = wl.make_inputs(M, N, K, "int2", "zeros", seed=200 + idx)
        rng = np.random.default_rng(idx)
        C0 = rng.integers(-4, 5, size=(M, N)).astype(CDT[mode])      # |C| <= 4*448 + 4 < 2048
        _check(oracle_mod, A, B, C0, mode, exact=True, what=f"cfg {cfg} ints {(M, N, K)}")


@pytest.mark.parametrize("cfg", ALL_CONFIGS)
def test_identity_and_permutation(oracle_mod, cfg):
    binding.force_config(cfg)
    n = 384
    rng = np.random.default_rng(5)
    perm = rng.permutation(n)
    P = np.zeros((n, n), np.float16)
    P[np.arange(n), perm] = 1
    _, B, C0 = wl.make_inputs(n, 328, n, "uniform", "zeros", seed=6)
    got = run_gemm(P, B, C0, "f32")
    assert np.array_equal(got, B.astype(np.float32)[perm])          # one non-zero product per element: exact
    # with a non-zero C0 the single product is added to it inside the matrix
    # unit, whose internal rounding is the hardware's own: the f32 bar applies
    _, B, C0 = wl.make_inputs(n, 328, n, "uniform", "uniform", seed=6)
    got = run_gemm(P, B, C0, "f32")
    Cref, S = oracle_mod.gemm_f16(P, B, C0)
    assert_close(got, Cref, S, C0, "f32", what="permutation with C0")
    A, _, C0 = wl.make_inputs(200, n, n, "uniform", "zeros", seed=7)
    got = run_gemm(A, P, C0, "f32")
    inv = np.argsort(perm)
    assert np.array_equal(got, A.astype(np.float32)[:, inv])


# ---- unaligned shapes, pitches and base pointers (any-shape kernel) ----------

def test_shape_fuzz_unaligned(oracle_mod):
    rng = np.random.default_rng(2024)
    worst = 0.0
    for it in range(48):
        M, N, K = (int(x) for x in rng.integers(1, 301, size=3))
        if it % 6 == 0:
            M, N, K = [(1, 1, 1), (3, 5, 7), (127, 129, 131), (299, 1, 299), (1, 300, 1), (64, 65, 33),
                       (33, 64, 65), (257, 257, 257)][it // 6]
        mode = "f32" if it % 2 == 0 else "f16"
        lda, ldb, ldc = K + int(rng.integers(0, 9)), N + int(rng.integers(0, 9)), N + int(rng.integers(0, 9))
        offs = tuple(int(x) for x in rng.integers(0, 4, size=3))
        A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=300 + it, c_dtype=CDT[mode])
        worst = max(worst, _check(oracle_mod, A, B, C0, mode, what=f"fuzz {it} {(M, N, K)} ld {(lda, ldb, ldc)} offs {offs}",
                                  lda=lda, ldb=ldb, ldc=ldc, offs=offs))
    print(f"fuzz worst err/bound {worst:.3f}")


def test_aligned_pitches_keep_tuned_path(oracle_mod):
    # pitches that are multiples of 8 but larger than the row: tuned kernels, strided rows
    for cfg in ALL_CONFIGS[1:]:
        binding.force_config(cfg)
        M, N, K = 270, 200, 328
        A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=400 + cfg)
        assert binding.query_config(0, M, N, K, 16, K + 8, 16, N + 24, 16, N + 3)["id"] == cfg
        _check(oracle_mod, A, B, C0, "f32", what=f"cfg {cfg} strided", lda=K + 8, ldb=N + 24, ldc=N + 3,
               offs=(8, 16, 1))


def test_subnormal_inputs(oracle_mod):
    # binary16 subnormals times powers of two: every product and sum is exact in f32
    for cfg in ALL_CONFIGS:
        binding.force_config(cfg)
        M = N = K = 64
        m = (np.arange(M * K, dtype=np.uint32) % 1023 + 1).astype(np.uint16)
        A = m.view(np.float16).reshape(M, K)
        B = np.zeros((K, N), np.float16)
        B[np.arange(K), (np.arange(K) * 7) % N] = np.float16(2.0) ** (np.arange(K) % 8)
        C0 = np.zeros((M, N), np.float32)
        _check(oracle_mod, A, B, C0, "f32", exact=True, what=f"cfg {cfg} subnormals")


def test_k_zero_and_empty():
    C0 = np.arange(12, dtype=np.float32).reshape(3, 4)
    got = run_gemm(np.zeros((3, 0), np.float16), np.zeros((0, 4), np.float16), C0, "f32")
    assert np.array_equal(got, C0)
    run_gemm(np.zeros((0, 5), np.float16), np.zeros((5, 4), np.float16), np.zeros((0, 4), np.float32), "f32")
    run_gemm(np.zeros((3, 5), np.float16), np.zeros((5, 0), np.float16), np.zeros((3, 0), np.float16), "f16")


def test_f16_store_rounds_once_to_nearest_even():
    # K = 1: C0 + a*b is exact in f32, so the f16 result is one rounding of it.
    a = np.array([[1.0], [1.0], [3.0], [-1.0]], np.float16)
    b = np.array([[2.0**-11, 3 * 2.0**-11, 2.0**-11, 2.0**-11]], np.float16)
    C0 = np.array([[1.0, 1.0, 2048.0, 65504.0]] * 4, np.float16)
    got = run_gemm(a, b, C0, "f16")
    exact = C0.astype(np.float64) + a.astype(np.float64) * b.astype(np.float64)
    with np.errstate(over="ignore"):
        want = exact.astype(np.float16)      # numpy rounds binary64 -> binary16 once, ties to even
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_overflow_to_infinity_in_f16_mode():
    A = np.full((8, 8), 256.0, np.float16)
    B = np.full((8, 8), 256.0, np.float16)
    got = run_gemm(A, B, np.zeros((8, 8), np.float16), "f16")      # 8 * 65536 > 65504
    assert np.all(np.isinf(got)) and np.all(got > 0)


def test_same_call_twice_same_bits():
    for cfg in ALL_CONFIGS:
        binding.force_config(cfg)
        A, B, C0 = wl.make_inputs(777, 520, 1096, "uniform", "uniform", seed=9)
        r1 = run_gemm(A, B, C0, "f32")
        r2 = run_gemm(A, B, C0, "f32")
        assert np.array_equal(r1.view(np.uint32), r2.view(np.uint32))


def test_non_default_stream(oracle_mod):
    A, B, C0 = wl.make_inputs(300, 264, 200, "uniform", "uniform", seed=11)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        got = run_gemm(A, B, C0, "f32")
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    assert_close(got, Cref, S, C0, "f32")


def test_two_streams_concurrently(oracle_mod):
    """Two different problems enqueued on two streams without ordering between
    them: the library keeps no per-call state, so both must come out right."""
    from gpu_util import DevMat
    cases = []
    for seed, (M, N, K) in enumerate([(1536, 1280, 2048), (1100, 2056, 1544)]):
        A, B, C0 = wl.make_inputs(M, N, K, "int2", "zeros", seed=40 + seed)
        cases.append((A, B, C0, DevMat(A, nan_canary=True), DevMat(B, nan_canary=True), DevMat(C0), torch.cuda.Stream()))
    torch.cuda.synchronize()
    for _ in range(3):
        for A, B, C0, dA, dB, dC, s in cases:
            M, K = A.shape
            binding.check(binding.gemm_f16_f32acc(M, B.shape[1], K, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld, s.cuda_stream))
    torch.cuda.synchronize()
    for A, B, C0, dA, dB, dC, s in cases:
        Cref, _ = oracle_mod.gemm_f16(A, B, C0)
        assert np.array_equal(dC.fetch(), oracle_mod.round_to_f32(3.0 * Cref))      # integer data: exact


@pytest.mark.parametrize("shape", [(1024, 1032, 520), (72, 520, 4096)])
def test_under_hip_graph_capture(oracle_mod, shape):
    """The entry points only enqueue kernels (no allocation, no synchronisation,
    no memset), so a call can be captured into a HIP graph; every replay, with
    eager work and synchronisations in between, must equal the eager result.  The second
    shape runs with its k loop cut into parts that add to C atomically."""
    from gpu_util import DevMat
    M, N, K = shape
    A, B, C0 = wl.make_inputs(M, N, K, "int2", "zeros", seed=50)
    dA, dB, dC = DevMat(A, nan_canary=True), DevMat(B, nan_canary=True), DevMat(C0)
    Cref, _ = oracle_mod.gemm_f16(A, B, C0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                  # warm-up outside capture, as torch asks
        binding.check(binding.gemm_f16_f32acc(M, N, K, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld, side.cuda_stream))
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rc = binding.gemm_f16_f32acc(M, N, K, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld,
                                     torch.cuda.current_stream().cuda_stream)
    assert rc == binding.OK
    torch.cuda.synchronize()
    assert np.array_equal(dC.fetch(), oracle_mod.round_to_f32(1.0 * Cref))          # capture itself ran nothing
    for rep in range(2, 5):
        g.replay()
        torch.cuda.synchronize()
        scratch = torch.ones(1 << 20, device="cuda").sum().item()  # eager work between replays
        assert scratch == float(1 << 20)
        assert np.array_equal(dC.fetch(), oracle_mod.round_to_f32(float(rep) * Cref)), f"replay {rep - 1}"


@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_row_split_plan(oracle_mod, mode):
    """A problem the selector runs as two launches (whole rounds of 256 x 256 tiles
    on the first rows, another configuration on the rest): every element against
    the oracle, bit-exact on integer inputs, ragged last rows included."""
    M, N, K = 5000, 5120, 192
    q = binding.query_config(mode == "f16", M, N, K, 256, K, 256, N, 256, N)
    assert 0 < q["split_rows"] < M and q["id2"] >= 0, q
    A, B, C0 = wl.make_inputs(M, N, K, "int1", "zeros", seed=61, c_dtype=CDT[mode])
    C0[:] = (np.arange(M)[:, None] + np.arange(N)[None, :]) % 5 - 2
    _check(oracle_mod, A, B, C0, mode, exact=True, what=f"row split {q}")
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=62, c_dtype=CDT[mode])
    _check(oracle_mod, A, B, C0, mode, what=f"row split {q}")


# ---- NaN and infinities through the plain entry points -------------------------

def _class_of(x):
    """0 finite, 1 +inf, 2 -inf, 3 NaN."""
    x = np.asarray(x, dtype=np.float64)
    return np.where(np.isnan(x), 3, np.where(np.isposinf(x), 1, np.where(np.isneginf(x), 2, 0)))


@pytest.mark.parametrize("mode", ["f32", "f16"])
@pytest.mark.parametrize("name", ["pp256x256x64_w2x4_mi16", "pp128x128x64_w2x4_mi16", "t64x64x64_w2x2", "generic64x64x32"])
def test_nan_and_inf_propagate_like_ieee(oracle_mod, name, mode):
    """NaN and +-inf inside A, B and C0 reach exactly the outputs the definition says (the
    oracle's binary64 sum gives the class of every element: NaN where a NaN or inf - inf or
    0 * inf enters the sum, an infinity where only one sign of infinity does); all other
    outputs meet the tolerance.  A k tail (K = 200) and ragged edges: zero-filled padding
    must not meet a NaN or an infinity."""
    binding.force_config(config_id(name))
    M, N, K = 300, 264, 200
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=31, c_dtype=CDT[mode])
    A[5, 17] = np.nan                    # a NaN row of results
    A[40, 199] = np.inf                  # in the k tail's last element: +-inf by the sign of B[199, j]
    B[0, 7] = -np.inf                    # a column: -inf * A[i, 0]
    A[41, 3] = np.inf
    B[3, 9] = 0.0                        # inf * 0 = NaN at (41, 9)
    C0[77, 100] = np.inf
    C0[78, 101] = np.nan
    A[299, 0] = np.inf                   # last row (edge tile) times the -inf column: (299, 7) = inf * -inf = -inf
    got = run_gemm(A, B, C0, mode)
    with np.errstate(invalid="ignore", over="ignore"):
        Cref, S = oracle_mod.gemm_f16(A, B, C0)
    want_cls, got_cls = _class_of(Cref), _class_of(got)
    if mode == "f16":                    # finite sums beyond the f16 range become infinities on the store
        with np.errstate(over="ignore", invalid="ignore"):
            want_cls = _class_of(Cref.astype(np.float16))
    assert np.array_equal(got_cls, want_cls), np.argwhere(got_cls != want_cls)[:5]
    assert want_cls[5].min() == 3 and want_cls[41, 9] == 3 and want_cls[299, 7] == 2 and want_cls[77, 100] == 1
    fin = want_cls == 0
    with np.errstate(invalid="ignore"):
        err = np.abs(got.astype(np.float64) - Cref)[fin]
    bound = (TOL[mode] * (S + np.abs(C0.astype(np.float64))))[fin]
    assert np.all(err <= bound)


# ---- the late start of every other XCD on the one-workgroup-per-tile launches --------

@pytest.mark.parametrize("mode", ["f32", "f16"])
@pytest.mark.parametrize("case", [("pp256x256x64_w2x4_mi16", (8448, 8192, 128)),      # 1056 tiles, K a multiple of 64
                                  ("pp256x256x64_w2x4_mi16", (8300, 8200, 200)),      # 1089 tiles, ragged, k tail
                                  ("pp128x128x64_w2x4_mi16", (5900, 5640, 72))])      # 2115 tiles (two per compute unit at once)
def test_late_started_plain_launches(oracle_mod, case, mode):
    """Four or more rounds of workgroups and K <= 2048: the workgroups that begin with the
    launch on every other XCD wait about 12 us first.  Results must not depend on it."""
    name, (M, N, K) = case
    binding.force_config(config_id(name))
    A, B, C0 = wl.make_inputs(M, N, K, "int2", "int2", seed=K, c_dtype=CDT[mode])
    got = run_gemm(A, B, C0, mode)
    Cref, _ = oracle_mod.gemm_f16(A, B, C0)
    want = oracle_mod.round_to_f32(Cref) if mode == "f32" else oracle_mod.round_to_f16(Cref)
    assert np.array_equal(got, want), f"{name} {(M, N, K)} {mode}"
