"""GPU parity of what is particular to the two kernels with an assembly k loop (four wavefronts of
128 x 128 on a 256 x 256 tile: the long-k kernel; of 64 x 64 on a 128 x 128 tile over five LDS
stages): leaving the loop at each of its exits, C read inside the loop, and where the selector
takes them.  The tests over all configurations (test_gpu_parity.py,
test_gpu_fused_epilogue.py) cover it like every other product kernel."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2108_13191_amd import binding, workloads as wl   # noqa: E402
from gpu_util import run_gemm, assert_close, config_id       # noqa: E402

CDT = {"f32": np.float32, "f16": np.float16}
NAME = "w4a_256x256x64"
NAME128 = "w4a_128x128x64"


@pytest.fixture(autouse=True)
def _unforce():
    binding.force_config(-1)
    yield
    binding.force_config(-1)


def test_assembly_k_loop_at_every_exit_of_its_six_step_body(oracle_mod):
    """The assembly k loop is unrolled six k steps deep and can leave
    after any of them: 1 to 14 full k steps (two trips and more), with and without a k tail,
    on several tiles with ragged edges; integers, so every bit counts."""
    binding.force_config(config_id(NAME))
    for steps in range(1, 15):
        for tail in (0, 24):
            M, N, K = 300, 520, 64 * steps + tail
            A, B, _ = wl.make_inputs(M, N, K, "int2", "zeros", seed=900 + steps)
            C0 = np.random.default_rng(steps).integers(-4, 5, size=(M, N)).astype(np.float32)
            got = run_gemm(A, B, C0, "f32")
            Cref, _ = oracle_mod.gemm_f16(A, B, C0)
            assert np.array_equal(got, oracle_mod.round_to_f32(Cref)), f"K = {K}"


def test_c_read_inside_the_assembly_loop(oracle_mod):
    """In f32 mode, with enough full k steps (a few dozen), the long-k kernel reads C during its
    first k steps and adds it to the running sums there, through range-checked buffer loads, and
    stores through the same view of C.  Shapes with interior and edge tiles side by side, edge
    tiles whose wavefront blocks lie inside, across and outside C's border (160, 88, 44 and 8 of
    256 rows or columns inside C), 40 to 51 full k steps, with and without a k tail, a C pitch
    that is not N: integers bit for bit (and nothing outside C written: the helper compares the
    canaries around it), random data to tolerance (both modes: f16 takes the path that adds C
    behind the loop)."""
    binding.force_config(config_id(NAME))
    for idx, (M, N, K) in enumerate([(256, 256, 2560), (512, 768, 2624), (600, 520, 2688 + 24), (256, 512, 3264), (768, 300, 2816), (416, 672, 2560)]):
        A, B, _ = wl.make_inputs(M, N, K, "int2", "zeros", seed=950 + idx)
        C0 = np.random.default_rng(idx).integers(-4, 5, size=(M, N)).astype(np.float32)
        got = run_gemm(A, B, C0, "f32", ldc=N + 8 * idx)
        Cref, _ = oracle_mod.gemm_f16(A, B, C0)
        assert np.array_equal(got, oracle_mod.round_to_f32(Cref)), f"ints {(M, N, K)}"
        for mode in ("f32", "f16"):
            A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=960 + idx, c_dtype=CDT[mode])
            got = run_gemm(A, B, C0, mode)
            Cref, S = oracle_mod.gemm_f16(A, B, C0)
            assert_close(got, Cref, S, C0, mode, what=f"w4a, C in the loop {(M, N, K)} {mode}")


def test_selected_for_long_k_loops_and_right_there(oracle_mod):
    """K >= 12288 on whole 256 x 256 tiles (and K >= 8192 at no more than one tile per compute
    unit) goes to this kernel under automatic selection; sampled rows of such a problem
    against the oracle, both modes."""
    M, N, K = 4096, 4096, 8192
    for mode in ("f32", "f16"):
        q = binding.query_config(mode == "f16", M, N, K, 16, K, 16, N, 16, N)
        assert q["name"] == NAME, q
        A, B, C0 = wl.make_inputs(M, N, K, "normal_rsqrtk", "uniform", seed=31, c_dtype=CDT[mode])
        got = run_gemm(A, B, C0, mode)
        rows = np.array([0, 1, 127, 128, 255, 256, 300, 511, 2047, 2048, 4095])
        Cref, S = oracle_mod.gemm_f16(A, B, C0, rows=rows)
        assert_close(got[rows], Cref, S, C0[rows], mode, what=f"long k, auto {mode}")
    assert binding.query_config(0, 8192, 8192, 8192, 16, 8192, 16, 8192, 16, 8192)["name"].endswith("_chain")
    for n in (12288, 16384):
        assert binding.query_config(0, n, n, n, 16, n, 16, n, 16, n)["name"] == NAME


def test_five_stage_k_loop_at_every_exit(oracle_mod):
    """The 128 x 128 kernel's assembly k loop is unrolled five k steps deep (one per LDS stage),
    with copies four k steps ahead: 1 to 14 full k steps, with and without a k tail, several
    tiles with ragged edges, both modes; integers."""
    binding.force_config(config_id(NAME128))
    for steps in range(1, 15):
        for tail in (0, 24):
            M, N, K = 300, 264, 64 * steps + tail
            A, B, _ = wl.make_inputs(M, N, K, "int2", "zeros", seed=700 + steps)
            for mode in ("f32", "f16"):
                C0 = np.random.default_rng(steps).integers(-4, 5, size=(M, N)).astype(CDT[mode])
                got = run_gemm(A, B, C0, mode)
                Cref, _ = oracle_mod.gemm_f16(A, B, C0)
                want = oracle_mod.round_to_f32(Cref) if mode == "f32" else Cref.astype(np.float16)
                assert np.array_equal(got, want), f"K = {K} {mode}"


def test_five_stage_kernel_selected_for_few_tiles_and_a_long_k_loop(oracle_mod):
    """At most one 128 x 128 tile per compute unit and K >= 6144: the five-stage kernel; sampled
    rows of such a problem against the oracle, both modes."""
    M, N, K = 2048, 1920, 6144
    for mode in ("f32", "f16"):
        q = binding.query_config(mode == "f16", M, N, K, 16, K, 16, N, 16, N)
        assert q["name"] == NAME128, q
        A, B, C0 = wl.make_inputs(M, N, K, "normal_rsqrtk", "uniform", seed=41, c_dtype=CDT[mode])
        got = run_gemm(A, B, C0, mode)
        rows = np.array([0, 1, 63, 64, 127, 128, 300, 1023, 1024, 2047])
        Cref, S = oracle_mod.gemm_f16(A, B, C0, rows=rows)
        assert_close(got[rows], Cref, S, C0[rows], mode, what=f"five stages, auto {mode}")
    for k in (2048, 4096):
        assert binding.query_config(0, 2048, 2048, k, 16, k, 16, 2048, 16, 2048)["name"].startswith("pp128x128")
    assert binding.query_config(0, 2048, 4096, 8192, 16, 8192, 16, 4096, 16, 4096)["name"] != NAME128
    assert binding.query_config(0, 256, 7168, 7168, 16, 7168, 16, 7168, 16, 7168)["name"] == NAME128      # a strip of 112 tiles


def test_split_k_plans_of_skinny_problems(oracle_mod):
    """Few 128 x 128 tiles and a long k loop, f32 mode: the k loop is cut into parts of at least
    16 k steps (as many as keep the additions under four million), one workgroup of the
    five-stage kernel per tile and part, which add to C atomically.  Integers bit for bit (any order of exact additions), random data to tolerance,
    with a k tail, ragged edges, a C pitch that is not N; the same problems in f16 mode and
    with a fused epilogue run unsplit."""
    from gpu_util import DevMat
    cases = [((16, 1024, 2048), 2), ((100, 520, 4096 + 24), 4), ((300, 264, 8192), 8), ((64, 8192, 8192), 4), ((256, 512, 16384 + 8), 16)]
    for idx, ((M, N, K), parts) in enumerate(cases):
        tiles = ((M + 127) // 128) * ((N + 127) // 128)
        q = binding.query_config(False, M, N, K, 16, K, 16, N, 16, N + 8 * idx)
        assert q["name"] == NAME128 and q["grid"] == tiles * parts, (M, N, K, q)
        assert binding.query_config(True, M, N, K, 16, K, 16, N, 16, N)["grid"] <= max(tiles, ((M + 63) // 64) * ((N + 63) // 64))
        A, B, _ = wl.make_inputs(M, N, K, "int2", "zeros", seed=1100 + idx)
        C0 = np.random.default_rng(idx).integers(-4, 5, size=(M, N)).astype(np.float32)
        got = run_gemm(A, B, C0, "f32", ldc=N + 8 * idx)
        Cref, _ = oracle_mod.gemm_f16(A, B, C0)
        assert np.array_equal(got, oracle_mod.round_to_f32(Cref)), f"ints {(M, N, K)}"
        for mode in ("f32", "f16"):
            A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=1110 + idx, c_dtype=CDT[mode])
            got = run_gemm(A, B, C0, mode, ldc=N + 8 * idx)
            Cref, S = oracle_mod.gemm_f16(A, B, C0)
            assert_close(got, Cref, S, C0, mode, what=f"split k {(M, N, K)} {mode}")
    # a fused epilogue on such a problem: one pass over k, bias and ReLU behind it
    M, N, K = 100, 520, 4096
    A, B, _ = wl.make_inputs(M, N, K, "int2", "zeros", seed=1150)
    C0 = np.random.default_rng(5).integers(-4, 5, size=(M, N)).astype(np.float32)
    bias = (np.arange(N) % 7 - 3).astype(np.float32)
    dA, dB, dC, dbias = DevMat(A, nan_canary=True), DevMat(B, nan_canary=True), DevMat(C0), torch.from_numpy(bias).cuda()
    binding.check(binding.gemm_f16_f32acc_bias_act(M, N, K, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld, dbias, binding.ACT_RELU, 0))
    torch.cuda.synchronize()
    Cref, _ = oracle_mod.gemm_f16(A, B, C0)
    assert np.array_equal(dC.fetch(), np.maximum(oracle_mod.round_to_f32(Cref) + bias[None, :], 0).astype(np.float32))


def test_split_k_on_random_skinny_shapes(oracle_mod):
    """Seeded random skinny problems (1 to 500 rows, 8 to 2048 columns, K up to 16384 with and without
    a k tail) under automatic selection, f32 mode and the f16 mode with a workspace: sampled rows
    against the oracle, integers bit for bit; most of them run with a split k loop."""
    rng = np.random.default_rng(4242)
    split = 0
    for idx in range(14):
        M = int(rng.integers(1, 500))
        N = int(rng.integers(1, 257)) * 8
        K = int(rng.integers(256, 2049)) * 8
        tiles = ((M + 127) // 128) * ((N + 127) // 128)
        q = binding.query_config(False, M, N, K, 16, K, 16, N, 16, N)
        split += q["name"] == NAME128 and q["grid"] > tiles
        A, B, _ = wl.make_inputs(M, N, K, "int2", "zeros", seed=1400 + idx)
        C0 = rng.integers(-4, 5, size=(M, N)).astype(np.float32)
        rows = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, size=min(M, 12))]))
        Cref, _ = oracle_mod.gemm_f16(A, B, C0, rows=rows)
        got = run_gemm(A, B, C0, "f32")
        assert np.array_equal(got[rows], oracle_mod.round_to_f32(Cref)), f"f32 {(M, N, K)} {q['name']} grid {q['grid']}"
        # the f16 mode through the workspace entry point (also where no workspace is needed)
        from gpu_util import DevMat
        C16 = C0.astype(np.float16)
        need = binding.gemm_f16_f16acc_workspace_bytes(M, N, K)
        ws = torch.full((max(need // 4, 4),), float("nan"), device="cuda")
        dA, dB, dC = DevMat(A, nan_canary=True), DevMat(B, nan_canary=True), DevMat(C16)
        binding.check(binding.gemm_f16_f16acc_workspace(M, N, K, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld, ws, need, 0))
        torch.cuda.synchronize()
        Cref16, _ = oracle_mod.gemm_f16(A, B, C16, rows=rows)
        assert np.array_equal(dC.fetch()[rows], Cref16.astype(np.float16)), f"f16 workspace {(M, N, K)} need {need}"
    assert split >= 8, split


def test_split_k_leaves_special_values_of_c_alone():
    """Parts that sum to zero do not touch C: subnormal f32 values, signed zeros, infinities and
    NaN in C come back bit for bit from a split-k problem whose product is zero."""
    M, N, K = 64, 520, 4096
    assert binding.query_config(False, M, N, K, 16, K, 16, N, 16, N)["grid"] > ((M + 127) // 128) * ((N + 127) // 128)
    A = np.zeros((M, K), np.float16)
    B = wl.make_inputs(M, N, K, "uniform", "zeros", seed=5)[1]
    C0 = np.zeros((M, N), np.float32)
    C0.view(np.uint32)[:] = np.random.default_rng(3).integers(0, 1 << 20, size=(M, N), dtype=np.uint32)      # subnormals
    C0[0, :6] = [np.inf, -np.inf, np.nan, -0.0, 0.0, np.float32(1e-45)]
    got = run_gemm(A, B, C0, "f32")
    assert np.array_equal(got.view(np.uint32), C0.view(np.uint32))


def test_split_k_propagates_nan_and_infinities(oracle_mod):
    """Infinities and NaN in A, B and C reach the same results through a split k loop as through
    one pass: the class of every result (finite, +inf, -inf, NaN) equals the oracle's, the finite
    ones are within tolerance."""
    M, N, K = 100, 520, 4096
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=77)
    A[5, 17] = np.nan                    # a NaN row of results
    A[40, 4095] = np.inf                 # in the last part: +-inf by the sign of B[4095, j]
    B[0, 7] = -np.inf                    # a column: -inf * A[i, 0] (first part)
    A[41, 3] = np.inf
    B[3, 9] = 0.0                        # inf * 0 = NaN at (41, 9)
    A[42, 10] = np.inf
    A[42, 3000] = -np.inf                # +inf from one part, -inf from another: NaN in the columns where B has one sign in both rows
    C0[77, 100] = np.inf
    C0[78, 101] = np.nan
    got = run_gemm(A, B, C0, "f32")
    with np.errstate(invalid="ignore", over="ignore"):
        Cref, S = oracle_mod.gemm_f16(A, B, C0)

    def cls(x):
        x = np.asarray(x, dtype=np.float64)
        return np.where(np.isnan(x), 3, np.where(np.isposinf(x), 1, np.where(np.isneginf(x), 2, 0)))
    want_cls, got_cls = cls(Cref), cls(got)
    assert np.array_equal(got_cls, want_cls), np.argwhere(got_cls != want_cls)[:5]
    assert want_cls[5].min() == 3 and want_cls[41, 9] == 3 and want_cls[77, 100] == 1 and (want_cls[42] == 3).any()
    fin = want_cls == 0
    with np.errstate(invalid="ignore"):
        err = np.abs(got.astype(np.float64) - Cref)[fin]
    assert np.all(err <= (1e-5 * (S + np.abs(C0.astype(np.float64))))[fin])


def test_half_precision_mode_with_a_workspace(oracle_mod):
    """gemm_f16_f16acc_workspace: with M x N floats of scratch memory the skinny problems that the
    f32 mode cuts along k are cut in the f16 mode too (the parts add to the zeroed workspace, a last
    pass rounds C + workspace once).  Integers bit for bit against the oracle's one rounding, random
    data to the mode's tolerance, a C pitch that is not N, a workspace that holds garbage before;
    without a workspace, or with one that is too small, the call runs unsplit with the same result."""
    from gpu_util import DevMat
    cases = [(16, 1024, 2048), (100, 520, 4096 + 24), (300, 264, 8192), (64, 2048, 4096)]
    for idx, (M, N, K) in enumerate(cases):
        need = binding.gemm_f16_f16acc_workspace_bytes(M, N, K)
        assert need == M * N * 4, (M, N, K, need)
        ws = torch.full((need // 4 + 4,), float("nan"), device="cuda")
        for dist, exact in (("int2", True), ("uniform", False)):
            A, B, C0 = wl.make_inputs(M, N, K, dist, "zeros" if exact else "uniform", seed=1200 + idx, c_dtype=np.float16)
            if exact:
                C0 = np.random.default_rng(idx).integers(-4, 5, size=(M, N)).astype(np.float16)
            Cref, S = oracle_mod.gemm_f16(A, B, C0)
            for ws_bytes in (need, need - 4, 0):
                dA, dB, dC = DevMat(A, nan_canary=True), DevMat(B, nan_canary=True), DevMat(C0, N + 8 * idx, 1)
                ws.fill_(float("nan"))
                binding.check(binding.gemm_f16_f16acc_workspace(M, N, K, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld,
                                                                ws if ws_bytes else 0, ws_bytes, 0))
                torch.cuda.synchronize()
                got = dC.fetch()
                if exact:
                    assert np.array_equal(got, Cref.astype(np.float16)), f"ints {(M, N, K)} workspace {ws_bytes}"
                else:
                    assert_close(got, Cref, S, C0, "f16", what=f"workspace {(M, N, K)} {ws_bytes}")
    # nothing to gain: no workspace asked for, and a workspace changes nothing
    assert binding.gemm_f16_f16acc_workspace_bytes(4096, 4096, 4096) == 0
    assert binding.gemm_f16_f16acc_workspace_bytes(16, 1024, 512) == 0
    ws = torch.zeros(64, device="cuda")
    A, B, C0 = wl.make_inputs(64, 64, 64, "int2", "zeros", seed=3, c_dtype=np.float16)
    dA, dB, dC = DevMat(A), DevMat(B), DevMat(C0)
    assert binding.gemm_f16_f16acc_workspace(64, 64, 64, dA.ptr, 64, dB.ptr, 64, dC.ptr, 64, ws.data_ptr() + 4, 252, 0) == binding.ERR_ALIGN
