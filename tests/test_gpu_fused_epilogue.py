"""GPU parity of the fused epilogue entry points (per-column bias, ReLU) against
the CPU oracle: act(C0 + A B + bias) in binary64.  Bars as for the plain entry
points: bit-exact on integer-valued inputs; otherwise
|C - C_ref| <= tol * (sum_k|a||b| + |c0| + |bias|) elementwise (ReLU is
1-Lipschitz, the bias adds one more f32 rounding)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2108_13191_amd import binding, workloads as wl   # noqa: E402
from gpu_util import DevMat, TOL                             # noqa: E402

CDT = {"f32": np.float32, "f16": np.float16}
CONFIGS = list(range(binding.num_configs()))


@pytest.fixture(autouse=True)
def _auto_config():
    binding.force_config(-1)
    yield
    binding.force_config(-1)


def run_fused(A, B, C0, bias, act, mode, ldc=None, expect=binding.OK):
    M, K = A.shape
    N = B.shape[1]
    dA, dB, dC = DevMat(A, nan_canary=True), DevMat(B, nan_canary=True), DevMat(C0, ldc)
    dbias = None if bias is None else DevMat(bias.reshape(1, -1), offset=3, nan_canary=True)      # element-aligned only
    fn = binding.gemm_f16_f32acc_bias_act if mode == "f32" else binding.gemm_f16_f16acc_bias_act
    rc = fn(M, N, K, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld, None if dbias is None else dbias.ptr, act,
            torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert rc == expect, f"return code {rc} ({binding.strerror(rc)})"
    if dbias is not None:
        dbias.fetch()                                                            # canaries around the bias intact
    return dC.fetch()


def check(oracle_mod, A, B, C0, bias, act, mode, exact=False, what="", **kw):
    got = run_fused(A, B, C0, bias, act, mode, **kw)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    want = oracle_mod.bias_act(Cref, bias, act == binding.ACT_RELU)
    if exact:
        w = oracle_mod.round_to_f32(want) if mode == "f32" else oracle_mod.round_to_f16(want)
        bits = np.uint32 if mode == "f32" else np.uint16
        assert np.array_equal(got.view(bits), w.view(bits)), f"{what}: not bit-exact"
        return
    bound = TOL[mode] * (S + np.abs(C0.astype(np.float64)) + (0 if bias is None else np.abs(bias.astype(np.float64))[None, :]))
    err = np.abs(got.astype(np.float64) - want)
    bad = ~(err <= bound)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} out of tolerance, worst {np.nanmax(err - bound):.3e}"
    if act == binding.ACT_RELU:
        assert (got >= 0).all() and not np.signbit(got[want > bound]).any()


SHAPES = [(320, 264, 200), (513, 520, 72), (256, 768, 128), (1000, 1000, 1000)]


@pytest.mark.parametrize("cfg", CONFIGS)
@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_each_config_bias_relu(oracle_mod, cfg, mode):
    binding.force_config(cfg)
    for si, (M, N, K) in enumerate(SHAPES):
        A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=20 + si, c_dtype=CDT[mode])
        bias = np.random.default_rng(si).uniform(-4, 4, size=N).astype(CDT[mode])
        check(oracle_mod, A, B, C0, bias, binding.ACT_RELU, mode, what=f"cfg{cfg} {M}x{N}x{K} {mode}")


@pytest.mark.parametrize("cfg", CONFIGS)
@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_each_config_integers_bit_exact(oracle_mod, cfg, mode):
    binding.force_config(cfg)
    M, N, K = 384, 520, 136
    A, B, C0 = wl.make_inputs(M, N, K, "int2", "zeros", seed=31, c_dtype=CDT[mode])
    C0[:] = np.arange(M * N).reshape(M, N) % 9 - 4
    bias = (np.arange(N) % 11 - 5).astype(CDT[mode])
    for act in (binding.ACT_NONE, binding.ACT_RELU):
        check(oracle_mod, A, B, C0, bias, act, mode, exact=True, what=f"cfg{cfg} act{act} {mode}")
    check(oracle_mod, A, B, C0, None, binding.ACT_RELU, mode, exact=True, what=f"cfg{cfg} relu only {mode}")


@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_unaligned_shapes_and_pitches(oracle_mod, mode):
    rng = np.random.default_rng(77)
    for _ in range(6):
        M, N, K = (int(x) for x in rng.integers(1, 300, size=3))
        A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=int(rng.integers(1 << 30)), c_dtype=CDT[mode])
        bias = rng.uniform(-2, 2, size=N).astype(CDT[mode])
        check(oracle_mod, A, B, C0, bias, binding.ACT_RELU, mode, ldc=N + int(rng.integers(0, 9)), what=f"{M}x{N}x{K} {mode}")


def test_no_bias_no_act_equals_plain_entry_point():
    A, B, C0 = wl.make_inputs(512, 512, 256, "uniform", "uniform", seed=2)
    fused = run_fused(A, B, C0, None, binding.ACT_NONE, "f32")
    dA, dB, dC = DevMat(A, nan_canary=True), DevMat(B, nan_canary=True), DevMat(C0)
    binding.check(binding.gemm_f16_f32acc(512, 512, 256, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld, 0))
    torch.cuda.synchronize()
    assert np.array_equal(fused.view(np.uint32), dC.fetch().view(np.uint32))


def test_k_zero_applies_the_epilogue_to_c(oracle_mod):
    M, N = 70, 45
    C0 = np.random.default_rng(5).uniform(-3, 3, size=(M, N)).astype(np.float32)
    bias = np.random.default_rng(6).uniform(-1, 1, size=N).astype(np.float32)
    A = np.zeros((M, 0), np.float16); B = np.zeros((0, N), np.float16)
    got = run_fused(A, B, C0, bias, binding.ACT_RELU, "f32")
    want = oracle_mod.round_to_f32(oracle_mod.bias_act(C0.astype(np.float64), bias, True))
    assert np.allclose(got, want, rtol=0, atol=1e-6)


def test_relu_passes_nan_and_keeps_infinities():
    A = np.zeros((64, 64), np.float16); B = np.zeros((64, 64), np.float16)
    C0 = np.zeros((64, 64), np.float32)
    C0[0, 0], C0[0, 1], C0[0, 2], C0[0, 3] = np.nan, np.inf, -np.inf, -5.0
    got = run_fused(A, B, C0, None, binding.ACT_RELU, "f32")
    assert np.isnan(got[0, 0]) and got[0, 1] == np.inf and got[0, 2] == 0 and got[0, 3] == 0


def test_errors():
    A, B, C0 = wl.make_inputs(64, 64, 64, "uniform", "zeros", seed=1)
    run_fused(A, B, C0, None, 7, "f32", expect=binding.ERR_CONFIG)            # unknown activation
    dA, dB, dC = DevMat(A, nan_canary=True), DevMat(B, nan_canary=True), DevMat(C0)
    rc = binding.gemm_f16_f32acc_bias_act(64, 64, 64, dA.ptr, 64, dB.ptr, 64, dC.ptr, 64, dC.ptr + 2, 0, 0)
    assert rc == binding.ERR_ALIGN                                             # f32 bias on a 2-byte boundary


def test_fused_epilogue_on_a_row_split_plan(oracle_mod):
    """Both launches of a split plan apply the same bias and activation."""
    M, N, K = 5000, 5120, 192
    q = binding.query_config(False, M, N, K, 256, K, 256, N, 256, N)
    assert 0 < q["split_rows"] < M
    A, B, C0 = wl.make_inputs(M, N, K, "int1", "zeros", seed=71)
    C0[:] = (np.arange(M)[:, None] * 3 + np.arange(N)[None, :]) % 7 - 3
    bias = (np.arange(N) % 13 - 6).astype(np.float32)
    check(oracle_mod, A, B, C0, bias, binding.ACT_RELU, "f32", exact=True, what="fused + row split")
