"""GPU parity of the kernel that keeps two accumulator sets per wavefront and
sends a finished tile to C while the next one is multiplied (256 x 128 tiles,
one workgroup per compute unit, k a multiple of 64 with at least 9 k steps).
Shapes: one tile, fewer tiles than compute units, one to five tiles per
workgroup, ragged edges in both directions, the minimum and longer k loops;
both C types, integers bit-exact, the same bits as the plain 256 x 256 tiling,
fused epilogue, k loops it does not take.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2108_13191_amd import binding, workloads as wl   # noqa: E402
from gpu_util import run_gemm, assert_close                  # noqa: E402

CDT = {"f32": np.float32, "f16": np.float16}
NAME = "ov256x128x64_w2x4_mi16"


def _id(name=NAME):
    return [i for i in range(binding.num_configs()) if binding.describe_config(i)["name"] == name][0]


@pytest.fixture(autouse=True)
def _ladder_library():
    # the kernel is a comparison row: it lives in the ladder build of the library
    with binding.library("ladder"):
        binding.force_config(-1)
        yield
        binding.force_config(-1)


# tiles of 256 x 128: 1, 15, 260 (two for 4 workgroups), 512, 1080, 1320
SHAPES = [(256, 128, 576), (700, 520, 576), (3328, 2560, 640), (4096, 4096, 576), (6000, 5704, 768), (5000, 8440, 1024)]


@pytest.mark.parametrize("mode", ["f32", "f16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_tolerance(oracle_mod, mode, shape):
    M, N, K = shape
    assert binding.force_config(_id()) == 0
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=K + M, c_dtype=CDT[mode])
    q = binding.query_config(mode == "f16", M, N, K, 16, K, 16, N, 16, N)
    assert q["name"] == NAME and q["grid"] == min(256, ((M + 255) // 256) * ((N + 127) // 128))
    got = run_gemm(A, B, C0, mode)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    assert_close(got, Cref, S, C0, mode, what=f"{NAME} {shape} {mode}")


@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_integers_bit_exact(oracle_mod, mode):
    M, N, K = 6000, 5704, 768
    assert binding.force_config(_id()) == 0
    A, B, C0 = wl.make_inputs(M, N, K, "int2", "int2", seed=3, c_dtype=CDT[mode])
    got = run_gemm(A, B, C0, mode)
    Cref, _ = oracle_mod.gemm_f16(A, B, C0)
    want = oracle_mod.round_to_f32(Cref) if mode == "f32" else oracle_mod.round_to_f16(Cref)
    u = np.uint16 if mode == "f16" else np.uint32
    assert np.array_equal(got.view(u), want.view(u))


@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_same_bits_as_plain_tiling(mode):
    """Same products, same k order, same final addition: bit-identical to the 256 x 256 kernel."""
    M, N, K = 5000, 4360, 768
    A, B, C0 = wl.make_inputs(M, N, K, "normal_rsqrtk", "uniform", seed=11, c_dtype=CDT[mode])
    binding.force_config(_id("pp256x256x64_w2x4_mi16"))
    want = run_gemm(A, B, C0, mode)
    binding.force_config(_id())
    got = run_gemm(A, B, C0, mode)
    u = np.uint16 if mode == "f16" else np.uint32
    assert np.array_equal(got.view(u), want.view(u))


def test_run_twice_same_bits():
    M, N, K = 4100, 3000, 896
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=4, c_dtype=np.float32)
    binding.force_config(_id())
    a = run_gemm(A, B, C0, "f32")
    b = run_gemm(A, B, C0, "f32")
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_fused_epilogue(oracle_mod, mode):
    M, N, K = 6000, 5704, 768
    assert binding.force_config(_id()) == 0
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=5, c_dtype=CDT[mode])
    bias = np.random.default_rng(9).uniform(-1, 1, N).astype(CDT[mode])
    dev = torch.device("cuda:0")
    dA, dB, dC, db = (torch.from_numpy(x).to(dev) for x in (A, B, C0, bias))
    fn = binding.gemm_f16_f32acc_bias_act if mode == "f32" else binding.gemm_f16_f16acc_bias_act
    binding.check(fn(M, N, K, dA, dA.stride(0), dB, dB.stride(0), dC, dC.stride(0), db,
                     binding.ACT_RELU, torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    want = oracle_mod.bias_act(Cref, bias, True)
    got = dC.cpu().numpy().astype(np.float64)
    tol = 1e-5 if mode == "f32" else 4e-3
    assert np.all(np.abs(got - want) <= tol * (S + np.abs(C0.astype(np.float64)) + np.abs(bias.astype(np.float64))[None, :]) + 1e-30)


def test_other_k_loops_are_passed_on(oracle_mod):
    """Forced onto a problem with a k tail or fewer than 9 k steps the configuration hands
    the call to the plain 256 x 256 kernel."""
    binding.force_config(_id())
    for K in (512, 584):
        A, B, C0 = wl.make_inputs(300, 264, K, "uniform", "uniform", seed=1, c_dtype=np.float32)
        got = run_gemm(A, B, C0, "f32")
        Cref, S = oracle_mod.gemm_f16(A, B, C0)
        assert_close(got, Cref, S, C0, "f32", what=f"K={K}")
