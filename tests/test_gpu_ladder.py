"""GPU parity of the comparison kernels and ablation rows that only the ladder build of
the library holds (libgemm_f16_ladder.so: the plain ring-buffered tiling at 128 x 128 and
256 x 256, the same without the LDS swizzle, the phase-alternating kernel on 32x32x16
MFMAs and without the XCD-aware tile order, the four-wavefront kernel, the kernel whose
wavefronts all multiply all the time, C moved in every k step).  None of them is ever
selected; each is forced by name and held to the same bars as the product's kernels."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2108_13191_amd import binding, workloads as wl   # noqa: E402
from gpu_util import run_gemm, assert_close, config_id       # noqa: E402

CDT = {"f32": np.float32, "f16": np.float16}
ROWS = ["t128x128x64_w2x2", "t256x256x64_w2x4", "t256x256x64_w2x4_noswz", "pp256x256x64_w2x4",
        "pp256x256x64_w2x4_mi16_noxcd", "pp192x192x64_w2x4_mi16", "pp256x256x64_w2x4_mi16_rowwise", "w4_256x256x64", "il256x256x64_w2x4_mi16", "generic64x64x32_c_in_loop",
        "generic64x64x32_f16_round_per_slice"]
SHAPES = [(64, 64, 64), (300, 264, 200), (520, 776, 136), (257, 8, 8), (1, 520, 72), (130, 136, 1000),
          (513, 264, 64), (256, 256, 8), (1100, 1296, 448)]


@pytest.fixture(autouse=True)
def _ladder_library():
    with binding.library("ladder"):
        binding.force_config(-1)
        yield
        binding.force_config(-1)


def test_the_ladder_appends_to_the_product_table():
    with binding.library("product"):
        product = [binding.describe_config(i)["name"] for i in range(binding.num_configs())]
    ladder = [binding.describe_config(i)["name"] for i in range(binding.num_configs())]
    assert ladder[:len(product)] == product and set(ROWS) <= set(ladder[len(product):])
    # selection is the product's: nothing the ladder adds is ever chosen
    for M, N, K in [(8192, 8192, 8192), (1024, 1024, 1024), (16384, 3072, 768), (4000, 4000, 4000), (300, 264, 200)]:
        q = binding.query_config(0, M, N, K, 256, K, 256, N, 256, N)
        with binding.library("product"):
            assert q == binding.query_config(0, M, N, K, 256, K, 256, N, 256, N)


@pytest.mark.parametrize("name", ROWS)
@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_tolerance(oracle_mod, name, mode):
    cfg = config_id(name)
    assert binding.force_config(cfg) == 0
    for idx, (M, N, K) in enumerate(SHAPES):
        A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=500 + idx, c_dtype=CDT[mode])
        assert binding.query_config(mode == "f16", M, N, K, 16, K, 16, N, 16, N)["id"] == cfg
        got = run_gemm(A, B, C0, mode)
        Cref, S = oracle_mod.gemm_f16(A, B, C0)
        assert_close(got, Cref, S, C0, mode, what=f"{name} {(M, N, K)} {mode}")


@pytest.mark.parametrize("name", ROWS)
@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_integers_bit_exact(oracle_mod, name, mode):
    assert binding.force_config(config_id(name)) == 0
    for idx, (M, N, K) in enumerate([(300, 264, 200), (512, 512, 256), (96, 1032, 448)]):
        A, B, _ = wl.make_inputs(M, N, K, "int2", "zeros", seed=600 + idx)
        C0 = np.random.default_rng(idx).integers(-4, 5, size=(M, N)).astype(CDT[mode])
        got = run_gemm(A, B, C0, mode)
        Cref, _ = oracle_mod.gemm_f16(A, B, C0)
        want = oracle_mod.round_to_f32(Cref) if mode == "f32" else oracle_mod.round_to_f16(Cref)
        assert np.array_equal(got, want), f"{name} ints {(M, N, K)} {mode}"


def test_rows_that_change_no_arithmetic_give_the_product_kernels_bits(oracle_mod):
    """Tile order and LDS placement do not enter the sums: without the XCD-aware order the
    256 x 256 kernel, and without the swizzle the plain tiling, return the same bits."""
    M, N, K = 1300, 1544, 320
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=77)
    out = {}
    for name in ("pp256x256x64_w2x4_mi16", "pp256x256x64_w2x4_mi16_noxcd", "t256x256x64_w2x4", "t256x256x64_w2x4_noswz"):
        binding.force_config(config_id(name))
        out[name] = run_gemm(A, B, C0, "f32")
    assert np.array_equal(out["pp256x256x64_w2x4_mi16"], out["pp256x256x64_w2x4_mi16_noxcd"])
    assert np.array_equal(out["t256x256x64_w2x4"], out["t256x256x64_w2x4_noswz"])


def test_f16_running_sum_rounded_every_16_k_matches_the_literal_reading(oracle_mod):
    """The ladder row that rounds the running sum to binary16 after every 16-deep k slice against
    the oracle's function for that reading of the paper's half-precision mode: bit for bit where
    every slice sum is exact in f32 (integers, incl. sums beyond 2048, where binary16 rounds and
    ties go to even), and on random data inside the f16 bar against the exact result, close to
    the literal oracle (the matrix unit adds a slice in f32, the oracle exactly: a slice sum can
    land on the other side of a binary16 rounding boundary now and then)."""
    binding.force_config(config_id("generic64x64x32_f16_round_per_slice"))
    # all ones: the running sum walks 16, 32, ... and sticks at 2048 + ties
    for K in (2064, 4096):
        A = np.ones((64, K), np.float16)
        B = np.ones((K, 72), np.float16)
        C0 = np.zeros((64, 72), np.float16)
        C0[:, 1] = 1.0                     # odd running sums: ties on the way
        got = run_gemm(A, B, C0, "f16")
        want = oracle_mod.gemm_f16_rounding_every_slice(A, B, C0)
        assert np.array_equal(got.astype(np.float64), want), f"all ones, K = {K}"
    A, B, C0 = wl.make_inputs(200, 136, 2000, "int2", "int2", seed=9, c_dtype=np.float16)
    got = run_gemm(A, B, C0, "f16")
    want = oracle_mod.gemm_f16_rounding_every_slice(A, B, C0)
    assert np.array_equal(got.astype(np.float64), want), "integers -2..2, K = 2000"
    worst_lit, worst_ref = 0.0, 0.0
    for K in (1024, 8192):
        A, B, C0 = wl.make_inputs(130, 136, K, "normal_rsqrtk", "zeros", seed=K, c_dtype=np.float16)
        got = run_gemm(A, B, C0, "f16").astype(np.float64)
        Cref, S = oracle_mod.gemm_f16(A, B, C0)
        lit = oracle_mod.gemm_f16_rounding_every_slice(A, B, C0)
        assert np.all(np.abs(got - Cref) <= 4e-3 * S)
        worst_ref = max(worst_ref, float(np.max(np.abs(got - Cref) / S)))
        worst_lit = max(worst_lit, float(np.max(np.abs(got - lit) / S)))
        assert np.mean(got == lit) > 0.9 and np.all(np.abs(got - lit) <= 1e-3 * S)
    print(f"per-slice rounding on the GPU: worst |C - C_ref| / S = {worst_ref:.2e}, worst |C - literal oracle| / S = {worst_lit:.2e}")


def test_the_four_wavefront_ladder_kernel_has_no_fused_epilogue():
    binding.force_config(config_id("w4_256x256x64"))
    dev = torch.device("cuda:0")
    A = torch.zeros(256, 64, dtype=torch.float16, device=dev)
    B = torch.zeros(64, 256, dtype=torch.float16, device=dev)
    C = torch.zeros(256, 256, dtype=torch.float32, device=dev)
    bias = torch.ones(256, dtype=torch.float32, device=dev)
    rc = binding.gemm_f16_f32acc_bias_act(256, 256, 64, A, 64, B, 256, C, 256, bias, binding.ACT_NONE, 0)
    torch.cuda.synchronize()
    assert rc == binding.ERR_CONFIG and float(C.abs().max()) == 0.0
