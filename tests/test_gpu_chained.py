"""GPU parity of the two launch forms that only differ from the plain 256 x 256
tiling when a compute unit gets several tiles: one workgroup per unit walking
its tiles (a tile's first operands requested before the epilogue of the tile
before it), and the form whose first workgroups on every other unit take half a
tile.  Both fall back to the plain tiling on small problems, so the shapes here
have more than two tiles per compute unit of an MI355X (256 units), with short
k loops so that the oracle stays quick: k tails, one and two k steps, ragged
edges in both directions, both C types, fused epilogue.
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


def _ids():
    names = {binding.describe_config(i)["name"]: i for i in range(binding.num_configs())}
    return names["pp256x256x64_w2x4_mi16_chain"], names["pp256x256x64_w2x4_mi16_stag"]


@pytest.fixture(autouse=True)
def _auto_config():
    binding.force_config(-1)
    yield
    binding.force_config(-1)


# (M, N, K): 552 / 600 / 792 / 520 / 552 / 1188 tiles of 256 x 256 (three and more per compute unit: the chained
# form then also starts every other XCD late)
SHAPES = [(6000, 5704, 200), (6144, 6400, 128), (8440, 5896, 40), (5120, 6656, 64), (6100, 5640, 328), (9000, 8200, 136)]


@pytest.mark.parametrize("which", [0, 1])
@pytest.mark.parametrize("mode", ["f32", "f16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_tolerance(oracle_mod, which, mode, shape):
    cfg = _ids()[which]
    M, N, K = shape
    assert binding.force_config(cfg) == 0
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=7 + K, c_dtype=CDT[mode])
    q = binding.query_config(mode == "f16", M, N, K, 16, K, 16, N, 16, N)
    assert q["id"] == cfg
    # the chained form runs one workgroup per compute unit, the staggered one 128 more than there are tiles
    tiles = ((M + 255) // 256) * ((N + 255) // 256)
    assert q["grid"] == (tiles + 128 if which else 256), q
    got = run_gemm(A, B, C0, mode)
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    assert_close(got, Cref, S, C0, mode, what=f"cfg {cfg} {shape} {mode}")


@pytest.mark.parametrize("which", [0, 1])
@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_integers_bit_exact(oracle_mod, which, mode):
    cfg = _ids()[which]
    M, N, K = 6000, 5704, 200
    assert binding.force_config(cfg) == 0
    A, B, C0 = wl.make_inputs(M, N, K, "int2", "int2", seed=3, c_dtype=CDT[mode])
    got = run_gemm(A, B, C0, mode)
    Cref, _ = oracle_mod.gemm_f16(A, B, C0)
    want = oracle_mod.round_to_f32(Cref) if mode == "f32" else oracle_mod.round_to_f16(Cref)
    u = np.uint16 if mode == "f16" else np.uint32
    assert np.array_equal(got.view(u), want.view(u))


@pytest.mark.parametrize("which", [0, 1])
def test_same_bits_as_plain_tiling(which):
    """Tile contents do not depend on who computes them or when: the result is
    bit-identical to the plain 256 x 256 tiling's."""
    cfg = _ids()[which]
    M, N, K = 6100, 5640, 328
    A, B, C0 = wl.make_inputs(M, N, K, "normal_rsqrtk", "uniform", seed=11, c_dtype=np.float32)
    plain = [i for i in range(binding.num_configs()) if binding.describe_config(i)["name"] == "pp256x256x64_w2x4_mi16"][0]
    binding.force_config(plain)
    want = run_gemm(A, B, C0, "f32")
    binding.force_config(cfg)
    got = run_gemm(A, B, C0, "f32")
    # (the staggered form's half tiles use the 128-row kernel: same products, same k order within a row)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("which", [0, 1])
def test_fused_epilogue(oracle_mod, which):
    cfg = _ids()[which]
    M, N, K = 6000, 5704, 72
    assert binding.force_config(cfg) == 0
    A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=5, c_dtype=np.float32)
    bias = np.random.default_rng(9).uniform(-1, 1, N).astype(np.float32)
    dev = torch.device("cuda:0")
    dA, dB, dC, db = (torch.from_numpy(x).to(dev) for x in (A, B, C0, bias))
    binding.check(binding.gemm_f16_f32acc_bias_act(M, N, K, dA, dA.stride(0), dB, dB.stride(0), dC, dC.stride(0), db,
                                                   binding.ACT_RELU, torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    Cref, S = oracle_mod.gemm_f16(A, B, C0)
    want = oracle_mod.bias_act(Cref, bias, True)
    got = dC.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - want) <= 1e-5 * (S + np.abs(C0) + np.abs(bias)[None, :]) + 1e-30)


def test_chained_and_late_started_launch_under_hip_graph_capture(oracle_mod):
    """A problem the selector runs chained with every other XCD started late (three tiles per
    compute unit, short k loop), captured into a HIP graph: every replay, with eager work in
    between, adds the same exact product (integer inputs)."""
    from gpu_util import DevMat
    M, N, K = 6144, 8192, 128
    q = binding.query_config(0, M, N, K, 256, K, 256, N, 256, N)
    assert q["name"].endswith("_chain") and q["grid"] == 256, q
    A, B, C0 = wl.make_inputs(M, N, K, "int2", "zeros", seed=51)
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
    for rep in range(2, 5):
        g.replay()
        torch.cuda.synchronize()
        assert torch.ones(1 << 20, device="cuda").sum().item() == float(1 << 20)      # eager work between replays
        assert np.array_equal(dC.fetch(), oracle_mod.round_to_f32(float(rep) * Cref)), f"replay {rep - 1}"
