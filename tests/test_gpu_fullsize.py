"""GPU parity at the benchmark's full sizes, in the launch configuration that
bench.py times (automatic kernel selection, dense leading dimensions).

A full binary64 oracle pass over 8192^3 takes about half a minute on the box's
host and is done once, for the headline launch (f32-accumulate); otherwise the
oracle is evaluated on sampled rows of C (first, last, both sides of tile
boundaries, random) x all N columns and compared element by element, and a
property test covers EVERY output element of an 8192^3 launch with integer
inputs whose exact result has a closed form.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2108_13191_amd import binding, workloads as wl   # noqa: E402
from gpu_util import TOL                                      # noqa: E402

CDT = {"f32": np.float32, "f16": np.float16}


def _launch(A, B, C0, mode):
    dev = torch.device("cuda:0")
    M, K = A.shape
    N = B.shape[1]
    dA, dB, dC = (torch.from_numpy(x).to(dev) for x in (A, B, C0))
    fn = binding.gemm_f16_f32acc if mode == "f32" else binding.gemm_f16_f16acc
    binding.force_config(-1)
    binding.check(fn(M, N, K, dA, K, dB, N, dC, N, torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    cfg = binding.query_config(mode == "f16", M, N, K, dA, K, dB, N, dC, N)
    return dC, cfg


def _check_rows(oracle_mod, A, B, C0, dC, mode, nrows, tile, what):
    M = A.shape[0]
    rows = wl.sample_rows(M, nrows, tile, seed=3)
    Cref, S = oracle_mod.gemm_f16(A, B, C0, rows=rows)
    got = dC[torch.from_numpy(rows).to(dC.device)].cpu().numpy().astype(np.float64)
    err = np.abs(got - Cref)
    bound = TOL[mode] * S                      # the literal bar: C0 is zero in these workloads
    bad = ~(err <= bound)
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} sampled elements out of tolerance, "
                           f"worst ratio {np.nanmax(err / np.maximum(bound, 1e-300)):.3g}")
    return float(np.max(err / np.maximum(bound, 1e-300)))


@pytest.mark.parametrize("mode", ["f32", "f16"])
def test_headline_8192_sampled_rows(oracle_mod, mode):
    A, B, C0 = wl.workload_inputs("sq8192_normal", mode)
    dC, cfg = _launch(A, B, C0, mode)
    r = _check_rows(oracle_mod, A, B, C0, dC, mode, 64, cfg["block_m"], f"8192^3 {mode}")
    print(f"8192^3 {mode}: tile {cfg['name']}, worst err/bound on {64} sampled rows {r:.3f}")


def test_headline_8192_every_element(oracle_mod):
    """The headline launch (f32-accumulate, bench.py's configuration) against a complete oracle
    pass: all 8192 x 8192 outputs, in row blocks so that the binary64 reference and bound of a
    block (2 x 64 MB) are all that is held at a time.  About half a minute of host time."""
    A, B, C0 = wl.workload_inputs("sq8192_normal", "f32")
    dC, cfg = _launch(A, B, C0, "f32")
    got = dC.cpu().numpy()
    M = A.shape[0]
    worst = 0.0
    for r0 in range(0, M, 1024):
        rows = np.arange(r0, min(M, r0 + 1024), dtype=np.int64)
        Cref, S = oracle_mod.gemm_f16(A, B, C0, rows=rows)
        err = np.abs(got[rows].astype(np.float64) - Cref)
        bound = TOL["f32"] * S
        bad = ~(err <= bound)
        assert not bad.any(), f"rows {r0}..: {bad.sum()} elements out of tolerance"
        worst = max(worst, float(np.max(err / np.maximum(bound, 1e-300))))
    print(f"8192^3 f32, every element: tile {cfg['name']}, worst err/bound {worst:.3f}")


@pytest.mark.parametrize("name", ["ffn_up", "ffn_down", "qkv", "ragged4000"])
def test_transformer_and_ragged_sampled_rows(oracle_mod, name):
    A, B, C0 = wl.workload_inputs(name, "f32")
    dC, cfg = _launch(A, B, C0, "f32")
    r = _check_rows(oracle_mod, A, B, C0, dC, "f32", 48, cfg["block_m"], name)
    print(f"{name}: tile {cfg['name']}, worst err/bound {r:.3f}")


def test_sweep_top_16384_sampled_rows(oracle_mod):
    n = 16384
    A, B, _ = wl.make_inputs(n, n, n, "uniform", "zeros", seed=0)
    for mode in ("f32", "f16"):
        C0 = np.zeros((n, n), CDT[mode])
        dC, cfg = _launch(A, B, C0, mode)
        r = _check_rows(oracle_mod, A, B, C0, dC, mode, 24, cfg["block_m"], f"16384^3 {mode}")
        print(f"16384^3 {mode}: tile {cfg['name']}, worst err/bound {r:.3f}")
        del dC


def test_every_element_of_8192_rank_one_b(oracle_mod):
    # A: integers in {-2..2}; B[k][j] = u[k] * v[j] with u in {-1,0,1}, v in {-2..2}.
    # Then C[i][j] = (sum_k A[i][k] u[k]) * v[j], |.| <= 2 * 8192 * 2 < 2^24: every
    # partial sum is an exact f32 integer, so ALL 8192^2 outputs must match exactly.
    n = 8192
    rng = np.random.default_rng(17)
    A = rng.integers(-2, 3, size=(n, n)).astype(np.float16)
    u = rng.integers(-1, 2, size=n).astype(np.int64)
    v = rng.integers(-2, 3, size=n).astype(np.int64)
    B = np.outer(u, v).astype(np.float16)
    C0 = np.zeros((n, n), np.float32)
    dC, cfg = _launch(A, B, C0, "f32")
    got = dC.cpu().numpy()
    want = np.outer(A.astype(np.int64) @ u, v).astype(np.float32)
    assert np.array_equal(got, want), f"{np.count_nonzero(got != want)} of {got.size} elements differ ({cfg['name']})"
    # the closed form itself is tied to the oracle on sampled rows
    rows = wl.sample_rows(n, 8, cfg["block_m"], seed=5)
    Cref, _ = oracle_mod.gemm_f16(A, B, C0, rows=rows)
    assert np.array_equal(Cref, want[rows].astype(np.float64))


def test_auto_selection_on_random_mid_size_shapes(oracle_mod):
    """Seeded random problems large enough for every kind of plan (single launch of each tile
    form, chained, staggered, row split), under automatic selection as bench.py runs it: sampled
    rows against the oracle, both C types."""
    rng = np.random.default_rng(2024)
    seen = set()
    shapes = [(int(rng.integers(2, 80)) * 128 - int(rng.integers(0, 2)) * int(rng.integers(1, 100)),
               int(rng.integers(16, 900)) * 8,
               int(rng.integers(8, 160)) * 8) for _ in range(14)]
    shapes += [(16384, 2304, 512), (9216, 9216, 256), (7168, 7168, 192), (5120, 5120, 320), (8192, 4096, 320)]   # staggered / split / chained plans for certain
    for idx, (M, N, K) in enumerate(shapes):
        mode = "f32" if idx % 2 == 0 else "f16"
        A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=500 + idx, c_dtype=CDT[mode])
        dC, cfg = _launch(A, B, C0, mode)
        seen.add(cfg["name"] + ("+split" if cfg["split_rows"] else ""))
        rows = wl.sample_rows(M, min(M, 48), cfg["block_m"], seed=idx)
        Cref, S = oracle_mod.gemm_f16(A, B, C0, rows=rows)
        got = dC[torch.from_numpy(rows).to(dC.device)].cpu().numpy().astype(np.float64)
        bound = TOL[mode] * (S + np.abs(C0[rows].astype(np.float64)))
        bad = ~(np.abs(got - Cref) <= bound)
        assert not bad.any(), f"{(M, N, K)} {mode} {cfg['name']}: {bad.sum()} sampled elements out of tolerance"
    print("plans exercised:", sorted(seen))
    assert any(s.endswith("_chain") or "_chain+" in s for s in seen) and any("_stag" in s for s in seen) and any("+split" in s for s in seen)
