"""gemm_f16_f16acc_static_workspace, the entry point for callers that cannot allocate: the same
results as gemm_f16_f16acc_workspace, on the library's own scratch array, on calls in a row that
share the array (the second smaller, so that it finds the first one's sums in it)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2108_13191_amd import binding, workloads as wl   # noqa: E402
from gpu_util import DevMat, assert_close                    # noqa: E402


def _both(A, B, C0, ldc):
    """C of the static-workspace entry point and of the lent-workspace one, through the C ABI."""
    M, K = A.shape
    N = B.shape[1]
    need = binding.gemm_f16_f16acc_workspace_bytes(M, N, K)
    assert need == M * N * 4                                   # a problem that is cut along k
    out = []
    for static in (True, False):
        dA, dB, dC = DevMat(A, nan_canary=True), DevMat(B, nan_canary=True), DevMat(C0, ldc, 1)
        if static:
            rc = binding.gemm_f16_f16acc_static_workspace(M, N, K, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld, 0)
        else:
            ws = torch.full((need // 4,), float("nan"), device="cuda")
            rc = binding.gemm_f16_f16acc_workspace(M, N, K, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld, ws, need, 0)
        assert rc == binding.OK, binding.strerror(rc)
        torch.cuda.synchronize()
        out.append(dC.fetch())
    return out


def test_static_workspace_entry_point_matches_the_workspace_one(oracle_mod):
    binding.force_config(-1)
    # two calls in a row on the one array, the second smaller; then the first shape again
    for idx, (M, N, K) in enumerate([(300, 520, 8192), (72, 264, 4096 + 24), (300, 520, 8192)]):
        A, B, _ = wl.make_inputs(M, N, K, "int2", "zeros", seed=1300 + idx, c_dtype=np.float16)
        C0 = np.random.default_rng(idx).integers(-4, 5, size=(M, N)).astype(np.float16)
        got_static, got_lent = _both(A, B, C0, N + 8)
        Cref, _ = oracle_mod.gemm_f16(A, B, C0)
        assert np.array_equal(got_static, got_lent), f"ints {(M, N, K)}"               # exact sums: bit for bit
        assert np.array_equal(got_static, Cref.astype(np.float16)), f"ints {(M, N, K)} against the oracle"
        A, B, C0 = wl.make_inputs(M, N, K, "uniform", "uniform", seed=1310 + idx, c_dtype=np.float16)
        got_static, got_lent = _both(A, B, C0, N)
        Cref, S = oracle_mod.gemm_f16(A, B, C0)
        assert_close(got_static, Cref, S, C0, "f16", what=f"static workspace {(M, N, K)}")
        assert_close(got_lent, Cref, S, C0, "f16", what=f"lent workspace {(M, N, K)}")
    # a problem that runs unsplit takes the ordinary path (and the array is not needed)
    A, B, C0 = wl.make_inputs(200, 264, 328, "int2", "zeros", seed=9, c_dtype=np.float16)
    dA, dB, dC = DevMat(A, nan_canary=True), DevMat(B, nan_canary=True), DevMat(C0)
    assert binding.gemm_f16_f16acc_static_workspace(200, 264, 328, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld, 0) == binding.OK
    torch.cuda.synchronize()
    Cref, _ = oracle_mod.gemm_f16(A, B, C0)
    assert np.array_equal(dC.fetch(), Cref.astype(np.float16))
    assert "scratch" in binding.strerror(binding.ERR_WORKSPACE)
