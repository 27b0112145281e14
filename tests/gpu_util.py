"""Helpers for the GPU parity tests: move numpy inputs to the device with any
pitch / base offset, call the C ABI through the binding, fetch the result."""
import numpy as np
import torch

from paper_2108_13191_amd import binding

TOL = {"f32": 1e-5, "f16": 4e-3}       # |C - C_ref| <= TOL * sum_k |a||b|  (elementwise)
CANARY16 = np.float16(-1234.0)
CANARY32 = np.float32(-1234.0)


def config_id(name: str) -> int:
    """Index of the configuration with this name in the active library's table."""
    for i in range(binding.num_configs()):
        if binding.describe_config(i)["name"] == name:
            return i
    raise KeyError(name)


class DevMat:
    """A rows x cols matrix inside a larger device buffer: row pitch `ld`
    elements, first element `offset` elements into the allocation; everything
    around the matrix holds a canary value: NaN for an operand that is only read (a
    kernel that multiplies padding, even by zero, shows it in the result), a finite
    value for C, where "everything outside the matrix is untouched" is checked by
    comparing bits."""

    def __init__(self, host: np.ndarray, ld=None, offset=0, nan_canary=False):
        rows, cols = host.shape
        self.rows, self.cols = rows, cols
        self.ld = cols if ld is None else ld
        assert self.ld >= cols
        self.offset = offset
        n = offset + max(rows, 1) * max(self.ld, 1) + 8
        canary = host.dtype.type(np.nan) if nan_canary else CANARY16 if host.dtype == np.float16 else CANARY32
        buf = np.full(n, canary, dtype=host.dtype)
        view = buf[offset:offset + rows * self.ld].reshape(rows, self.ld) if rows and self.ld else buf[:0].reshape(rows, 0)
        if rows and cols:
            view[:, :cols] = host
        self.host_buf = buf
        self.dev = torch.from_numpy(buf).cuda()
        self.itemsize = host.dtype.itemsize

    @property
    def ptr(self):
        return self.dev.data_ptr() + self.offset * self.itemsize

    def fetch(self):
        buf = self.dev.cpu().numpy()
        out = buf[self.offset:self.offset + self.rows * self.ld].reshape(self.rows, self.ld)[:, :self.cols].copy()
        # everything outside the matrix must be untouched
        mask = np.ones(buf.shape, dtype=bool)
        inner = mask[self.offset:self.offset + self.rows * self.ld].reshape(self.rows, self.ld)
        inner[:, :self.cols] = False
        assert np.array_equal(buf[mask].view(np.uint8), self.host_buf[mask].view(np.uint8)), "memory outside C was written"
        return out


def run_gemm(A, B, C0, mode, lda=None, ldb=None, ldc=None, offs=(0, 0, 0), expect=binding.OK):
    """Run the library on device copies of A, B, C0; return the new C (numpy)."""
    M, K = A.shape
    N = B.shape[1]
    dA, dB, dC = DevMat(A, lda, offs[0], nan_canary=True), DevMat(B, ldb, offs[1], nan_canary=True), DevMat(C0, ldc, offs[2])
    fn = binding.gemm_f16_f32acc if mode == "f32" else binding.gemm_f16_f16acc
    rc = fn(M, N, K, dA.ptr, dA.ld, dB.ptr, dB.ld, dC.ptr, dC.ld, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert rc == expect, f"return code {rc} ({binding.strerror(rc)})"
    return dC.fetch()


def assert_close(got, Cref, S, C0, mode, literal=False, what=""):
    """The parity bar: |C - C_ref| <= TOL[mode] * S elementwise (literal form);
    for small adversarial cases S is widened by |C0| (the f16 store rounds a
    value of the size of C, not of S)."""
    err = np.abs(got.astype(np.float64) - Cref)
    bound = TOL[mode] * (S if literal else S + np.abs(C0.astype(np.float64)))
    bad = ~(err <= bound)
    if bad.any():
        i = np.unravel_index(np.argmax(np.where(bad, err - bound, -np.inf)), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements out of tolerance; worst at {i}: "
                             f"got {got[i]}, ref {Cref[i]}, err {err[i]:.3e}, bound {bound[i]:.3e}")
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(bound > 0, err / bound, 0.0)
    return float(ratio.max()) if ratio.size else 0.0
