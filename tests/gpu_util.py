"""Helpers of the GPU parity tests: device upload, guarded outputs, the error measure."""
import numpy as np

GUARD = 128           # 16-bit elements of guard band on each side of an output
SENTINEL = 0x7B7B


def rel_err(Y_bits: np.ndarray, Y_ref: np.ndarray):
    """max |Y - Yref| / max(|Yref|, 0.05 * rms(Yref)) over all outputs (the floor keeps outputs that
    cancel to almost zero from dominating), plus the plain max-norm ratio."""
    Y = Y_bits.view(np.float16).astype(np.float64)
    ref = np.asarray(Y_ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), max(0.05 * rms, 1e-30))
    diff = np.abs(Y - ref)
    return float(np.max(diff / den)) if ref.size else 0.0, float(np.max(diff) / max(np.max(np.abs(ref)), 1e-30)) if ref.size else 0.0


class Guarded:
    """A 16-bit device buffer with sentinel bands before and after the payload."""

    def __init__(self, torch, n):
        self.torch = torch
        self.n = int(n)
        self.buf = torch.full((self.n + 2 * GUARD,), SENTINEL, dtype=torch.int16, device="cuda")
        self.view = self.buf[GUARD:GUARD + self.n]
        assert self.view.data_ptr() % 16 == 0

    def check_and_get(self) -> np.ndarray:
        self.torch.cuda.synchronize()
        host = self.buf.cpu().numpy().view(np.uint16)
        assert np.all(host[:GUARD] == SENTINEL) and np.all(host[GUARD + self.n:] == SENTINEL), "guard band overwritten"
        return host[GUARD:GUARD + self.n].copy()


def to_dev(torch, arr: np.ndarray):
    t = torch.from_numpy(np.ascontiguousarray(arr)).cuda()
    assert t.data_ptr() % 16 == 0
    return t


class Workspace:
    """Device workspace for mpq.gemm of the size the library asks for, with a sentinel band behind it."""

    def __init__(self, torch, mpq, header, M, plan=None):
        self.torch = torch
        self.bytes = mpq.gemm_workspace_size_planned(header, M, plan) if plan is not None else mpq.gemm_workspace_size(header, M)
        self.buf = torch.full((self.bytes + 256,), 0x5A, dtype=torch.uint8, device="cuda")
        assert self.buf.data_ptr() % 256 == 0
        self.view = self.buf[:self.bytes] if self.bytes else None

    def check(self):
        self.torch.cuda.synchronize()
        assert bool((self.buf[self.bytes:] == 0x5A).all()), "workspace overrun"
