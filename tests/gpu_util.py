"""Helpers for the GPU parity tests: device upload of the seeded host arrays, the error metric and
guard bands.  No arithmetic of the method lives here."""
import numpy as np
import torch

OUT_TOL = 2e-3     # outputs, against the fp64 oracle
STATE_TOL = 1e-4   # fp32 recurrent states after 256 steps


def dev(a: np.ndarray) -> torch.Tensor:
    """Upload a host array; uint16 (bf16 bit patterns) travels as int16."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max_i |g_i - r_i| / (|r_i| + rms(r)): relative where the reference is large, scaled by the
    tensor's rms where it is near zero."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref ** 2)))
    if rms == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref) / (np.abs(ref) + rms)))


class Guarded:
    """A device buffer with sentinel bands before and after the payload."""
    BAND = 4096  # bytes

    def __init__(self, payload: np.ndarray):
        payload = np.ascontiguousarray(payload)
        raw = payload.view(np.uint8).reshape(-1)
        self.nbytes = raw.size
        pad = (-self.nbytes) % 16
        buf = np.full(self.BAND + self.nbytes + pad + self.BAND, 0xA5, dtype=np.uint8)
        buf[self.BAND:self.BAND + self.nbytes] = raw
        self.buf = torch.from_numpy(buf).cuda()
        self.dtype, self.shape = payload.dtype, payload.shape

    def ptr(self) -> int:
        return self.buf.data_ptr() + self.BAND

    def read(self) -> np.ndarray:
        raw = self.buf.cpu().numpy()
        return raw[self.BAND:self.BAND + self.nbytes].view(self.dtype).reshape(self.shape).copy()

    def bands_intact(self) -> bool:
        raw = self.buf.cpu().numpy()
        return bool((raw[:self.BAND] == 0xA5).all() and (raw[self.BAND + self.nbytes + ((-self.nbytes) % 16):] == 0xA5).all())
