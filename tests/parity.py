"""Error measures and helpers shared by the GPU parity tests (not a test module)."""
import numpy as np
import torch

from paper_2605_26636_amd import synth

FP32_TOL = 1e-4   # max |g - r| / max(|r|, RMS r)
BF16_TOL = 2e-2   # max |g - r| / RMS r


def err_fp32(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    rms = np.sqrt(np.mean(ref * ref))
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rms)))


def err_bf16(got, ref, rms=None):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if rms is None:
        rms = np.sqrt(np.mean(ref * ref))
    return float(np.max(np.abs(got - ref)) / rms)


def to_device(a, bf16):
    """float32 numpy array (bf16-representable when bf16) -> device tensor of the kernel dtype."""
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def to_host(t):
    return t.float().cpu().numpy().astype(np.float64)


def rows_of(o_dev, rows):
    """Gather rows (b, h, i) of a device output tensor -> float64 [n_rows, d]."""
    r = torch.as_tensor(rows, device=o_dev.device)
    return o_dev[r[:, 0], r[:, 1], r[:, 2]].float().cpu().numpy().astype(np.float64)
