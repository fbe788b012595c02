"""Helpers of the GPU parity tests: host<->device marshalling and error metrics (no attention math)."""
import sys

import numpy as np

from synth_inputs import bf16_bits_to_f64


def say(msg):
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


def dev_bf16(bits):
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 tensor on cuda:0."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to("cuda:0")


def host_f64(t):
    """torch tensor (bf16 or fp32, any device) -> float64 numpy."""
    import torch
    if t.dtype == torch.bfloat16:
        bits = t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return bf16_bits_to_f64(bits)
    return t.detach().to("cpu", torch.float64).numpy()


def rel_l2(x, ref):
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((x - ref).ravel())
    return num / den if den > 0 else num


def max_abs(x, ref):
    both_ninf = np.isneginf(x) & np.isneginf(ref)
    d = np.where(both_ninf, 0.0, np.abs(x - ref))
    return float(np.nanmax(d)) if d.size else 0.0


# tolerances of the parity bar (bf16-rounded inputs, fp64 oracle)
TOL_OUT = 1e-2
TOL_LSE = 1e-3
TOL_GRAD = 2e-2
