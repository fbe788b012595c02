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
    """Largest |x - ref| over the finite entries, after checking that x is finite exactly where ref is and
    equal to it where ref is not (-inf for rows without a visible key).  A NaN anywhere in x fails here:
    it is never dropped from the maximum."""
    x, ref = np.asarray(x, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert x.shape == ref.shape, (x.shape, ref.shape)
    fin_x, fin_r = np.isfinite(x), np.isfinite(ref)
    assert np.array_equal(fin_x, fin_r), "%d entries are finite on one side only (NaN/inf in the result?)" % int((fin_x != fin_r).sum())
    assert np.array_equal(x[~fin_r], ref[~fin_r]), "non-finite entries differ"
    d = np.abs(x[fin_r] - ref[fin_r])
    return float(d.max()) if d.size else 0.0


def out_err(o, o_ref, bf16_out):
    """Forward output error under the stated bound.  A bf16 result is at best half an ulp from the exact value,
    which passes 1e-2 once |out| >= 4 (rows with a handful of visible keys): such elements are held to half a
    bf16 ulp at their magnitude plus 2e-3 and counted; all others (every element of a float32 result) to the
    1e-2 bound.  Returns (largest error among the elements under the 1e-2 rule, count of the others)."""
    o, o_ref = np.asarray(o, dtype=np.float64), np.asarray(o_ref, dtype=np.float64)
    assert np.isfinite(o).all(), "non-finite forward output"
    err = np.abs(o - o_ref)
    big = (np.abs(o_ref) >= 4.0) if bf16_out else np.zeros(o_ref.shape, dtype=bool)
    if big.any():
        half_ulp = 2.0 ** (np.floor(np.log2(np.abs(o_ref[big]))) - 8)
        assert np.all(err[big] <= half_ulp + 2e-3), "bf16 output off by more than half an ulp + 2e-3 where |out| >= 4"
    small = err[~big]
    return (float(small.max()) if small.size else 0.0), int(big.sum())


# tolerances of the parity bar (bf16-rounded inputs, fp64 oracle)
TOL_OUT = 1e-2
TOL_LSE = 1e-3
TOL_GRAD = 2e-2
