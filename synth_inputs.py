"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no attention arithmetic: only a seeded normal generator, round-to-nearest-even
bf16 quantisation and exact widening.  Every tensor is N(0,1) rounded to bf16, as in
the workload configurations (Llama-shaped head counts and head_dim from the paper's
model table; the paper names no dataset, so none is stood in for).
"""
import numpy as np

SEED_BASE = 0x51170000
TENSOR_ID = {"q": 0, "k": 1, "v": 2, "do": 3}


def f32_to_bf16_bits(x):
    """float32 array -> uint16 bf16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f64(bits):
    """uint16 bf16 bit patterns -> float64 (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def bf16_bits_to_f32(bits):
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(shape, config_id, tensor, salt=0):
    """N(0,1) rounded to bf16; returns uint16 bit patterns of the given shape."""
    seed = SEED_BASE + 16 * config_id + TENSOR_ID[tensor] + (salt << 20)
    rng = np.random.Generator(np.random.Philox(seed))
    x = rng.standard_normal(size=shape, dtype=np.float32)
    return f32_to_bf16_bits(x)


# The five workload configurations (sequence length, slices, heads, head_dim).
CONFIGS = {
    0: dict(name="tiny", N=2048, n=4, Hq=4, Hkv=4, D=64),
    1: dict(name="llama13b_share", N=32768, n=8, Hq=40, Hkv=40, D=128),
    2: dict(name="llama70b_tp8_share", N=262144, n=16, Hq=8, Hkv=1, D=128),
    3: dict(name="redistribution", N=131072, n=32, Hq=8, Hkv=1, D=128),
    4: dict(name="longest", N=1048576, n=64, Hq=8, Hkv=1, D=128),
}
