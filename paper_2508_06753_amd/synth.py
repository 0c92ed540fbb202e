"""Seeded synthetic inputs shared by the tests, the smoke check and the bench.

This module draws random codes, scales and activations with the shapes and
value distributions of the workloads; it holds none of the method's
arithmetic (no quantisation, no matmul, no packing).  The only numeric step
is rounding freshly drawn fp32 numbers to bf16 storage, which is part of the
input recipe ("scales are bf16", "w2a16 activations are bf16").
"""
import numpy as np

CODEC_INT2 = 0
CODEC_TERNARY = 1


def f32_to_bf16_bits(a):
    """Round float32 to bf16 storage (nearest even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r.reshape(a.shape)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def make_weights(K, N, G, codec=CODEC_INT2, seed=0, rng=None):
    """codes uint8 [K,N] uniform over the codec's alphabet; scales bf16 bits [K/G,N]
    drawn uniform [0.005, 0.05] in fp32 and rounded to bf16."""
    rng = rng or np.random.Generator(np.random.PCG64(seed))
    hi = 4 if codec == CODEC_INT2 else 3
    codes = rng.integers(0, hi, size=(K, N), dtype=np.uint8)
    sw = rng.uniform(0.005, 0.05, size=(K // G, N)).astype(np.float32)
    return codes, f32_to_bf16_bits(sw)


def make_activations(M, K, seed=0, rng=None):
    """fp32 N(0,1) activations [M,K]."""
    rng = rng or np.random.Generator(np.random.PCG64(seed))
    return rng.standard_normal((M, K), dtype=np.float32)


def make_problem(M, K, N, G, codec=CODEC_INT2, seed=0):
    """One seeded problem: weights first, then activations, from one generator."""
    rng = np.random.Generator(np.random.PCG64(seed))
    codes, scales = make_weights(K, N, G, codec, rng=rng)
    X = make_activations(M, K, rng=rng)
    return codes, scales, X


# Shapes (K, N) of the workloads named in the benchmark configurations.
SHAPES_8B = {"qkv": (4096, 6144), "o": (4096, 4096), "gate_up": (4096, 28672),
             "down": (14336, 4096)}
SHAPES_27B = {"qkv": (5120, 7168), "o": (5120, 5120), "gate_up": (5120, 34816),
              "down": (17408, 5120)}
SHAPES_70B = {"gate_up": (8192, 57344), "down": (28672, 8192)}
