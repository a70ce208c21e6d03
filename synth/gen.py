"""Seeded tensor generators (numpy PCG64).  No arithmetic of the method lives here."""
import numpy as np


def seed_for(config, layer=0, run=0):
    """Seed convention: 1000*config + layer, plus 1_000_000*run for repeated runs."""
    return 1000 * int(config) + int(layer) + 1_000_000 * int(run)


def int8_tensors(shape, seed, lo=-128, hi=127):
    """Uniform integers in [lo, hi]: x[N,H,W,C] int8, w[K,R,S,C] int8."""
    g = np.random.Generator(np.random.PCG64(seed))
    x = g.integers(lo, hi + 1, size=(shape.N, shape.H, shape.W, shape.C), dtype=np.int64).astype(np.int8)
    w = g.integers(lo, hi + 1, size=(shape.K, shape.R, shape.S, shape.C), dtype=np.int64).astype(np.int8)
    return x, w


def fp16_tensors(shape, seed):
    """x ~ N(0,1), w ~ N(0, std = 1/sqrt(R*S*C)), both rounded to fp16."""
    g = np.random.Generator(np.random.PCG64(seed))
    x = g.standard_normal((shape.N, shape.H, shape.W, shape.C)).astype(np.float16)
    std = 1.0 / np.sqrt(shape.R * shape.S * shape.C)
    w = (g.standard_normal((shape.K, shape.R, shape.S, shape.C)) * std).astype(np.float16)
    return x, w


def ones_tensors(shape, dtype=np.int8):
    """All-ones activations and filters (the paper's injection and beam runs, Sec. 5.4)."""
    return (np.ones((shape.N, shape.H, shape.W, shape.C), dtype=dtype),
            np.ones((shape.K, shape.R, shape.S, shape.C), dtype=dtype))


def requant_params(shape, seed, sigma_x=73.9, sigma_w=73.9):
    """Per-output-channel scale and bias for the int8 epilog, sized so that
    requantised outputs use the int8 range for uniform int8 inputs
    (sigma of uniform[-128,127] is about 73.9)."""
    g = np.random.Generator(np.random.PCG64(seed + 7919))
    base = 32.0 / (sigma_x * sigma_w * np.sqrt(shape.C * shape.R * shape.S))
    scale = (base * g.uniform(0.5, 1.5, size=shape.K)).astype(np.float32)
    bias = g.uniform(-4.0, 4.0, size=shape.K).astype(np.float32)
    return scale, bias
