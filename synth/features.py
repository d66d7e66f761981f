"""Seeded dense inputs: node features and layer weights (float32 numpy arrays).

Conversion to fp16 / bf16 storage is done by the caller (torch), after which both the
oracle and the HIP path read the same rounded values.
"""
import numpy as np


def uniform_features(n, d, seed, lo=-1.0, hi=1.0):
    rng = np.random.default_rng(seed)
    return rng.uniform(lo, hi, size=(n, d)).astype(np.float32)


def normal_features(n, d, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(size=(n, d), dtype=np.float32)


def glorot_uniform(d_in, d_out, seed):
    rng = np.random.default_rng(seed)
    lim = np.sqrt(6.0 / (d_in + d_out))
    return rng.uniform(-lim, lim, size=(d_in, d_out)).astype(np.float32)
