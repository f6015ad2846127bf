"""Seeded synthetic inputs for tests and benchmarks (no arithmetic of the method lives here).

The paper's workloads are MNIST / CIFAR-10 images and trained weights, which
are not available; these generators give tensors of the same shapes and value
ranges instead.
"""
import numpy as np


def slot_vector(seed, count, lo=-1.0, hi=1.0, complex_values=False):
    """Message slots uniform in [lo, hi) (the micro-benchmark messages)."""
    rng = np.random.default_rng(seed)
    v = rng.uniform(lo, hi, count)
    if complex_values:
        v = v + 1j * rng.uniform(lo, hi, count)
    return v


def plaintext_coeffs(seed, n, bits):
    """Signed integer plaintext coefficients, uniform in [-2^bits, 2^bits)."""
    rng = np.random.default_rng(seed)
    return rng.integers(-(1 << bits), 1 << bits, n, dtype=np.int64)


def image(seed, channels, height, width):
    """Pixels uniform in [0, 1)."""
    return np.random.default_rng(seed).uniform(0.0, 1.0, (channels, height, width))


def conv_weights(seed, fh, fw, ic, oc, dist="uniform", std=0.1):
    """[FH][FW][IC][OC]; uniform in [-1, 1) or normal(0, std^2)."""
    rng = np.random.default_rng(seed)
    if dist == "uniform":
        return rng.uniform(-1.0, 1.0, (fh, fw, ic, oc))
    return rng.normal(0.0, std, (fh, fw, ic, oc))


def fc_weights(seed, out_features, channels, height, width, std=0.1):
    return np.random.default_rng(seed).normal(0.0, std, (out_features, channels, height, width))


def uniform_residues(seed, shape, primes):
    """Residues uniform in [0, q_i) along the limb axis (second to last): stand-ins for ciphertext data."""
    rng = np.random.default_rng(seed)
    out = np.zeros(shape, dtype=np.uint64)
    for i, q in enumerate(primes):
        out[..., i, :] = rng.integers(0, q, out[..., i, :].shape, dtype=np.uint64)
    return out
