"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds none of the method's arithmetic: it only draws index matrices, centroid tables and
activations with the shapes and value distributions of the benchmark configurations
(uniform 8-bit parent indices, per-row ascending N(0, sigma) binary16 tables for each
bit-width 3..8, N(0, 1) binary16 activations).  These stand in for the SqueezeLLM-quantised
Llama-2 linear layers the paper measures on (Section 6.2), whose weights are not available.
"""
import numpy as np

BASE_SEED = 20240210

# (config id) -> list of (M, K), sigma, batches; M = output channels, K = input channels.
CONFIGS = {
    1: dict(name="tiny", shapes=[(512, 512)], sigma=0.02, batches=[1]),
    2: dict(name="llama2-7b", shapes=[(4096, 4096), (11008, 4096), (4096, 11008)], sigma=0.02,
            batches=[1]),
    3: dict(name="llama2-13b", shapes=[(5120, 5120), (13824, 5120), (5120, 13824)], sigma=0.02,
            batches=[1]),
    5: dict(name="llama2-70b", shapes=[(8192, 8192), (1024, 8192), (28672, 8192), (8192, 28672)],
            sigma=0.01, batches=[1, 2, 4, 8]),
}

# One decoder layer of the 7B-shaped decode step (config 4): q, k, v, o, gate, up, down.
DECODE_LAYER_SHAPES = [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
DECODE_LAYERS = 32


def make_case(config_id, M, K, batch=1, sigma=0.02, n=8, bit_widths=range(3, 9), salt=0):
    """Draw (idx, luts, x) for one matrix.  Draw order is fixed: idx, tables b ascending, x.

    idx  : (M, K) uint8, uniform in [0, 2**n)
    luts : {b: (M, 2**b) float16, each row sorted ascending}
    x    : (batch, K) float16
    """
    rng = np.random.default_rng([BASE_SEED, config_id, M, K, salt])
    idx = rng.integers(0, 1 << n, size=(M, K), dtype=np.uint8)
    luts = {}
    for b in bit_widths:
        luts[b] = np.sort(rng.normal(0.0, sigma, size=(M, 1 << b)).astype(np.float16), axis=1)
    x = rng.normal(0.0, 1.0, size=(batch, K)).astype(np.float16)
    return idx, luts, x


def make_dense_weights(config_id, M, K, sigma=0.02, salt=0):
    """Draw (W, S) for the quantiser: W (M, K) float32 heavy-tailed around 0 (Student t, 5 degrees of
    freedom, scaled to sigma: LLM weight rows have a few large outliers), S (M, K) float32 positive,
    skewed per-weight sensitivities (gamma, shape 0.5), standing in for the calibration gradients."""
    rng = np.random.default_rng([BASE_SEED, config_id, M, K, salt, 1])
    W = (rng.standard_t(5, size=(M, K)) * sigma).astype(np.float32)
    S = (rng.gamma(0.5, 1.0, size=(M, K)) + 1e-6).astype(np.float32)
    return W, S


def decode_bit_sequence(steps=64):
    """Seeded per-step bit-widths of the decode-step configuration (config 4)."""
    rng = np.random.default_rng([BASE_SEED, 4])
    return rng.integers(3, 9, size=steps).tolist()


def algorithmic_bytes(M, K, b, batch=1):
    """Bytes one call must move: index bits, one centroid table, activations, outputs."""
    return M * K * b // 8 + M * (1 << b) * 2 + batch * K * 2 + batch * M * 2
