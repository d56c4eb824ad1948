"""Seeded synthetic inputs for the PEQA quantized-linear hot path.

This module serves both the CPU oracle's tests and the GPU library's tests and
benchmark.  It holds none of the method's arithmetic: it only draws random
tensors with the shapes and value distributions of the workloads, and converts
between fp32 and bf16 bit patterns (an input encoding, not a step of the method).

Workload table (index = configuration):
  0  one 256x256 layer, 4-bit per-channel, T = 64
  1  LLaMA-7B decoder-block linears, 4-bit per-channel, T = 2048   (headline)
  2  LLaMA-7B shapes, 3-bit per-channel, T = 4096, 0.1% outlier weights
  3  LLaMA-65B shapes, 4-bit per-channel, T = 2048
  4  LLaMA-13B shapes, 3-bit, group size 128, T = 2048 (training) and 1 / 16 (deployment)
Each entry lists (N_out, K_in, count) per distinct layer of one decoder block:
q/k/v/o projections, gate/up projections, down projection.
"""
import numpy as np

BASE_SEED = 230514152

CONFIGS = {
    0: dict(name="single-256", layers=[(256, 256, 1)], bits=4, group=0, T=64,
            w_std=0.02, x_std=1.0, dy_std=1.0, outlier_p=0.0, outlier_std=0.0),
    1: dict(name="llama7b-4bit-pc", layers=[(4096, 4096, 4), (11008, 4096, 2), (4096, 11008, 1)],
            bits=4, group=0, T=2048, w_std=0.02, x_std=1.0, dy_std=1e-2,
            outlier_p=0.0, outlier_std=0.0),
    2: dict(name="llama7b-3bit-pc-outliers", layers=[(4096, 4096, 4), (11008, 4096, 2), (4096, 11008, 1)],
            bits=3, group=0, T=4096, w_std=0.02, x_std=1.0, dy_std=1e-2,
            outlier_p=1e-3, outlier_std=0.2),
    3: dict(name="llama65b-4bit-pc", layers=[(8192, 8192, 4), (22016, 8192, 2), (8192, 22016, 1)],
            bits=4, group=0, T=2048, w_std=0.015, x_std=1.0, dy_std=1e-2,
            outlier_p=0.0, outlier_std=0.0),
    4: dict(name="llama13b-3bit-g128", layers=[(5120, 5120, 4), (13824, 5120, 2), (5120, 13824, 1)],
            bits=3, group=128, T=2048, w_std=0.02, x_std=1.0, dy_std=1e-2,
            outlier_p=0.0, outlier_std=0.0),
}

TENSOR_W, TENSOR_X, TENSOR_DY, TENSOR_MASK, TENSOR_OUTLIER, TENSOR_DS = 0, 1, 2, 3, 4, 5


def seed_for(config, layer, tensor_id):
    return BASE_SEED + 1000 * config + 10 * layer + tensor_id


def rng(seed):
    """Counter-based generator (Philox), fully determined by the integer seed."""
    return np.random.Generator(np.random.Philox(key=int(seed)))


def f32_to_bf16_bits(a):
    """fp32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    """bf16 bit patterns (uint16) -> the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_f32(seed, shape, std):
    return (rng(seed).standard_normal(size=shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def normal_bf16(seed, shape, std):
    return f32_to_bf16_bits(normal_f32(seed, shape, std))


def weights(config, layer, N=None, K=None):
    """fp32 pre-trained weight W0 [N,K] of layer `layer` (index into the config's
    layer list) ~ N(0, w_std), with the config's outlier mixture if any."""
    c = CONFIGS[config]
    n, k, _ = c["layers"][layer]
    N = n if N is None else N
    K = k if K is None else K
    W = normal_f32(seed_for(config, layer, TENSOR_W), (N, K), c["w_std"])
    if c["outlier_p"] > 0.0:
        mask = rng(seed_for(config, layer, TENSOR_MASK)).random(size=(N, K), dtype=np.float32) < c["outlier_p"]
        out = normal_f32(seed_for(config, layer, TENSOR_OUTLIER), (N, K), c["outlier_std"])
        W = np.where(mask, out, W).astype(np.float32)
    return W


def activations(config, layer, T=None, K=None):
    """bf16 bit patterns of X [T,K] ~ N(0, x_std)."""
    c = CONFIGS[config]
    _, k, _ = c["layers"][layer]
    return normal_bf16(seed_for(config, layer, TENSOR_X), (c["T"] if T is None else T, k if K is None else K),
                       c["x_std"])


def output_grads(config, layer, T=None, N=None):
    """bf16 bit patterns of dY [T,N] ~ N(0, dy_std)."""
    c = CONFIGS[config]
    n, _, _ = c["layers"][layer]
    return normal_bf16(seed_for(config, layer, TENSOR_DY), (c["T"] if T is None else T, n if N is None else N),
                       c["dy_std"])


def block_flops(config, T=None, passes=3):
    """Counted flops of one decoder block: `passes` dense contractions of 2*T*N*K each
    (forward, dX, and the product recomputed for the scale gradient)."""
    c = CONFIGS[config]
    T = c["T"] if T is None else T
    return sum(2 * passes * T * n * k * cnt for n, k, cnt in c["layers"])
