"""GPU parity on seeded random shapes within the documented limits: bit width, N, K, group size and T
drawn per case; quantizer bit for bit, then forward, dX, scale and zero-point gradients (plain calls and
the trainable-zero-point calls) against the oracle, to the tolerances of the fixed-shape tests.  Every
third case forces the contraction kernel's four-wave form, which such small shapes would not take."""
import numpy as np
import pytest

from paper_2305_14152_amd import synth

pytestmark = pytest.mark.gpu

Y_TOL = 2e-2
G_TOL = 1e-3


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available()
    from paper_2305_14152_amd import peqa
    peqa.lib()
    import gpu_util
    return gpu_util


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for case in range(n):
        bits = int(rng.choice([3, 4]))
        N = 128 * int(rng.integers(1, 9))
        K = 128 * int(rng.integers(1, 17))
        groups = [0] + [g for g in (64, 128, 192, 256, 384, 512) if K % g == 0 and g <= K]
        group = int(rng.choice(groups))
        T = int(rng.choice([1, 2, 5, 16, 17, 31, 64, 100, 128, 129, 200, 257, 300]))
        out.append((case, bits, N, K, group, T))
    return out


@pytest.mark.parametrize("case,bits,N,K,group,T", _cases(24, 20240607))
def test_random_shape(gpu, oracle, case, bits, N, K, group, T):
    from paper_2305_14152_amd import peqa
    print("random shape %d: bits=%d N=%d K=%d g=%d T=%d" % (case, bits, N, K, group, T), flush=True)
    peqa.set_option(peqa.PEQA_OPT_GEMM_WAVES, 4 if case % 3 == 2 else 0)
    try:
        _random_shape(gpu, oracle, case, bits, N, K, group, T)
    finally:
        peqa.set_option(peqa.PEQA_OPT_GEMM_WAVES, 0)


def _random_shape(gpu, oracle, case, bits, N, K, group, T):
    seed = 300000 + 10 * case
    W = synth.normal_f32(seed, (N, K), 0.02)
    X = synth.normal_bf16(seed + 1, (T, K), 1.0)
    dY = synth.normal_bf16(seed + 2, (T, N), 1.0)
    layer = gpu.GpuLayer(W, bits, group)
    codes, s0, z0 = oracle.quantize(W, bits, group)
    packed, gs0, gz0 = layer.host_quant()
    assert (packed == oracle.pack(codes, bits)).all()
    assert (gs0.view(np.uint32) == s0.view(np.uint32)).all() and (gz0 == z0).all()
    ds = synth.normal_f32(seed + 3, s0.shape, 1.0) * 0.05 * s0
    dz = synth.normal_f32(seed + 4, s0.shape, 0.5)

    Y = gpu.bf16_dev_to_f64(layer.fwd(X, ds))
    Yref = oracle.fwd(codes, s0, ds, z0, X, group)
    assert np.abs(Y - Yref).max() <= Y_TOL * np.abs(Yref).max()
    dX, dds = layer.bwd(X, dY, ds)
    dXref, gref, _ = oracle.bwd(codes, s0, ds, z0, X, dY, group)
    assert np.abs(gpu.bf16_dev_to_f64(dX) - dXref).max() <= Y_TOL * np.abs(dXref).max()
    gpu.assert_scale_grad_close(gpu.to_host(dds), gref)

    Yz = gpu.bf16_dev_to_f64(layer.fwd_z(X, ds, dz))
    Yzref = oracle.fwd_z(codes, s0, ds, z0, dz, X, group)
    assert np.abs(Yz - Yzref).max() <= Y_TOL * np.abs(Yzref).max()
    dXz, ddsz, ddz = layer.bwd_z(X, dY, ds, dz)
    dXzref, gsref, gzref = oracle.bwd_z(codes, s0, ds, z0, dz, X, dY, group)
    assert np.abs(gpu.bf16_dev_to_f64(dXz) - dXzref).max() <= Y_TOL * np.abs(dXzref).max()
    gpu.assert_scale_grad_close(gpu.to_host(ddsz), gsref, "d_ds")
    gpu.assert_scale_grad_close(gpu.to_host(ddz), gzref, "d_dz")
