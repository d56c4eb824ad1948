"""The forward entry point that allocates nothing (peqa_linear_fwd_static: scratch in the library's own device
image) against peqa_linear_fwd, through the C-ABI: same kernels, so the same bits.  Two calls in a row per layer
kind, the second with a smaller input, so that what the first call left in the shared scratch is in the way."""
import numpy as np
import pytest

from paper_2305_14152_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available()
    from paper_2305_14152_amd import peqa
    peqa.lib()
    import gpu_util
    return gpu_util


@pytest.mark.parametrize("bits,N,K,group,Ts", [
    (4, 384, 640, 0, (300, 130)),       # tiled contraction, per-channel: row sums in the scratch
    (3, 512, 768, 128, (200, 77)),      # group-wise: the (s, b) table in the scratch
    (4, 640, 2048, 0, (16, 3)),         # matrix-vector path with feature slices: partial sums in the scratch
    (3, 384, 1024, 64, (9, 1)),
    (4, 256, 512, 0, (150, 8)),         # from the tiled contraction to the matrix-vector path
])
def test_static_forward_equals_workspace_forward(gpu, oracle, bits, N, K, group, Ts):
    import torch
    from paper_2305_14152_amd import peqa
    print("static forward bits=%d N=%d K=%d g=%d T=%s" % (bits, N, K, group, Ts), flush=True)
    seed = 88000 + bits * 1000 + N + K + group
    W = synth.normal_f32(seed, (N, K), 0.02)
    layer = gpu.GpuLayer(W, bits, group)
    codes, s0, z0 = oracle.quantize(W, bits, group)
    ds = synth.normal_f32(seed + 3, s0.shape, 1e-3)
    dsd = gpu.to_dev(ds)
    for T in Ts:                                   # the second call is the smaller one
        X = synth.normal_bf16(seed + 10 + T, (T, K), 1.0)
        Xd = gpu.to_dev(X)
        assert peqa.workspace_bytes(layer.L, T, peqa.PEQA_OP_FWD) <= peqa.STATIC_SCRATCH_BYTES
        Y = torch.zeros((T, N), dtype=torch.int16, device="cuda")
        peqa.linear_fwd_static(layer.L, layer.packed, layer.s0, dsd, layer.z0, Xd, T, Y)
        torch.cuda.synchronize()
        want = layer.fwd(Xd, dsd)
        assert (gpu.to_host(Y) == gpu.to_host(want)).all(), T
        Yref = oracle.fwd(codes, s0, ds, z0, X, group)
        assert np.abs(gpu.bf16_dev_to_f64(Y) - Yref).max() <= 2e-2 * np.abs(Yref).max()


def test_static_forward_refuses_what_does_not_fit(gpu):
    """A forward whose scratch need exceeds the array is refused before anything runs; bad arguments likewise."""
    import ctypes
    from paper_2305_14152_amd import peqa
    L = peqa.layout(128 * 1024, 128 * 40, 3, 128)        # group table of 8 N G bytes = 40 MiB
    assert peqa.workspace_bytes(L, 64, peqa.PEQA_OP_FWD) > peqa.STATIC_SCRATCH_BYTES
    good = 0x10000
    lib = peqa.lib()
    assert lib.peqa_linear_fwd_static(ctypes.byref(L), good, good, None, good, good, 64, good, None) == peqa.PEQA_ERR_WORKSPACE
    L2 = peqa.layout(256, 256, 4)
    assert lib.peqa_linear_fwd_static(ctypes.byref(L2), None, good, None, good, good, 64, good, None) == peqa.PEQA_ERR_NULL
    assert lib.peqa_linear_fwd_static(ctypes.byref(L2), good, good, None, good, good, 0, good, None) == peqa.PEQA_ERR_SHAPE
