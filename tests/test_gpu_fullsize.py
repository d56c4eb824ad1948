"""GPU parity at the full sizes of the benchmark workloads (the launch configuration bench.py
times): every distinct layer shape of configs 1-4 through the C-ABI, quantized codes and packed
words compared in full, Y / dX / d_ds on sampled rows and channels that the oracle computes one
by one (rows of Y and dX are independent; d_ds of a channel needs only that channel's codes)."""
import numpy as np
import pytest

from paper_2305_14152_amd import synth

pytestmark = pytest.mark.gpu

Y_TOL = 2e-2


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available()
    from paper_2305_14152_amd import peqa
    peqa.lib()
    import gpu_util
    return gpu_util


def _sample(n, edges, rng, count):
    """Indices at the ends, around tile boundaries, and random ones."""
    picks = {0, n - 1}
    for e in edges:
        for d in (-1, 0):
            if 0 <= e + d < n:
                picks.add(e + d)
    picks.update(int(v) for v in rng.integers(0, n, size=count))
    return np.array(sorted(picks))


def _one_per_tile(n, tile, edges, rng):
    """One index in every run of `tile` (a random position in it), both ends of the range, and both sides of
    the given boundaries: every tile of a launch is touched, whatever workgroup ran it."""
    picks = {0, n - 1}
    for b in range(0, n, tile):
        picks.add(b + int(rng.integers(0, min(tile, n - b))))
    for e in edges:
        for d in (-1, 0):
            if 0 <= e + d < n:
                picks.add(e + d)
    return np.array(sorted(picks))


CASES = [(cfg, li) for cfg in (1, 2, 3, 4) for li in range(3)]


# the layers bench.py runs stacked along their output channels: q, k, v and gate, up of configs 1 and 4
STACKED = [(1, 0, 3), (1, 1, 2), (4, 0, 3), (4, 1, 2)]


@pytest.mark.parametrize("cfg,li", CASES)
def test_full_size_layer(gpu, oracle, cfg, li):
    _full_size_layer(gpu, oracle, cfg, li, 1)


@pytest.mark.parametrize("cfg,li,count", STACKED)
def test_full_size_stacked_layer(gpu, oracle, cfg, li, count):
    """`count` layers of one shape as one layer of count x N channels (dY and Y [T, count x N], dX the
    gradient of the shared input), the shapes of bench.py's default run."""
    _full_size_layer(gpu, oracle, cfg, li, count)


def _full_size_layer(gpu, oracle, cfg, li, count):
    c = synth.CONFIGS[cfg]
    N, K, _ = c["layers"][li]
    N *= count
    bits, group, T = c["bits"], c["group"], c["T"]
    print("full size cfg=%d layer=%d x%d N=%d K=%d T=%d bits=%d g=%d" % (cfg, li, count, N, K, T, bits, group), flush=True)
    rng = np.random.default_rng(1000 * cfg + li + 100 * (count - 1))
    W = synth.weights(cfg, li, N=N)
    layer = gpu.GpuLayer(W, bits, group)
    codes, s0, z0 = oracle.quantize(W, bits, group)
    packed, gs0, gz0 = layer.host_quant()
    assert (gz0 == z0).all()
    assert (gs0.view(np.uint32) == s0.view(np.uint32)).all()
    assert (packed == oracle.pack(codes, bits)).all()
    del W
    layer.W0 = None

    X = synth.activations(cfg, li)
    dY = synth.output_grads(cfg, li, N=N)
    ds = synth.normal_f32(77 + cfg, s0.shape, 1e-3 * float(np.mean(s0)))
    # token rows: one in every 128-row tile (and the edges of some); channels: one in every 128-channel half of a
    # 256-column tile (and the edges of some, and of the stacked members)
    ts = _one_per_tile(T, 128, (128, 1024, T - 128), rng)
    ns = _one_per_tile(N, 128, (128, 256, N // 2, N // count), rng)
    ks = _one_per_tile(K, 128, (128, 256, K // 2), rng)
    assert len(ts) >= T // 128 and len(ns) >= N // 128

    # forward: the sampled rows against every channel
    Y = gpu.bf16_dev_to_f64(layer.fwd(X, ds))
    Yref = oracle.fwd(codes, s0, ds, z0, X[ts], group)
    assert np.abs(Y[ts] - Yref).max() <= Y_TOL * np.abs(Yref).max()
    # every output tile is non-trivial: no 128 x 128 block of Y was left unwritten or zero
    blocks = np.abs(Y).reshape(T // 128, 128, N // 128, 128).max(axis=(1, 3))
    assert (blocks > 0).all()

    # backward: whole rows of dX for the sampled tokens, d_ds of the sampled channels
    dX, dds = layer.bwd(X, dY, ds)
    dXref, _, _ = oracle.bwd(codes, s0, ds, z0, X[ts], dY[ts], group, want_P=False)
    got = gpu.bf16_dev_to_f64(dX)
    assert np.abs(got[ts] - dXref).max() <= Y_TOL * np.abs(dXref).max()
    blocks = np.abs(got).reshape(T // 128, 128, K // 128, 128).max(axis=(1, 3))
    assert (blocks > 0).all()
    del got, ks
    _, gref, _ = oracle.bwd(codes[ns], s0[ns], ds[ns], z0[ns], X, np.ascontiguousarray(dY[:, ns]), group, want_dX=False)
    g = gpu.to_host(dds).astype(np.float64)[ns]
    gpu.assert_scale_grad_close(g, gref)
    assert np.isfinite(gpu.to_host(dds)).all() and (np.abs(gpu.to_host(dds)).reshape(N // 128, -1).max(axis=1) > 0).all()

    if cfg == 4:
        # deployment forward of the same layer: T = 1 and T = 16, every channel
        for Ts in (1, 16):
            Xs = np.ascontiguousarray(X[:Ts])
            Ys = gpu.bf16_dev_to_f64(layer.fwd(Xs, ds))
            Ysref = oracle.fwd(codes, s0, ds, z0, Xs, group)
            assert np.abs(Ys - Ysref).max() <= Y_TOL * np.abs(Ysref).max()


@pytest.mark.parametrize("cfg,li", [(1, 1), (4, 1)])
def test_full_size_variants(gpu, oracle, cfg, li):
    """The optional paths at the benchmark's sizes, on sampled rows and channels: the kept-product
    backward (per-channel workload) and trainable zero-points (both workloads)."""
    c = synth.CONFIGS[cfg]
    N, K, _ = c["layers"][li]
    bits, group, T = c["bits"], c["group"], c["T"]
    print("full size variants cfg=%d layer=%d N=%d K=%d T=%d bits=%d g=%d" % (cfg, li, N, K, T, bits, group), flush=True)
    rng = np.random.default_rng(2000 * cfg + li)
    W = synth.weights(cfg, li)
    layer = gpu.GpuLayer(W, bits, group)
    codes, s0, z0 = oracle.quantize(W, bits, group)
    del W
    layer.W0 = None
    X = synth.activations(cfg, li)
    dY = synth.output_grads(cfg, li)
    ds = synth.normal_f32(78 + cfg, s0.shape, 1e-3 * float(np.mean(s0)))
    dz = synth.normal_f32(79 + cfg, s0.shape, 0.4)
    ts = _sample(T, (128, 1024), rng, 3)
    ns = _sample(N, (128, 256, N // 2), rng, 8)
    dYn = np.ascontiguousarray(dY[:, ns])

    # trainable zero-points
    Y = gpu.bf16_dev_to_f64(layer.fwd_z(X, ds, dz))
    Yref = oracle.fwd_z(codes[ns], s0[ns], ds[ns], z0[ns], dz[ns], X[ts], group)
    assert np.abs(Y[np.ix_(ts, ns)] - Yref).max() <= Y_TOL * np.abs(Yref).max()
    dX, dds, ddz = layer.bwd_z(X, dY, ds, dz)
    dXref, _, _ = oracle.bwd_z(codes, s0, ds, z0, dz, X[ts], dY[ts], group)
    assert np.abs(gpu.bf16_dev_to_f64(dX)[ts] - dXref).max() <= Y_TOL * np.abs(dXref).max()
    _, gs_ref, gz_ref = oracle.bwd_z(codes[ns], s0[ns], ds[ns], z0[ns], dz[ns], X, dYn, group, want_dX=False)
    gs = gpu.to_host(dds).astype(np.float64)[ns]
    gz = gpu.to_host(ddz).astype(np.float64)[ns]
    gpu.assert_scale_grad_close(gs, gs_ref, "d_ds")
    gpu.assert_scale_grad_close(gz, gz_ref, "d_dz")

    if group == 0:
        # kept product: P on the sampled entries, the scale gradient of the sampled channels from it
        Yk, P = layer.fwd_keep(X, ds)
        Pref = oracle.fwd(codes[ns], np.ones_like(s0[ns]), None, z0[ns], X[ts], 0)
        Ph = gpu.to_host(P).astype(np.float64)[np.ix_(ts, ns)]
        assert np.abs(Ph - Pref).max() <= 1e-5 * np.abs(Pref).max()
        _, ddsk = layer.bwd_kept(P, dY, ds, want_dX=False)
        _, gref, _ = oracle.bwd(codes[ns], s0[ns], ds[ns], z0[ns], X, dYn, 0, want_dX=False)
        gk = gpu.to_host(ddsk).astype(np.float64)[ns]
        gpu.assert_scale_grad_close(gk, gref)


def test_full_size_quantize_search(gpu, oracle):
    """Error-minimising initialisation of a whole 4096 x 4096 layer (8 register vectors per thread, 512
    workgroups): every scale, zero-point and packed word against the oracle."""
    import torch
    from paper_2305_14152_amd import peqa
    cfg, li, n, m = 1, 0, 8, 0.5
    c = synth.CONFIGS[cfg]
    N, K, _ = c["layers"][li]
    bits, group = c["bits"], c["group"]
    print("full size search N=%d K=%d bits=%d n=%d" % (N, K, bits, n), flush=True)
    W = synth.weights(cfg, li)
    L = peqa.layout(N, K, bits, group)
    packed = torch.empty(peqa.packed_words(L), dtype=torch.int32, device="cuda")
    s0 = torch.empty((N, L.groups), dtype=torch.float32, device="cuda")
    z0 = torch.empty((N, L.groups), dtype=torch.uint8, device="cuda")
    Wd = gpu.to_dev(W)
    peqa.quantize_search(L, Wd, n, m, packed, s0, z0)
    torch.cuda.synchronize()
    codes, rs0, rz0, choice = oracle.quantize_search(W, bits, group, n, m)
    same = (gpu.to_host(s0).view(np.uint32) == rs0.view(np.uint32)) & (gpu.to_host(z0) == rz0)
    print("  candidates kept beyond the plain range: %d of %d; rows differing: %d"
          % (int((choice > 0).sum()), choice.size, int((~same).sum())), flush=True)
    words = gpu.to_host(packed, np.uint32)
    got = oracle.unpack(words, N, K, bits)
    rows = same[:, 0]
    assert (got[rows] == codes[rows]).all()
    if not rows.all():
        # another candidate is right only as a tie: the two reconstruction errors (fp64) agree to 1e-12
        bad = np.nonzero(~rows)[0]
        Wb = W[bad].astype(np.float64)
        gs0, gz0 = gpu.to_host(s0)[bad], gpu.to_host(z0)[bad]
        e_ref = ((Wb - oracle.dequant(codes[bad], rs0[bad], None, rz0[bad], group)) ** 2).sum(axis=1)
        e_gpu = ((Wb - oracle.dequant(got[bad], gs0, None, gz0, group)) ** 2).sum(axis=1)
        assert (np.abs(e_gpu - e_ref) <= 1e-12 * e_ref).all()
