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


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_full_size_block(gpu, oracle, cfg):
    """The launch configuration bench.py times: the whole decoder block behind peqa_block_fwd / peqa_block_bwd, q, k, v
    and gate, up stacked (4 items), at the workload's full size.  Y and dX on one token row of every 128-row tile
    against all channels / features, d_ds on one channel of every 128; for the 7B and the 13B workload also the
    T <= 16 block forward with the seven layers as separate items (slices of the stacked arrays), every channel."""
    import torch
    from paper_2305_14152_amd import peqa
    c = synth.CONFIGS[cfg]
    bits, group, T = c["bits"], c["group"], c["T"]
    (n_a, k_a, _), (n_m, k_m, _), (n_d, k_d, _) = c["layers"]
    shapes = [(3 * n_a, k_a, 0, 0), (n_a, k_a, 0, 1), (2 * n_m, k_m, 1, 2), (n_d, k_d, 2, 3)]    # N, K, layer index, input
    print("full size block cfg=%d T=%d bits=%d g=%d" % (cfg, T, bits, group), flush=True)
    rng = np.random.default_rng(5000 + cfg)
    members, dicts, inputs = [], [], {}
    for (N, K, li, xi) in shapes:
        W = synth.weights(cfg, li, N=N)
        layer = gpu.GpuLayer(W, bits, group)
        codes, s0, z0 = oracle.quantize(W, bits, group)
        del W
        layer.W0 = None
        ds = synth.normal_f32(500 + cfg + xi, s0.shape, 1e-3 * float(np.mean(s0)))
        if xi not in inputs:
            X = synth.activations(cfg, li) if xi != 1 else synth.normal_bf16(900 + cfg, (T, K), 1.0)
            inputs[xi] = (X, gpu.to_dev(X), torch.zeros((T, 2), dtype=torch.float32, device="cuda"))
        X, Xd, rs = inputs[xi]
        dY = synth.output_grads(cfg, li, N=N)
        members.append(dict(N=N, K=K, codes=codes, s0=s0, z0=z0, ds=ds, X=X, dY=dY, layer=layer))
        dicts.append(dict(L=layer.L, packed=layer.packed, s0=layer.s0, z0=layer.z0, ds=gpu.to_dev(ds), X=Xd,
                          Y=torch.zeros((T, N), dtype=torch.int16, device="cuda"), dY=gpu.to_dev(dY),
                          dX=torch.zeros((T, K), dtype=torch.int16, device="cuda"),
                          d_ds=torch.zeros(s0.shape, dtype=torch.float32, device="cuda"),
                          row_sums=rs if not group else None))
    items = peqa.block_items(dicts)
    nb = max(peqa.block_workspace_bytes(items, T, op) for op in (peqa.PEQA_OP_FWD, peqa.PEQA_OP_BWD))
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    peqa.block_fwd(items, T, ws, nb)
    peqa.block_bwd(items, T, ws, nb)
    torch.cuda.synchronize()
    ts = _one_per_tile(T, 128, (128, T - 128), rng)
    for m, d in zip(members, dicts):
        N, K = m["N"], m["K"]
        print("  item N=%d K=%d" % (N, K), flush=True)
        Y = gpu.bf16_dev_to_f64(d["Y"])
        Yref = oracle.fwd(m["codes"], m["s0"], m["ds"], m["z0"], m["X"][ts], group)
        assert np.abs(Y[ts] - Yref).max() <= Y_TOL * np.abs(Yref).max()
        assert (np.abs(Y).reshape(T // 128, 128, N // 128, 128).max(axis=(1, 3)) > 0).all()
        del Y
        dX = gpu.bf16_dev_to_f64(d["dX"])
        dXref, _, _ = oracle.bwd(m["codes"], m["s0"], m["ds"], m["z0"], m["X"][ts], m["dY"][ts], group, want_P=False)
        assert np.abs(dX[ts] - dXref).max() <= Y_TOL * np.abs(dXref).max()
        assert (np.abs(dX).reshape(T // 128, 128, K // 128, 128).max(axis=(1, 3)) > 0).all()
        del dX
        ns = _one_per_tile(N, 128, (128, 256, N // 2), rng)
        _, gref, _ = oracle.bwd(m["codes"][ns], m["s0"][ns], m["ds"][ns], m["z0"][ns], m["X"],
                                np.ascontiguousarray(m["dY"][:, ns]), group, want_dX=False)
        g = gpu.to_host(d["d_ds"]).astype(np.float64)
        gpu.assert_scale_grad_close(g[ns], gref)
        assert np.isfinite(g).all() and (np.abs(g).reshape(N // 128, -1).max(axis=1) > 0).all()
    if cfg not in (1, 4):
        return
    # deployment forward of the block: seven items (q, k, v and gate, up as slices of the stacked arrays), one call.
    # (T = 1 and 4 take the three-workgroups-per-unit slicing on the per-channel 7B block, T = 16 the other.)
    for Ts in ((1, 16) if cfg == 4 else (1, 4, 16)):
        seven, refs = [], []
        for m, d, (N, K, li, xi) in zip(members, dicts, shapes):
            count = {0: 3, 1: 1, 2: 2, 3: 1}[xi]
            n1 = N // count
            L1 = peqa.layout(n1, K, bits, group)
            w1 = peqa.packed_words(L1)
            Xs = np.ascontiguousarray(m["X"][:Ts])
            Xsd = gpu.to_dev(Xs)
            for i in range(count):
                sl = slice(i * n1, (i + 1) * n1)
                seven.append(dict(L=L1, packed=d["packed"][i * w1:(i + 1) * w1], s0=d["s0"][sl], z0=d["z0"][sl], ds=d["ds"][sl],
                                  X=Xsd, Y=torch.zeros((Ts, n1), dtype=torch.int16, device="cuda")))
                refs.append((m["codes"][sl], m["s0"][sl], m["ds"][sl], m["z0"][sl], Xs))
        it7 = peqa.block_items(seven)
        nb7 = peqa.block_workspace_bytes(it7, Ts, peqa.PEQA_OP_FWD)
        ws7 = torch.empty(nb7, dtype=torch.uint8, device="cuda")
        peqa.block_fwd(it7, Ts, ws7, nb7)
        torch.cuda.synchronize()
        for d7, (codes, s0, ds, z0, Xs) in zip(seven, refs):
            Yref = oracle.fwd(codes, s0, ds, z0, Xs, group)
            assert np.abs(gpu.bf16_dev_to_f64(d7["Y"]) - Yref).max() <= Y_TOL * np.abs(Yref).max()
