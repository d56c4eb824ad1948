"""GPU parity: every C-ABI call against the CPU oracle on the same seeded inputs.
Integer results (codes, packed words, zero-points) and the fp32 scales must match bit for
bit; Y and dX within 2e-2 * max|ref| (bf16 I/O, fp32 accumulation); the scale gradient
within 1e-3 relative L2."""
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


def _log(msg):
    print(msg, flush=True)


@pytest.fixture
def options():
    """Sets the library's test switches (peqa_set_option) and puts the defaults back afterwards."""
    from paper_2305_14152_amd import peqa
    yield peqa.set_option
    peqa.set_option(peqa.PEQA_OPT_GEMM_WAVES, 0)
    peqa.set_option(peqa.PEQA_OPT_BWD_PAIR, -1)
    peqa.set_option(peqa.PEQA_OPT_GROUPED_DDS, 0)


def _check_quant(gpu, oracle, layer, W, bits, group):
    codes, s0, z0 = oracle.quantize(W, bits, group)
    packed, gs0, gz0 = layer.host_quant()
    assert (gz0 == z0).all()
    assert (gs0.view(np.uint32) == s0.view(np.uint32)).all()
    ref_words = oracle.pack(codes, bits)
    bad = np.nonzero(packed != ref_words)[0]
    assert bad.size == 0, "first differing word %d: %08x vs %08x" % (bad[0], packed[bad[0]], ref_words[bad[0]])
    return codes, s0, z0


def _check_fwd_bwd(gpu, oracle, layer, codes, s0, z0, X, dY, ds, group):
    Y = gpu.bf16_dev_to_f64(layer.fwd(X, ds))
    Yref = oracle.fwd(codes, s0, ds, z0, X, group)
    assert np.abs(Y - Yref).max() <= Y_TOL * np.abs(Yref).max()
    dX, dds = layer.bwd(X, dY, ds)
    dXref, gref, _ = oracle.bwd(codes, s0, ds, z0, X, dY, group)
    assert np.abs(gpu.bf16_dev_to_f64(dX) - dXref).max() <= Y_TOL * np.abs(dXref).max()
    g = gpu.to_host(dds).astype(np.float64)
    l2, _ = gpu.assert_scale_grad_close(g, gref)
    # informative: typical error is far below the tolerance
    return (np.abs(Y - Yref).max() / np.abs(Yref).max(), l2)


@pytest.mark.parametrize("bits", [4, 3])
def test_config0_full_parity(gpu, oracle, bits):
    """The 256x256, T=64 layer: quantize, forward, backward, all elements."""
    _log("config0 bits=%d" % bits)
    W, X, dY = synth.weights(0, 0), synth.activations(0, 0), synth.output_grads(0, 0)
    layer = gpu.GpuLayer(W, bits, 0)
    codes, s0, z0 = _check_quant(gpu, oracle, layer, W, bits, 0)
    ds = np.zeros_like(s0)
    e = _check_fwd_bwd(gpu, oracle, layer, codes, s0, z0, X, dY, None, 0)
    _log("  errors (Y rel-max, dds rel-L2): %.2e %.2e" % e)
    _check_fwd_bwd(gpu, oracle, layer, codes, s0, z0, X, dY, ds, 0)


@pytest.mark.parametrize("bits,N,K,T", [
    (4, 384, 640, 200),     # 2 column tiles (second half empty), 2 token tiles with a ragged tail
    (3, 384, 640, 200),
    (4, 128, 128, 1),       # smallest layer, one token
    (3, 512, 384, 129),     # one row into the second token tile
    (4, 640, 1152, 17),
    (3, 256, 896, 300),     # 7 contraction steps per half
    (4, 896, 256, 300),
])
def test_ragged_shapes_parity(gpu, oracle, bits, N, K, T):
    _log("ragged bits=%d N=%d K=%d T=%d" % (bits, N, K, T))
    seed = 7000 + bits * 1000 + N + K + T
    W = synth.normal_f32(seed, (N, K), 0.02)
    X = synth.normal_bf16(seed + 1, (T, K), 1.0)
    dY = synth.normal_bf16(seed + 2, (T, N), 1.0)
    layer = gpu.GpuLayer(W, bits, 0)
    codes, s0, z0 = _check_quant(gpu, oracle, layer, W, bits, 0)
    ds = synth.normal_f32(seed + 3, s0.shape, 1e-3)
    e = _check_fwd_bwd(gpu, oracle, layer, codes, s0, z0, X, dY, ds, 0)
    _log("  errors: %.2e %.2e" % e)


@pytest.mark.parametrize("bits,N,K,T,group", [
    (3, 256, 512, 200, 128),    # 4 groups, ragged token tail
    (4, 256, 512, 64, 256),     # 2 groups, one per contraction half
    (3, 384, 384, 129, 128),    # odd number of groups; contraction halves start in mid-block
    (4, 384, 640, 300, 128),    # 5 groups, empty second column half
    (4, 640, 1024, 33, 512),
    (3, 1280, 2560, 150, 128),  # several column tiles, 20 groups
    (4, 256, 1152, 70, 128),    # 9 groups: the first contraction half idles through the last one
    (3, 256, 384, 40, 384),     # a single group: the per-channel kernels
    (4, 256, 512, 150, 64),     # groups of 64: two per 128-feature run
    (3, 384, 640, 77, 64),
    (4, 512, 768, 200, 192),    # a multiple of 64 that is not one of 128
    (3, 1280, 1024, 300, 64),
])
def test_groupwise_training_parity(gpu, oracle, bits, N, K, T, group):
    """Group-wise scales (Sec. 4.2, Table 5) through the tiled contractions: forward, dX and the
    per-(channel, group) scale gradient."""
    _log("group-wise bits=%d N=%d K=%d T=%d g=%d" % (bits, N, K, T, group))
    seed = 11000 + bits * 1000 + N + K + T + group
    W = synth.normal_f32(seed, (N, K), 0.02)
    X = synth.normal_bf16(seed + 1, (T, K), 1.0)
    dY = synth.normal_bf16(seed + 2, (T, N), 1.0)
    layer = gpu.GpuLayer(W, bits, group)
    codes, s0, z0 = _check_quant(gpu, oracle, layer, W, bits, group)
    ds = synth.normal_f32(seed + 3, s0.shape, 1e-3)
    e = _check_fwd_bwd(gpu, oracle, layer, codes, s0, z0, X, dY, ds, group)
    _log("  errors: %.2e %.2e" % e)
    _check_fwd_bwd(gpu, oracle, layer, codes, s0, z0, X, dY, None, group)


@pytest.mark.parametrize("bits,N,K,T,group", [
    (4, 384, 640, 200, 0), (3, 384, 640, 200, 0), (4, 128, 128, 17, 0), (3, 512, 384, 129, 0), (3, 256, 896, 300, 0),
    (4, 896, 256, 300, 0), (4, 1280, 512, 520, 0),
    (3, 256, 512, 200, 128), (4, 256, 512, 64, 256), (3, 384, 384, 129, 128), (4, 384, 640, 300, 128),
    (3, 1280, 2560, 150, 128), (4, 256, 512, 150, 64), (3, 384, 640, 77, 64), (4, 512, 768, 200, 192),
])
def test_four_wave_contraction_parity(gpu, oracle, options, bits, N, K, T, group):
    """The contraction kernels' second form (four waves over the whole contraction range, two workgroups per
    compute unit), which launches of at least two tiles per compute unit take by themselves, forced here on
    small shapes; the same checks as for the eight-wave form, and the two forms against each other."""
    _log("four waves bits=%d N=%d K=%d T=%d g=%d" % (bits, N, K, T, group))
    seed = 19000 + bits * 1000 + N + K + T + group
    W = synth.normal_f32(seed, (N, K), 0.02)
    X = synth.normal_bf16(seed + 1, (T, K), 1.0)
    dY = synth.normal_bf16(seed + 2, (T, N), 1.0)
    layer = gpu.GpuLayer(W, bits, group)
    codes, s0, z0 = _check_quant(gpu, oracle, layer, W, bits, group)
    ds = synth.normal_f32(seed + 3, s0.shape, 1e-3)
    from paper_2305_14152_amd import peqa
    options(peqa.PEQA_OPT_GEMM_WAVES, 8)
    Y8 = gpu.bf16_dev_to_f64(layer.fwd(X, ds))
    dX8, g8 = layer.bwd(X, dY, ds)
    options(peqa.PEQA_OPT_GEMM_WAVES, 4)
    options(peqa.PEQA_OPT_BWD_PAIR, 0)                     # the backward's two contractions as launches of their own
    e = _check_fwd_bwd(gpu, oracle, layer, codes, s0, z0, X, dY, ds, group)
    _log("  errors: %.2e %.2e" % e)
    _check_fwd_bwd(gpu, oracle, layer, codes, s0, z0, X, dY, None, group)
    Y4 = gpu.bf16_dev_to_f64(layer.fwd(X, ds))
    dX4, g4 = layer.bwd(X, dY, ds)
    # the two forms add the same products in a different order: a last bf16 bit here and there
    assert np.abs(Y4 - Y8).max() <= 2.0 ** -7 * np.abs(Y8).max()
    assert np.abs(gpu.bf16_dev_to_f64(dX4) - gpu.bf16_dev_to_f64(dX8)).max() <= 2.0 ** -7 * np.abs(gpu.bf16_dev_to_f64(dX8)).max()
    g4h, g8h = gpu.to_host(g4).astype(np.float64), gpu.to_host(g8).astype(np.float64)
    assert np.linalg.norm(g4h - g8h) <= 1e-5 * np.linalg.norm(g8h)
    if group == 0:
        # both contractions of the backward as one launch of four-wave workgroups (the default when both gradients
        # are asked for): the same products in the same order
        options(peqa.PEQA_OPT_BWD_PAIR, 1)
        _check_fwd_bwd(gpu, oracle, layer, codes, s0, z0, X, dY, ds, group)
        dXp, gp = layer.bwd(X, dY, ds)
        assert np.array_equal(gpu.to_host(dXp), gpu.to_host(dX4))
        assert np.array_equal(gpu.to_host(gp), gpu.to_host(g4))


@pytest.mark.parametrize("bits,N,K,T,group", [(4, 1152, 512, 9000, 0), (3, 640, 768, 16500, 128)])
def test_many_ragged_tiles(gpu, oracle, bits, N, K, T, group):
    """More tiles than compute units with a ragged last token tile and a half-empty last column tile: the
    launch takes the four-wave form by itself and runs several workgroups per compute unit one after the
    other.  Forward, dX and the scale gradient on sampled token rows and channels."""
    _log("many tiles bits=%d N=%d K=%d T=%d g=%d" % (bits, N, K, T, group))
    seed = 21000 + bits * 1000 + N + K + T + group
    rng = np.random.default_rng(seed)
    W = synth.normal_f32(seed, (N, K), 0.02)
    X = synth.normal_bf16(seed + 1, (T, K), 1.0)
    dY = synth.normal_bf16(seed + 2, (T, N), 1.0)
    layer = gpu.GpuLayer(W, bits, group)
    codes, s0, z0 = _check_quant(gpu, oracle, layer, W, bits, group)
    ds = synth.normal_f32(seed + 3, s0.shape, 1e-3)
    ts = np.unique(np.concatenate([[0, 127, 128, T - 1, T - 2, (T // 128) * 128, (T // 128) * 128 - 1],
                                   rng.integers(0, T, size=40)]))
    ns = np.unique(np.concatenate([[0, 255, 256, N - 1, N - 128, N - 129], rng.integers(0, N, size=24)]))
    Y = gpu.bf16_dev_to_f64(layer.fwd(X, ds))
    Yref = oracle.fwd(codes, s0, ds, z0, X[ts], group)
    assert np.abs(Y[ts] - Yref).max() <= Y_TOL * np.abs(Yref).max()
    dX, dds = layer.bwd(X, dY, ds)
    dXref, _, _ = oracle.bwd(codes, s0, ds, z0, X[ts], dY[ts], group)
    assert np.abs(gpu.bf16_dev_to_f64(dX)[ts] - dXref).max() <= Y_TOL * np.abs(dXref).max()
    _, gref, _ = oracle.bwd(codes[ns], s0[ns], ds[ns], z0[ns], X, np.ascontiguousarray(dY[:, ns]), group)
    g = gpu.to_host(dds).astype(np.float64)[ns]
    gpu.assert_scale_grad_close(g, gref)


@pytest.mark.parametrize("bits,N,K,group", [
    (4, 256, 512, 0), (3, 384, 640, 0), (3, 256, 1024, 128), (4, 512, 768, 64), (3, 640, 1152, 128),
    (4, 256, 512, 256), (3, 128, 128, 0), (4, 1280, 2048, 128),
    # 128-256 channel tiles, per-channel: the 12-wave workgroups that take all of K
    (4, 16384, 256, 0),       # 4 rounds for 12 waves: most waves have nothing to do
    (3, 20480, 1536, 0),      # 160 tiles, 2 rounds per wave
    (4, 32768, 896, 0),       # 256 tiles, 14 rounds: uneven shares
])
def test_small_batch_forward_parity(gpu, oracle, bits, N, K, group):
    """The T <= 16 matrix-vector path, per-channel and group-wise, every T from 1 to 16 sampled."""
    _log("small-batch bits=%d N=%d K=%d g=%d" % (bits, N, K, group))
    seed = 9000 + bits * 1000 + N + K + group
    W = synth.normal_f32(seed, (N, K), 0.02)
    layer = gpu.GpuLayer(W, bits, group)
    codes, s0, z0 = _check_quant(gpu, oracle, layer, W, bits, group)
    ds = synth.normal_f32(seed + 3, s0.shape, 1e-3)
    for T in (1, 2, 7, 16):
        X = synth.normal_bf16(seed + 10 + T, (T, K), 1.0)
        for d in (None, ds):
            Y = gpu.bf16_dev_to_f64(layer.fwd(X, d))
            Yref = oracle.fwd(codes, s0, d, z0, X, group)
            assert Y.shape == Yref.shape
            assert np.abs(Y - Yref).max() <= Y_TOL * np.abs(Yref).max(), (T, np.abs(Y - Yref).max(), np.abs(Yref).max())


@pytest.mark.parametrize("bits,Ns,K,group", [
    (4, (256, 384, 128), 512, 0), (3, (256, 256), 1024, 128), (4, (128, 128, 128, 640), 768, 64), (3, (1280,), 2048, 0),
    (4, (8192, 8192, 4096), 384, 0),       # 160 tiles together: the 12-wave workgroups, three layers side by side
])
def test_fused_forward_parity(gpu, oracle, bits, Ns, K, group):
    """Several layers reading one X through peqa_linear_fwd_fused: every Y equals the single-layer forward."""
    import torch
    from paper_2305_14152_amd import peqa
    _log("fused bits=%d Ns=%s K=%d g=%d" % (bits, Ns, K, group))
    seed = 13000 + bits * 1000 + sum(Ns) + K + group
    layers, refs = [], []
    for j, N in enumerate(Ns):
        W = synth.normal_f32(seed + 10 * j, (N, K), 0.02)
        layer = gpu.GpuLayer(W, bits, group)
        codes, s0, z0 = oracle.quantize(W, bits, group)
        ds = synth.normal_f32(seed + 10 * j + 1, s0.shape, 1e-3) if j % 2 == 0 else None
        layers.append((layer, gpu.to_dev(ds) if ds is not None else None))
        refs.append((codes, s0, ds, z0))
    for T in (1, 5, 16, 40):
        X = synth.normal_bf16(seed + 100 + T, (T, K), 1.0)
        Xd = gpu.to_dev(X)
        Ys = [torch.zeros((T, l.N), dtype=torch.int16, device="cuda") for l, _ in layers]
        items = [(l.L, l.packed, l.s0, dsd, l.z0, Y) for (l, dsd), Y in zip(layers, Ys)]
        nb = peqa.workspace_bytes_fused(items, T)
        ws = torch.empty(max(nb, 16), dtype=torch.uint8, device="cuda")
        peqa.linear_fwd_fused(items, Xd, T, ws, nb)
        torch.cuda.synchronize()
        for (codes, s0, ds, z0), Y in zip(refs, Ys):
            Yref = oracle.fwd(codes, s0, ds, z0, X, group)
            got = gpu.bf16_dev_to_f64(Y)
            assert np.abs(got - Yref).max() <= Y_TOL * np.abs(Yref).max(), T


@pytest.mark.parametrize("bits,Ns,K,T,group", [
    (4, (256, 128, 384), 512, 200, 0), (3, (384, 384), 640, 130, 0), (4, (128, 256), 768, 9, 0),
    (3, (256, 128, 128), 512, 150, 128), (4, (384, 256), 768, 70, 64),
])
def test_stacked_layers(gpu, oracle, bits, Ns, K, T, group):
    """Layers that read one input, stacked along the output channels, are one layer whose arrays are the
    members' arrays one after the other: quantized member by member into slices of the stacked arrays it
    gives the members' Y and scale gradients bit for bit, and dX is the sum of the members' dX."""
    import torch
    from paper_2305_14152_amd import peqa
    _log("stacked bits=%d Ns=%s K=%d T=%d g=%d" % (bits, Ns, K, T, group))
    seed = 17000 + bits * 1000 + sum(Ns) + K + T + group
    Ws = [synth.normal_f32(seed + 10 * j, (N, K), 0.02) for j, N in enumerate(Ns)]
    members = [gpu.GpuLayer(W, bits, group) for W in Ws]
    # the stacked layer, quantized through slices of its own arrays
    Nsum = sum(Ns)
    L = peqa.layout(Nsum, K, bits, group)
    G = L.groups
    packed = torch.empty(peqa.packed_words(L), dtype=torch.int32, device="cuda")
    s0 = torch.empty((Nsum, G), dtype=torch.float32, device="cuda")
    z0 = torch.empty((Nsum, G), dtype=torch.uint8, device="cuda")
    w_off = n_off = 0
    for m in members:
        nw = peqa.packed_words(m.L)
        peqa.quantize(m.L, m.W0, packed[w_off:w_off + nw], s0[n_off:n_off + m.N], z0[n_off:n_off + m.N])
        w_off += nw
        n_off += m.N
    torch.cuda.synchronize()
    assert w_off == packed.numel()
    whole = gpu.GpuLayer(np.concatenate(Ws), bits, group)          # the stack quantized as one matrix
    assert (gpu.to_host(packed) == gpu.to_host(whole.packed)).all()
    assert (gpu.to_host(s0).view(np.uint32) == gpu.to_host(whole.s0).view(np.uint32)).all()
    assert (gpu.to_host(z0) == gpu.to_host(whole.z0)).all()
    assert (gpu.to_host(packed) == np.concatenate([gpu.to_host(m.packed) for m in members])).all()

    X = synth.normal_bf16(seed + 1, (T, K), 1.0)
    dYs = [synth.normal_bf16(seed + 2 + j, (T, N), 1.0) for j, N in enumerate(Ns)]
    dss = [synth.normal_f32(seed + 50 + j, (N, G), 1e-3) for j, N in enumerate(Ns)]
    ds_all = np.concatenate(dss)
    Y = whole.fwd(X, ds_all)
    Yh = gpu.to_host(Y)
    n_off = 0
    for m, ds in zip(members, dss):
        assert (Yh[:, n_off:n_off + m.N] == gpu.to_host(m.fwd(X, ds))).all()
        n_off += m.N
    if T <= 16:
        return                                                     # the backward takes T of any size; one case is enough
    dX, dds = whole.bwd(X, np.concatenate(dYs, axis=1), ds_all)
    ddsh = gpu.to_host(dds)
    dXref = np.zeros((T, K))
    n_off = 0
    for m, W, ds, dY in zip(members, Ws, dss, dYs):
        _, g_m = m.bwd(X, dY, ds)                                  # both gradients, as for the stacked layer: the same kernel form
        assert (ddsh[n_off:n_off + m.N].view(np.uint32) == gpu.to_host(g_m).view(np.uint32)).all()
        codes, s0_m, z0_m = oracle.quantize(W, bits, group)
        dXm, gref, _ = oracle.bwd(codes, s0_m, ds, z0_m, X, dY, group)
        gpu.assert_scale_grad_close(ddsh[n_off:n_off + m.N], gref)
        dXref += dXm
        n_off += m.N
    assert np.abs(gpu.bf16_dev_to_f64(dX) - dXref).max() <= Y_TOL * np.abs(dXref).max()


@pytest.mark.parametrize("bits,group", [(4, 0), (3, 0), (4, 128), (3, 64)])
def test_zero_and_negative_scales(gpu, oracle, bits, group):
    """The trained scale s0 + ds may reach zero or change sign: Y and dX follow it linearly, the scale
    gradient does not depend on it.  Token counts that are exact tile multiples, and both forward paths."""
    N, K = 256, 512
    seed = 15000 + bits * 100 + group
    W = synth.normal_f32(seed, (N, K), 0.02)
    layer = gpu.GpuLayer(W, bits, group)
    codes, s0, z0 = _check_quant(gpu, oracle, layer, W, bits, group)
    ds = (-s0).copy()
    ds[N // 2:] = -2.5 * s0[N // 2:]            # first half of the channels: s = 0; second half: negative
    for T in (8, 128, 256):
        X = synth.normal_bf16(seed + T, (T, K), 1.0)
        dY = synth.normal_bf16(seed + T + 1, (T, N), 1.0)
        Y = gpu.bf16_dev_to_f64(layer.fwd(X, ds))
        Yref = oracle.fwd(codes, s0, ds, z0, X, group)
        assert (Y[:, :N // 2] == 0).all()
        assert np.abs(Y - Yref).max() <= Y_TOL * np.abs(Yref).max()
        if T > 16:
            dX, dds = layer.bwd(X, dY, ds)
            dXref, gref, _ = oracle.bwd(codes, s0, ds, z0, X, dY, group)
            assert np.abs(gpu.bf16_dev_to_f64(dX) - dXref).max() <= Y_TOL * np.abs(dXref).max()
            g = gpu.to_host(dds).astype(np.float64)
            gpu.assert_scale_grad_close(g, gref)
            # independent of the scale (asked for alone the contraction may run in its other form: same products,
            # another order of addition)
            _, dds0 = layer.bwd(X, dY, None, want_dX=False)
            assert np.linalg.norm(gpu.to_host(dds0).astype(np.float64) - g) <= 1e-5 * np.linalg.norm(g)
            _, dds1 = layer.bwd(X, dY, ds, want_dX=False)
            assert (gpu.to_host(dds0) == gpu.to_host(dds1)).all()


@pytest.mark.parametrize("bits,N,K,T", [
    (4, 384, 640, 200),     # ragged token tile, half-empty column tile
    (3, 512, 384, 129),
    (4, 128, 128, 1),       # one token: still the tiled contraction
    (3, 256, 896, 300),     # 5 slices of 64 rows, the last ragged
    (4, 640, 1152, 64),     # exactly one slice
])
def test_kept_product_training_parity(gpu, oracle, bits, N, K, T):
    """Forward that keeps P = X (Q - z0)^T and the backward that takes the scale gradient from it."""
    _log("kept product bits=%d N=%d K=%d T=%d" % (bits, N, K, T))
    seed = 9100 + bits * 1000 + N + K + T
    W = synth.normal_f32(seed, (N, K), 0.02)
    X = synth.normal_bf16(seed + 1, (T, K), 1.0)
    dY = synth.normal_bf16(seed + 2, (T, N), 1.0)
    layer = gpu.GpuLayer(W, bits, 0)
    codes, s0, z0 = _check_quant(gpu, oracle, layer, W, bits, 0)
    ds = synth.normal_f32(seed + 3, s0.shape, 1.0) * 0.05 * s0
    Yk, P = layer.fwd_keep(X, ds)
    Yref = oracle.fwd(codes, s0, ds, z0, X, 0)
    assert np.abs(gpu.bf16_dev_to_f64(Yk) - Yref).max() <= Y_TOL * np.abs(Yref).max()
    if T > 16:                                          # the same contraction kernel as the plain forward
        assert (gpu.to_host(Yk) == gpu.to_host(layer.fwd(X, ds))).all()
    # P against the oracle's forward with unit scales (fp32 accumulation of exact bf16 x integer products)
    Pref = oracle.fwd(codes, np.ones_like(s0), None, z0, X, 0)
    Ph = gpu.to_host(P).astype(np.float64)
    assert np.abs(Ph - Pref).max() <= 1e-5 * np.abs(Pref).max()
    dXk, ddsk = layer.bwd_kept(P, dY, ds)
    dXref, gref, _ = oracle.bwd(codes, s0, ds, z0, X, dY, 0)
    assert np.abs(gpu.bf16_dev_to_f64(dXk) - dXref).max() <= Y_TOL * np.abs(dXref).max()
    g = gpu.to_host(ddsk).astype(np.float64)
    err, _ = gpu.assert_scale_grad_close(g, gref)
    _log("  dds rel-L2 from the kept product: %.2e" % err)
    # skips, and agreement with the recomputing backward
    dX2, dds2 = layer.bwd(X, dY, ds)
    dX2o, _ = layer.bwd(X, dY, ds, want_dds=False)
    assert (gpu.to_host(dXk) == gpu.to_host(dX2o)).all()           # the same dX launch
    # with both gradients the recomputing backward may run the contraction in its other form: a last bf16 bit
    assert np.abs(gpu.bf16_dev_to_f64(dXk) - gpu.bf16_dev_to_f64(dX2)).max() <= 2.0 ** -7 * np.abs(dXref).max()
    assert np.linalg.norm(g - gpu.to_host(dds2)) <= 1e-5 * np.linalg.norm(gref)
    only_dx, none = layer.bwd_kept(None, dY, ds, want_dds=False)
    assert none is None and (gpu.to_host(only_dx) == gpu.to_host(dXk)).all()
    none, only_g = layer.bwd_kept(P, dY, ds, want_dX=False)
    assert none is None and (gpu.to_host(only_g) == gpu.to_host(ddsk)).all()


@pytest.mark.parametrize("bits,N,K,T,group", [
    (4, 384, 640, 200, 0),      # per-channel, tiled contraction
    (3, 256, 896, 300, 0),
    (4, 256, 512, 5, 0),        # matrix-vector forward
    (3, 384, 768, 16, 128),
    (4, 256, 1024, 150, 128),   # group-wise
    (3, 384, 768, 130, 64),
    (4, 256, 768, 70, 192),
    (3, 128, 1408, 90, 128),    # 11 groups: two group chunks of the zero-point reduction, the second ragged
])
def test_zero_point_training_parity(gpu, oracle, bits, N, K, T, group):
    """Zero-points z = z0 + dz as trainable parameters: forward, dX, scale and zero-point gradients."""
    _log("zero-point training bits=%d N=%d K=%d T=%d g=%d" % (bits, N, K, T, group))
    seed = 9500 + bits * 1000 + N + K + T + group
    W = synth.normal_f32(seed, (N, K), 0.02)
    X = synth.normal_bf16(seed + 1, (T, K), 1.0)
    dY = synth.normal_bf16(seed + 2, (T, N), 1.0)
    layer = gpu.GpuLayer(W, bits, group)
    codes, s0, z0 = _check_quant(gpu, oracle, layer, W, bits, group)
    ds = synth.normal_f32(seed + 3, s0.shape, 1.0) * 0.05 * s0
    dz = synth.normal_f32(seed + 4, s0.shape, 0.5)
    Y = gpu.bf16_dev_to_f64(layer.fwd_z(X, ds, dz))
    Yref = oracle.fwd_z(codes, s0, ds, z0, dz, X, group)
    assert np.abs(Y - Yref).max() <= Y_TOL * np.abs(Yref).max()
    # without dz it is the plain forward, bit for bit
    assert (gpu.to_host(layer.fwd_z(X, ds, None)) == gpu.to_host(layer.fwd(X, ds))).all()
    dX, dds, ddz = layer.bwd_z(X, dY, ds, dz)
    dXref, gs_ref, gz_ref = oracle.bwd_z(codes, s0, ds, z0, dz, X, dY, group)
    assert np.abs(gpu.bf16_dev_to_f64(dX) - dXref).max() <= Y_TOL * np.abs(dXref).max()
    gs = gpu.to_host(dds).astype(np.float64)
    gz = gpu.to_host(ddz).astype(np.float64)
    es, _ = gpu.assert_scale_grad_close(gs, gs_ref, "d_ds")
    ez, _ = gpu.assert_scale_grad_close(gz, gz_ref, "d_dz")
    _log("  rel-L2: d_ds %.2e  d_dz %.2e" % (es, ez))
    # the zero-point gradient alone (zero-points only, Appendix K), and it ignores dz
    none_x, none_s, only_z = layer.bwd_z(X, dY, ds, None, want_dX=False, want_dds=False)
    assert none_x is None and none_s is None
    assert (gpu.to_host(only_z) == gpu.to_host(ddz)).all()
    # one AdamW step on dz against the oracle's (no weight decay on zero-points)
    import torch
    dzd = gpu.to_dev(dz)
    m = torch.zeros_like(dzd); v = torch.zeros_like(dzd)
    from paper_2305_14152_amd import peqa
    lr = float(np.float32(1e-2))
    b1, b2, eps = (float(np.float32(x)) for x in (0.9, 0.999, 1e-8))
    peqa.scale_update(dzd.numel(), dzd, ddz, m, v, layer.s0, lr=lr, step=1)
    torch.cuda.synchronize()
    n = dz.size
    ref = oracle.adamw(dz.astype(np.float64).ravel(), gpu.to_host(ddz).astype(np.float64).ravel(), np.zeros(n),
                       np.zeros(n), s0.astype(np.float64).ravel(), lr, b1, b2, eps, 0.0, 1)
    assert np.abs(gpu.to_host(dzd).ravel() - ref[0]).max() <= 1e-6 * max(1.0, np.abs(ref[0]).max())


@pytest.mark.parametrize("bits,N,K,T,group", [(4, 384, 768, 200, 128), (3, 256, 640, 130, 64), (3, 640, 512, 1, 256)])
def test_groupwise_scale_gradient_both_routes(gpu, oracle, options, bits, N, K, T, group):
    """The group-wise scale gradient by the contraction over tokens (default) and by the contraction over
    features (option PEQA_OPT_GROUPED_DDS = 1): each against the oracle."""
    from paper_2305_14152_amd import peqa
    _log("both routes bits=%d N=%d K=%d T=%d g=%d" % (bits, N, K, T, group))
    seed = 9800 + bits * 1000 + N + K + T + group
    W = synth.normal_f32(seed, (N, K), 0.02)
    X = synth.normal_bf16(seed + 1, (T, K), 1.0)
    dY = synth.normal_bf16(seed + 2, (T, N), 1.0)
    layer = gpu.GpuLayer(W, bits, group)
    codes, s0, z0 = _check_quant(gpu, oracle, layer, W, bits, group)
    _, gref, _ = oracle.bwd(codes, s0, None, z0, X, dY, group, want_dX=False)
    got = {}
    for route in ("tokens", "pairs"):
        options(peqa.PEQA_OPT_GROUPED_DDS, int(route == "pairs"))
        _, dds = layer.bwd(X, dY, None, want_dX=False)
        got[route] = gpu.to_host(dds).astype(np.float64)
        err, _ = gpu.assert_scale_grad_close(got[route], gref, route)
        _log("  %s: rel-L2 %.2e" % (route, err))
    assert np.linalg.norm(got["tokens"] - got["pairs"]) <= 1e-4 * np.linalg.norm(gref)


@pytest.mark.parametrize("bits,N,K,group,n,m", [
    (4, 256, 512, 0, 20, 0.5),
    (3, 384, 1152, 0, 16, 0.4),
    (4, 128, 4096, 128, 12, 0.6),     # 8 register vectors per thread, 32 groups
    (3, 256, 640, 64, 24, 0.5),
    (4, 128, 6144, 0, 8, 0.7),        # 12 vectors per thread: the 16-vector instantiation
    (3, 128, 11008, 0, 6, 0.5),       # 22 vectors per thread: the 24-vector instantiation, ragged last step
    (4, 256, 256, 0, 1, 0.5),         # a single ratio is the plain quantizer
])
def test_quantize_search_parity(gpu, oracle, bits, N, K, group, n, m):
    """Error-minimising initialisation: scales, zero-points and packed codes bit for bit, except where two
    candidates tie to within the rounding of the error sums (then either is right)."""
    import torch
    from paper_2305_14152_amd import peqa
    _log("search bits=%d N=%d K=%d g=%d n=%d min=%.2f" % (bits, N, K, group, n, m))
    seed = 9900 + bits * 1000 + N + K + group
    W = synth.normal_f32(seed, (N, K), 0.02)
    W[::3, ::41] *= 5.0                                              # outliers, so that clipping pays
    W[5, :] = 0.0                                                    # a degenerate row
    L = peqa.layout(N, K, bits, group)
    G = L.groups
    Wd = gpu.to_dev(W)
    packed = torch.empty(peqa.packed_words(L), dtype=torch.int32, device="cuda")
    s0 = torch.empty((N, G), dtype=torch.float32, device="cuda")
    z0 = torch.empty((N, G), dtype=torch.uint8, device="cuda")
    peqa.quantize_search(L, Wd, n, m, packed, s0, z0)
    torch.cuda.synchronize()
    codes, rs0, rz0, choice = oracle.quantize_search(W, bits, group, n, m)
    gs0, gz0 = gpu.to_host(s0), gpu.to_host(z0)
    same = (gs0.view(np.uint32) == rs0.view(np.uint32)) & (gz0 == rz0)
    _log("  groups kept beyond the plain range: %d of %d; differing from the oracle: %d"
         % (int((choice > 0).sum()), choice.size, int((~same).sum())))
    gcodes = oracle.unpack(gpu.to_host(packed, np.uint32), N, K, bits)
    gsz = K // G
    if not same.all():
        # a different candidate is acceptable only as a tie: equal reconstruction error to 1e-12
        Wg = W.astype(np.float64).reshape(N, G, gsz)
        e_ref = ((Wg - oracle.dequant(codes, rs0, None, rz0, group).reshape(N, G, gsz)) ** 2).sum(axis=2)
        e_gpu = ((Wg - oracle.dequant(gcodes, gs0, None, gz0, group).reshape(N, G, gsz)) ** 2).sum(axis=2)
        assert (np.abs(e_gpu - e_ref)[~same] <= 1e-12 * e_ref[~same]).all()
        assert (~same).sum() <= max(1, same.size // 1000)
    ok = np.repeat(same, gsz, axis=1)
    assert (gcodes[ok] == codes[ok]).all()
    if n == 1:
        plain = oracle.quantize(W, bits, group)
        assert same.all() and (gcodes == plain[0]).all()


def test_graph_capture_replays_match_eager(gpu, oracle):
    """Forward + backward captured in a HIP graph: several replays, with eager work and
    synchronisation between them, all equal to the eager results."""
    import torch
    from paper_2305_14152_amd import peqa
    N, K, T = 384, 512, 200
    W = synth.normal_f32(77, (N, K), 0.02)
    layer = gpu.GpuLayer(W, 4, 0)
    X = gpu.to_dev(synth.normal_bf16(78, (T, K), 1.0))
    dY = gpu.to_dev(synth.normal_bf16(79, (T, N), 1.0))
    Y = torch.zeros((T, N), dtype=torch.int16, device="cuda")
    dX = torch.zeros((T, K), dtype=torch.int16, device="cuda")
    dds = torch.zeros((N, 1), dtype=torch.float32, device="cuda")
    nb = max(peqa.workspace_bytes(layer.L, T, peqa.PEQA_OP_FWD), peqa.workspace_bytes(layer.L, T, peqa.PEQA_OP_BWD))
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")

    def run(stream):
        peqa.linear_fwd(layer.L, layer.packed, layer.s0, None, layer.z0, X, T, Y, ws, nb, stream)
        peqa.linear_bwd(layer.L, layer.packed, layer.s0, None, layer.z0, X, dY, T, dX, dds, ws, nb, stream)

    run(torch.cuda.current_stream().cuda_stream)      # eager (also creates the library's stream before capture)
    torch.cuda.synchronize()
    want = (Y.clone(), dX.clone(), dds.clone())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        run(torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        for t in (Y, dX, dds):
            t.fill_(7)                                # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert (Y == want[0]).all() and (dX == want[1]).all() and (dds == want[2]).all(), rep


def test_quantizer_edge_rows(gpu, oracle):
    """Degenerate, one-sided, tie-laden and outlier rows go through the same decisions."""
    N, K = 128, 256
    W = synth.normal_f32(42, (N, K), 0.02)
    W[0] = 0.0
    W[1] = 0.25
    W[2] = -np.linspace(0, 1, K, dtype=np.float32)
    W[3, :] = 0.0; W[3, 0], W[3, 1] = -8.0, 7.0; W[3, 2:8] = [0.5, 1.5, 2.5, -0.5, -1.5, 3.5]
    W[4] *= 1e-30                               # tiny range
    W[5] *= 1e30                                # huge range
    W[6, ::7] = 0.0
    W[7, 5] = 3.0                               # single outlier
    for bits in (3, 4):
        for group in (0, 64, 128):
            layer = gpu.GpuLayer(W, bits, group)
            _check_quant(gpu, oracle, layer, W, bits, group)


def test_outlier_weights_3bit(gpu, oracle):
    """Config 2's weight distribution (0.1% entries from N(0, 0.2)) on a slab."""
    W = synth.weights(2, 0, N=256, K=1024)
    layer = gpu.GpuLayer(W, 3, 0)
    codes, s0, z0 = _check_quant(gpu, oracle, layer, W, 3, 0)
    X = synth.activations(2, 0, T=160, K=1024)
    dY = synth.output_grads(2, 0, T=160, N=256)
    e = _check_fwd_bwd(gpu, oracle, layer, codes, s0, z0, X, dY, None, 0)
    _log("  errors: %.2e %.2e" % e)


def test_backward_is_deterministic_and_skips(gpu, oracle):
    W = synth.normal_f32(90, (256, 512), 0.02)
    X = synth.normal_bf16(91, (300, 512), 1.0)
    dY = synth.normal_bf16(92, (300, 256), 1.0)
    layer = gpu.GpuLayer(W, 4, 0)
    dX1, g1 = layer.bwd(X, dY)
    dX2, g2 = layer.bwd(X, dY)
    assert (gpu.to_host(g1).view(np.uint32) == gpu.to_host(g2).view(np.uint32)).all()
    assert (gpu.to_host(dX1) == gpu.to_host(dX2)).all()
    # One gradient alone: a launch of its own, which may run the contraction in its other form (the same products
    # added in another order); twice the same bits, and the other call's to rounding.
    dX3, g3 = layer.bwd(X, dY, want_dds=False)
    dX3b, _ = layer.bwd(X, dY, want_dds=False)
    assert g3 is None and (gpu.to_host(dX3) == gpu.to_host(dX3b)).all()
    d1, d3 = gpu.bf16_dev_to_f64(dX1), gpu.bf16_dev_to_f64(dX3)
    assert np.abs(d3 - d1).max() <= 2.0 ** -7 * np.abs(d1).max()
    dX4, g4 = layer.bwd(X, dY, want_dX=False)
    g1h, g4h = gpu.to_host(g1).astype(np.float64), gpu.to_host(g4).astype(np.float64)
    assert dX4 is None and np.linalg.norm(g4h - g1h) <= 1e-5 * np.linalg.norm(g1h)
    # the scale gradient does not depend on the scale
    _, g5 = layer.bwd(X, dY, ds=np.full((256, 1), 0.01, np.float32), want_dX=False)
    assert (gpu.to_host(g5).view(np.uint32) == gpu.to_host(g4).view(np.uint32)).all()


def test_scale_update_parity(gpu, oracle):
    import torch
    from paper_2305_14152_amd import peqa
    n = 42496
    r = np.random.default_rng(3)
    s0 = (np.abs(r.standard_normal(n)) * 0.01 + 1e-3).astype(np.float32)
    ds = (r.standard_normal(n) * 1e-4).astype(np.float32)
    m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    d = {k: gpu.to_dev(a) for k, a in dict(s0=s0, ds=ds, m=m, v=v).items()}
    # the optimizer constants cross the boundary as fp32: the oracle gets those same values
    lr, b1, b2, eps, wd = (float(np.float32(x)) for x in (1e-3, 0.9, 0.999, 1e-8, 0.01))
    for step in range(1, 4):
        g = (r.standard_normal(n) * 10.0 ** r.uniform(-4, 1, n)).astype(np.float32)
        g[::97] = 0.0
        # each call is checked on its own: the oracle starts from the state the GPU call starts from
        before = tuple(gpu.to_host(d[k]).astype(np.float64) for k in ("ds", "m", "v"))
        peqa.scale_update(n, d["ds"], gpu.to_dev(g), d["m"], d["v"], d["s0"], lr=lr, beta1=b1, beta2=b2,
                          eps=eps, weight_decay=wd, step=step)
        torch.cuda.synchronize()
        ref = oracle.adamw(before[0], g, before[1], before[2], s0, lr, b1, b2, eps, wd, step)
        got = gpu.to_host(d["ds"]).astype(np.float64)
        # ds element by element, 1e-6 relative.  ds_new = ds - update is a difference, so "relative" is taken
        # against its two terms: |got - ref| <= 1e-6 (|ds| + |update|), which is 1e-6 of ds_new itself wherever the
        # two do not cancel
        floor = 1e-6 * (np.abs(before[0]) + np.abs(ref[0] - before[0]))
        assert (np.abs(got - ref[0]) <= floor).all(), float((np.abs(got - ref[0]) / floor).max())
        # m is a difference of two fp32 terms when the gradient changes sign: bound by their magnitudes
        m_bound = 1e-6 * (b1 * np.abs(before[1]) + (1 - b1) * np.abs(g)) + 1e-30
        assert (np.abs(gpu.to_host(d["m"]) - ref[1]) <= m_bound).all()
        np.testing.assert_allclose(gpu.to_host(d["v"]), ref[2], rtol=1e-6, atol=1e-30)


def test_scale_update_multi_equals_single_calls(gpu):
    """Several parameter vectors in one launch: bit-identical to one peqa_scale_update per vector."""
    import torch
    from paper_2305_14152_amd import peqa
    r = np.random.default_rng(11)
    sizes = [4096, 11008, 128, 4096 * 32, 5120 * 40 + 256]
    def fresh():
        out = []
        for n in sizes:
            s0 = (np.abs(r.standard_normal(n)) * 0.01 + 1e-3).astype(np.float32)
            t = dict(s0=s0, ds=(r.standard_normal(n) * 1e-4).astype(np.float32), g=r.standard_normal(n).astype(np.float32),
                     m=(r.standard_normal(n) * 0.1).astype(np.float32), v=np.abs(r.standard_normal(n)).astype(np.float32))
            out.append(t)
        return out
    host = fresh()
    a = [{k: gpu.to_dev(x) for k, x in t.items()} for t in host]
    b = [{k: gpu.to_dev(x) for k, x in t.items()} for t in host]
    kw = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=3)
    peqa.scale_update_multi([(t["ds"].numel(), t["ds"], t["g"], t["m"], t["v"], t["s0"]) for t in a], **kw)
    for t in b:
        peqa.scale_update(t["ds"].numel(), t["ds"], t["g"], t["m"], t["v"], t["s0"], **kw)
    torch.cuda.synchronize()
    for ta, tb, th in zip(a, b, host):
        for k in ("ds", "m", "v"):
            assert (gpu.to_host(ta[k]).view(np.uint32) == gpu.to_host(tb[k]).view(np.uint32)).all(), k
            assert not (gpu.to_host(ta[k]) == th[k]).all()           # and something was updated


@pytest.mark.parametrize("bits,group,T", [(4, 0, 150), (3, 128, 150), (4, 0, 9), (3, 64, 16)])
def test_buffers_at_16_byte_offsets(gpu, oracle, bits, group, T):
    """The boundary asks for 16-byte alignment only: every tensor here starts 16 bytes into its allocation."""
    import torch
    from paper_2305_14152_amd import peqa
    N, K = 384, 640
    seed = 7700 + bits + group + T
    W = synth.normal_f32(seed, (N, K), 0.02)
    X = synth.normal_bf16(seed + 1, (T, K), 1.0)
    dY = synth.normal_bf16(seed + 2, (T, N), 1.0)
    codes, s0, z0 = oracle.quantize(W, bits, group)
    L = peqa.layout(N, K, bits, group)
    G = L.groups

    def shifted(a, torch_dtype):
        """A device copy of `a` that starts 16 bytes past a 256-byte aligned allocation."""
        flat = np.ascontiguousarray(a).reshape(-1)
        pad = 16 // flat.dtype.itemsize
        buf = torch.zeros(flat.size + pad, dtype=torch_dtype, device="cuda")
        view = buf[pad:]
        view.copy_(gpu.to_dev(flat).view(torch_dtype))
        assert view.data_ptr() % 256 == 16
        return view

    Wd = shifted(W, torch.float32)
    packed = torch.zeros(peqa.packed_words(L) + 4, dtype=torch.int32, device="cuda")[4:]
    s0d = torch.zeros(N * G + 4, dtype=torch.float32, device="cuda")[4:]
    z0d = torch.zeros(N * G + 16, dtype=torch.uint8, device="cuda")[16:]
    peqa.quantize(L, Wd, packed, s0d, z0d)
    torch.cuda.synchronize()
    assert (gpu.to_host(packed, np.uint32) == oracle.pack(codes, bits)).all()
    assert (gpu.to_host(s0d).view(np.uint32) == s0.reshape(-1).view(np.uint32)).all()
    assert (gpu.to_host(z0d) == z0.reshape(-1)).all()
    Xd = shifted(X.view(np.int16), torch.int16)
    dYd = shifted(dY.view(np.int16), torch.int16)
    Y = torch.zeros(T * N + 8, dtype=torch.int16, device="cuda")[8:]
    dX = torch.zeros(T * K + 8, dtype=torch.int16, device="cuda")[8:]
    dds = torch.zeros(N * G + 4, dtype=torch.float32, device="cuda")[4:]
    nb = max(peqa.workspace_bytes(L, T, peqa.PEQA_OP_FWD), peqa.workspace_bytes(L, T, peqa.PEQA_OP_BWD))
    ws = torch.zeros(nb + 16, dtype=torch.uint8, device="cuda")[16:]
    peqa.linear_fwd(L, packed, s0d, None, z0d, Xd, T, Y, ws, nb)
    peqa.linear_bwd(L, packed, s0d, None, z0d, Xd, dYd, T, dX, dds, ws, nb)
    torch.cuda.synchronize()
    Yref = oracle.fwd(codes, s0, None, z0, X, group)
    dXref, gref, _ = oracle.bwd(codes, s0, None, z0, X, dY, group)
    assert np.abs(gpu.bf16_dev_to_f64(Y).reshape(T, N) - Yref).max() <= Y_TOL * np.abs(Yref).max()
    assert np.abs(gpu.bf16_dev_to_f64(dX).reshape(T, K) - dXref).max() <= Y_TOL * np.abs(dXref).max()
    g = gpu.to_host(dds).astype(np.float64).reshape(N, G)
    gpu.assert_scale_grad_close(g, gref)


def test_shared_row_sums_equal_the_plain_calls(gpu, oracle):
    """peqa_row_sums once, then the forward and backward that take the sums: bit-identical to the calls that
    take them themselves; the sums themselves against a plain fp64 sum of the bf16 inputs."""
    import torch
    from paper_2305_14152_amd import peqa
    bits, N, K, T = 4, 384, 640, 200
    W = synth.normal_f32(31, (N, K), 0.02)
    X = synth.normal_bf16(32, (T, K), 1.0)
    dY = synth.normal_bf16(33, (T, N), 1.0)
    layer = gpu.GpuLayer(W, bits, 0)
    Xd, dYd = gpu.to_dev(X), gpu.to_dev(dY)
    rs = torch.empty((T, 2), dtype=torch.float32, device="cuda")
    peqa.row_sums(Xd, T, K, rs)
    torch.cuda.synchronize()
    Xf = synth.bf16_bits_to_f32(X).astype(np.float64)
    ks = (K // 2) // 64 * 64
    ref = np.stack([Xf[:, :ks].sum(axis=1), Xf[:, ks:].sum(axis=1)], axis=1)
    assert np.abs(gpu.to_host(rs) - ref).max() <= 1e-5 * np.abs(Xf).sum(axis=1).max()
    # forward
    Y1 = torch.empty((T, N), dtype=torch.int16, device="cuda")
    items = [(layer.L, layer.packed, layer.s0, None, layer.z0, Y1)]
    nb = peqa.workspace_bytes_fused(items, T)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    peqa.linear_fwd_fused_rs(items, Xd, rs, T, ws, nb)
    torch.cuda.synchronize()
    assert (gpu.to_host(Y1) == gpu.to_host(layer.fwd(Xd, None))).all()
    # backward
    dX0, g0 = layer.bwd(Xd, dYd, None)
    dX1 = torch.empty_like(dX0); g1 = torch.empty_like(g0)
    wsb, nbb = layer.workspace(T, peqa.PEQA_OP_BWD)
    peqa.linear_bwd_rs(layer.L, layer.packed, layer.s0, None, layer.z0, Xd, rs, dYd, T, dX1, g1, wsb, nbb)
    torch.cuda.synchronize()
    assert (gpu.to_host(dX1) == gpu.to_host(dX0)).all()
    assert (gpu.to_host(g1).view(np.uint32) == gpu.to_host(g0).view(np.uint32)).all()


def test_trace_reports_kernels(gpu):
    from paper_2305_14152_amd import peqa
    W = synth.normal_f32(5, (256, 256), 0.02)
    layer = gpu.GpuLayer(W, 4, 0)
    X = synth.normal_bf16(6, (64, 256), 1.0)
    peqa.trace_begin(16)
    layer.fwd(X)
    out = peqa.trace_end()
    assert out["gemm_y"][0] == 1 and out["gemm_y"][1] > 0 and "rowsum" in out
