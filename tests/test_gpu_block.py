"""GPU parity of the block-level calls (peqa_block_fwd / peqa_block_bwd): several layers of different shapes and
inputs behind one call, every member against the oracle and against the single-layer calls."""
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


class Member:
    """One layer of a block with its own input, on both sides."""

    def __init__(self, gpu, oracle, seed, bits, N, K, group, T, X=None, with_ds=True):
        self.N, self.K, self.group = N, K, group
        W = synth.normal_f32(seed, (N, K), 0.02)
        self.layer = gpu.GpuLayer(W, bits, group)
        self.codes, self.s0, self.z0 = oracle.quantize(W, bits, group)
        self.ds = synth.normal_f32(seed + 1, self.s0.shape, 1e-3) if with_ds else None
        self.dsd = gpu.to_dev(self.ds) if with_ds else None
        self.X = X if X is not None else synth.normal_bf16(seed + 2, (T, K), 1.0)
        self.dY = synth.normal_bf16(seed + 3, (T, N), 1.0)


def _run_block(gpu, members, T, backward, share_row_sums=False):
    import torch
    from paper_2305_14152_amd import peqa
    xdev = {}
    dicts = []
    for m in members:
        if id(m.X) not in xdev:
            xdev[id(m.X)] = (gpu.to_dev(m.X), torch.zeros((T, 2), dtype=torch.float32, device="cuda"))
        Xd, rs = xdev[id(m.X)]
        d = dict(L=m.layer.L, packed=m.layer.packed, s0=m.layer.s0, z0=m.layer.z0, ds=m.dsd, X=Xd,
                 Y=torch.zeros((T, m.N), dtype=torch.int16, device="cuda"), dY=gpu.to_dev(m.dY),
                 dX=torch.zeros((T, m.K), dtype=torch.int16, device="cuda"),
                 d_ds=torch.zeros(m.s0.shape, dtype=torch.float32, device="cuda"),
                 row_sums=rs if share_row_sums else None)
        dicts.append(d)
    items = peqa.block_items(dicts)
    nb = peqa.block_workspace_bytes(items, T, peqa.PEQA_OP_FWD)
    assert nb > 0
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    peqa.block_fwd(items, T, ws, nb)
    if backward:
        nbb = peqa.block_workspace_bytes(items, T, peqa.PEQA_OP_BWD)
        assert nbb > 0
        wsb = torch.empty(nbb, dtype=torch.uint8, device="cuda")
        peqa.block_bwd(items, T, wsb, nbb)
    torch.cuda.synchronize()
    return dicts


BLOCKS = [
    # (bits, group, [(N, K, input index)]): members with equal input index read one X
    (4, 0, [(256, 512, 0), (384, 512, 0), (128, 512, 1), (512, 1152, 2)]),
    (3, 128, [(256, 512, 0), (256, 512, 0), (256, 512, 1), (384, 512, 2), (512, 1408, 3)]),
    (3, 0, [(1280, 640, 0), (640, 1280, 1)]),
    (4, 64, [(128, 256, 0), (256, 768, 1), (128, 128, 2)]),
    (4, 0, [(128, 128, 0)] * 8),
]


@pytest.mark.parametrize("bits,group,shapes", BLOCKS)
@pytest.mark.parametrize("T", [1, 7, 16, 40, 200])
def test_block_forward_parity(gpu, oracle, bits, group, shapes, T):
    print("block forward bits=%d g=%d T=%d shapes=%s" % (bits, group, T, shapes), flush=True)
    seed = 31000 + 100 * bits + group + T
    inputs = {}
    members = []
    for j, (N, K, xi) in enumerate(shapes):
        if xi not in inputs:
            inputs[xi] = synth.normal_bf16(seed + 7 * xi, (T, K), 1.0)
        members.append(Member(gpu, oracle, seed + 50 * j, bits, N, K, group, T, X=inputs[xi], with_ds=(j % 2 == 0)))
    dicts = _run_block(gpu, members, T, backward=False, share_row_sums=(T % 2 == 0))
    for m, d in zip(members, dicts):
        Yref = oracle.fwd(m.codes, m.s0, m.ds, m.z0, m.X, group)
        Y = gpu.bf16_dev_to_f64(d["Y"])
        assert np.abs(Y - Yref).max() <= Y_TOL * np.abs(Yref).max(), (m.N, m.K)
        single = gpu.bf16_dev_to_f64(m.layer.fwd(d["X"], m.dsd))
        # the same products, possibly added in another order (other slicing or kernel form): a last bf16 bit
        assert np.abs(Y - single).max() <= 2.0 ** -7 * np.abs(Yref).max()


@pytest.mark.parametrize("bits,group,shapes", BLOCKS[:4])
@pytest.mark.parametrize("T", [40, 200, 300])
def test_block_backward_parity(gpu, oracle, bits, group, shapes, T):
    print("block backward bits=%d g=%d T=%d shapes=%s" % (bits, group, T, shapes), flush=True)
    seed = 33000 + 100 * bits + group + T
    inputs = {}
    members = []
    for j, (N, K, xi) in enumerate(shapes):
        if xi not in inputs:
            inputs[xi] = synth.normal_bf16(seed + 7 * xi, (T, K), 1.0)
        members.append(Member(gpu, oracle, seed + 50 * j, bits, N, K, group, T, X=inputs[xi], with_ds=(j % 2 == 1)))
    for share in (False, True):
        dicts = _run_block(gpu, members, T, backward=True, share_row_sums=share)
        for m, d in zip(members, dicts):
            dXref, gref, _ = oracle.bwd(m.codes, m.s0, m.ds, m.z0, m.X, m.dY, group)
            dX = gpu.bf16_dev_to_f64(d["dX"])
            assert np.abs(dX - dXref).max() <= Y_TOL * np.abs(dXref).max(), (m.N, m.K)
            gpu.assert_scale_grad_close(gpu.to_host(d["d_ds"]), gref)


def test_block_skips_and_errors(gpu, oracle):
    """NULL dX / d_ds per item are skipped; mixed bit widths and missing workspace are refused."""
    import ctypes
    import torch
    from paper_2305_14152_amd import peqa
    T = 150
    a = Member(gpu, oracle, 35000, 4, 256, 512, 0, T)
    b = Member(gpu, oracle, 35100, 4, 384, 256, 0, T)
    dicts = []
    for m, (want_dx, want_g) in zip((a, b), ((True, False), (False, True))):
        dicts.append(dict(L=m.layer.L, packed=m.layer.packed, s0=m.layer.s0, z0=m.layer.z0, ds=None, X=gpu.to_dev(m.X),
                          dY=gpu.to_dev(m.dY), Y=None,
                          dX=torch.full((T, m.K), 7, dtype=torch.int16, device="cuda") if want_dx else None,
                          d_ds=torch.full(m.s0.shape, 7.0, dtype=torch.float32, device="cuda") if want_g else None))
    items = peqa.block_items(dicts)
    nb = peqa.block_workspace_bytes(items, T, peqa.PEQA_OP_BWD)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    peqa.block_bwd(items, T, ws, nb)
    torch.cuda.synchronize()
    dXref, _, _ = oracle.bwd(a.codes, a.s0, None, a.z0, a.X, a.dY, 0, want_P=False)
    assert np.abs(gpu.bf16_dev_to_f64(dicts[0]["dX"]) - dXref).max() <= Y_TOL * np.abs(dXref).max()
    _, gref, _ = oracle.bwd(b.codes, b.s0, None, b.z0, b.X, b.dY, 0, want_dX=False)
    gpu.assert_scale_grad_close(gpu.to_host(dicts[1]["d_ds"]), gref)
    lib = peqa.lib()
    assert lib.peqa_block_bwd(2, ctypes.addressof(items), T, None, 0, None) == peqa.PEQA_ERR_WORKSPACE
    c = Member(gpu, oracle, 35200, 3, 128, 128, 0, T)
    mixed = peqa.block_items([dicts[0], dict(L=c.layer.L, packed=c.layer.packed, s0=c.layer.s0, z0=c.layer.z0,
                                             X=gpu.to_dev(c.X), dY=gpu.to_dev(c.dY))])
    assert peqa.block_workspace_bytes(mixed, T, peqa.PEQA_OP_BWD) == 0
    assert lib.peqa_block_bwd(2, ctypes.addressof(mixed), T, ws.data_ptr(), nb, None) == peqa.PEQA_ERR_PARAM
    assert lib.peqa_block_fwd(9, ctypes.addressof(items), T, ws.data_ptr(), nb, None) == peqa.PEQA_ERR_PARAM


def test_block_graph_capture_replays_match_eager(gpu, oracle):
    """The block calls captured in a HIP graph (multi-contraction launches with their auxiliary workgroups, the
    row sums, the T <= 16 launch with its slice sums): replays, with eager work between them, equal the eager
    results bit for bit."""
    import torch
    from paper_2305_14152_amd import peqa
    T = 200
    members = [Member(gpu, oracle, 37000 + 100 * j, 4, N, K, 0, T) for j, (N, K) in enumerate(((384, 512), (256, 1152), (128, 256)))]
    dicts = []
    for m in members:
        dicts.append(dict(L=m.layer.L, packed=m.layer.packed, s0=m.layer.s0, z0=m.layer.z0, ds=m.dsd, X=gpu.to_dev(m.X),
                          Y=torch.zeros((T, m.N), dtype=torch.int16, device="cuda"), dY=gpu.to_dev(m.dY),
                          dX=torch.zeros((T, m.K), dtype=torch.int16, device="cuda"),
                          d_ds=torch.zeros(m.s0.shape, dtype=torch.float32, device="cuda"),
                          row_sums=torch.zeros((T, 2), dtype=torch.float32, device="cuda")))
    items = peqa.block_items(dicts)
    nb = max(peqa.block_workspace_bytes(items, T, op) for op in (peqa.PEQA_OP_FWD, peqa.PEQA_OP_BWD))
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    small = [dict(d, X=d["X"][:5].contiguous(), Y=torch.zeros((5, d["Y"].shape[1]), dtype=torch.int16, device="cuda")) for d in dicts]
    items5 = peqa.block_items(small)
    nb5 = peqa.block_workspace_bytes(items5, 5, peqa.PEQA_OP_FWD)
    ws5 = torch.empty(nb5, dtype=torch.uint8, device="cuda")

    def run(stream):
        peqa.block_fwd(items, T, ws, nb, stream)
        peqa.block_bwd(items, T, ws, nb, stream)
        peqa.block_fwd(items5, 5, ws5, nb5, stream)

    outs = [d[k] for d in dicts for k in ("Y", "dX", "d_ds")] + [d["Y"] for d in small]
    run(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = [t.clone() for t in outs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        run(torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        for t in outs:
            t.fill_(7)                                # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for t, w in zip(outs, want):
            assert (t == w).all(), rep
    # and the eager results are right
    for m, d in zip(members, dicts):
        Yref = oracle.fwd(m.codes, m.s0, m.ds, m.z0, m.X, 0)
        assert np.abs(gpu.bf16_dev_to_f64(d["Y"]) - Yref).max() <= Y_TOL * np.abs(Yref).max()


def test_block_is_deterministic(gpu, oracle):
    """Two block backward calls give the same bits (fixed reduction order, no atomics)."""
    import torch
    T = 300
    members = [Member(gpu, oracle, 38000 + 100 * j, 3, N, K, 0, T) for j, (N, K) in enumerate(((640, 384), (256, 896)))]
    a = _run_block(gpu, members, T, backward=True)
    b = _run_block(gpu, members, T, backward=True)
    for da, db in zip(a, b):
        assert (gpu.to_host(da["d_ds"]).view(np.uint32) == gpu.to_host(db["d_ds"]).view(np.uint32)).all()
        assert (gpu.to_host(da["dX"]) == gpu.to_host(db["dX"])).all()
        assert (gpu.to_host(da["Y"]) == gpu.to_host(db["Y"])).all()


@pytest.mark.parametrize("bits,group", [(3, 128), (4, 192), (4, 64)])
def test_block_groupwise_skips_and_shared_inputs(gpu, oracle, bits, group):
    """Group-wise members of one backward call: some want only dX, some only the scale gradient (among them members
    that read one X, whose transposed copy is made once), and a call in which nobody wants dX (its launch then has
    no tiles, only the workgroups that write the transposed copies).  Twice, for the same bits."""
    import torch
    from paper_2305_14152_amd import peqa
    T = 170
    K = 3 * group * 2 if group != 64 else 512
    print("block group-wise skips bits=%d g=%d K=%d" % (bits, group, K), flush=True)
    X = synth.normal_bf16(39000 + group, (T, K), 1.0)
    members = [Member(gpu, oracle, 39100 + 100 * j + group, bits, N, K, group, T, X=(X if shared else None), with_ds=(j != 1))
               for j, (N, shared) in enumerate(((256, True), (384, True), (128, False), (256, True)))]
    wants = ((True, False), (False, True), (True, True), (False, True))        # (dX, d_ds) per member
    for only_grad in (False, True):
        results = []
        for rep in range(2):
            Xd = gpu.to_dev(X)
            dicts = []
            for m, (want_dx, want_g) in zip(members, wants):
                want_dx = want_dx and not only_grad
                dicts.append(dict(L=m.layer.L, packed=m.layer.packed, s0=m.layer.s0, z0=m.layer.z0, ds=m.dsd,
                                  X=Xd if m.X is X else gpu.to_dev(m.X), dY=gpu.to_dev(m.dY), Y=None,
                                  dX=torch.full((T, m.K), 7, dtype=torch.int16, device="cuda") if want_dx else None,
                                  d_ds=torch.full(m.s0.shape, 7.0, dtype=torch.float32, device="cuda") if want_g else None))
            items = peqa.block_items(dicts)
            nb = peqa.block_workspace_bytes(items, T, peqa.PEQA_OP_BWD)
            ws = torch.full((nb,), 0x5A, dtype=torch.uint8, device="cuda")
            peqa.block_bwd(items, T, ws, nb)
            torch.cuda.synchronize()
            results.append(dicts)
        for m, d, d2 in zip(members, results[0], results[1]):
            dXref, gref, _ = oracle.bwd(m.codes, m.s0, m.ds, m.z0, m.X, m.dY, group)
            if d["dX"] is not None:
                assert np.abs(gpu.bf16_dev_to_f64(d["dX"]) - dXref).max() <= Y_TOL * np.abs(dXref).max(), (m.N, only_grad)
                assert (gpu.to_host(d["dX"]) == gpu.to_host(d2["dX"])).all()
            if d["d_ds"] is not None:
                gpu.assert_scale_grad_close(gpu.to_host(d["d_ds"]), gref)
                assert (gpu.to_host(d["d_ds"]).view(np.uint32) == gpu.to_host(d2["d_ds"]).view(np.uint32)).all()


def test_block_groupwise_graph_capture(gpu, oracle):
    """The block calls on group-wise layers captured in a HIP graph: replays equal the eager results bit for bit."""
    import torch
    from paper_2305_14152_amd import peqa
    T = 200
    members = [Member(gpu, oracle, 39500 + 100 * j, 3, N, K, 128, T) for j, (N, K) in enumerate(((384, 512), (256, 1152), (128, 256)))]
    dicts = []
    for m in members:
        dicts.append(dict(L=m.layer.L, packed=m.layer.packed, s0=m.layer.s0, z0=m.layer.z0, ds=m.dsd, X=gpu.to_dev(m.X),
                          Y=torch.zeros((T, m.N), dtype=torch.int16, device="cuda"), dY=gpu.to_dev(m.dY),
                          dX=torch.zeros((T, m.K), dtype=torch.int16, device="cuda"),
                          d_ds=torch.zeros(m.s0.shape, dtype=torch.float32, device="cuda")))
    items = peqa.block_items(dicts)
    nb = max(peqa.block_workspace_bytes(items, T, op) for op in (peqa.PEQA_OP_FWD, peqa.PEQA_OP_BWD))
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")

    def run(stream):
        peqa.block_fwd(items, T, ws, nb, stream)
        peqa.block_bwd(items, T, ws, nb, stream)

    outs = [d[k] for d in dicts for k in ("Y", "dX", "d_ds")]
    run(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = [t.clone() for t in outs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        run(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        for t in outs:
            t.fill_(7)
        ws.fill_(rep)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for t, w in zip(outs, want):
            assert (t == w).all(), rep
    for m, d in zip(members, dicts):
        dXref, gref, _ = oracle.bwd(m.codes, m.s0, m.ds, m.z0, m.X, m.dY, 128)
        assert np.abs(gpu.bf16_dev_to_f64(d["dX"]) - dXref).max() <= Y_TOL * np.abs(dXref).max()
        gpu.assert_scale_grad_close(gpu.to_host(d["d_ds"]), gref)
