"""Helpers for the GPU parity tests: move seeded host inputs to the device, call the C-ABI
through the binding, bring results back as numpy.  No arithmetic of the method here."""
import numpy as np


def _t():
    import torch
    return torch


def to_dev(a):
    torch = _t()
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).cuda()
    return torch.from_numpy(a).cuda()


def to_host(t, dtype=None):
    a = t.cpu().numpy()
    return a.view(dtype) if dtype is not None else a


class GpuLayer:
    """One PEQA linear resident on the GPU, quantized there by peqa_quantize."""

    def __init__(self, W0, bits, group=0):
        from paper_2305_14152_amd import peqa
        torch = _t()
        self.peqa, self.torch = peqa, torch
        N, K = W0.shape
        self.N, self.K, self.bits, self.group = N, K, bits, group
        self.L = peqa.layout(N, K, bits, group)
        G = self.L.groups
        self.G = G
        self.W0 = to_dev(np.ascontiguousarray(W0, np.float32))
        self.packed = torch.empty(peqa.packed_words(self.L), dtype=torch.int32, device="cuda")
        self.s0 = torch.empty((N, G), dtype=torch.float32, device="cuda")
        self.z0 = torch.empty((N, G), dtype=torch.uint8, device="cuda")
        peqa.quantize(self.L, self.W0, self.packed, self.s0, self.z0)
        self._ws = {}

    def workspace(self, T, op):
        key = (T, op)
        if key not in self._ws:
            nbytes = self.peqa.workspace_bytes(self.L, T, op)
            assert nbytes > 0
            self._ws[key] = (self.torch.empty(nbytes, dtype=self.torch.uint8, device="cuda"), nbytes)
        return self._ws[key]

    def host_quant(self):
        return (to_host(self.packed, np.uint32), to_host(self.s0), to_host(self.z0))

    def fwd(self, X_bits, ds=None):
        torch, peqa = self.torch, self.peqa
        X = to_dev(X_bits) if isinstance(X_bits, np.ndarray) else X_bits
        T = X.shape[0]
        Y = torch.empty((T, self.N), dtype=torch.int16, device="cuda")
        dsd = to_dev(np.ascontiguousarray(ds, np.float32)) if isinstance(ds, np.ndarray) else ds
        ws, nb = self.workspace(T, peqa.PEQA_OP_FWD)
        peqa.linear_fwd(self.L, self.packed, self.s0, dsd, self.z0, X, T, Y, ws, nb)
        torch.cuda.synchronize()
        return Y

    def bwd(self, X_bits, dY_bits, ds=None, want_dX=True, want_dds=True):
        torch, peqa = self.torch, self.peqa
        X = to_dev(X_bits) if isinstance(X_bits, np.ndarray) else X_bits
        dY = to_dev(dY_bits) if isinstance(dY_bits, np.ndarray) else dY_bits
        T = dY.shape[0]
        dX = torch.empty((T, self.K), dtype=torch.int16, device="cuda") if want_dX else None
        dds = torch.empty((self.N, self.G), dtype=torch.float32, device="cuda") if want_dds else None
        dsd = to_dev(np.ascontiguousarray(ds, np.float32)) if isinstance(ds, np.ndarray) else ds
        ws, nb = self.workspace(T, peqa.PEQA_OP_BWD)
        peqa.linear_bwd(self.L, self.packed, self.s0, dsd, self.z0, X, dY, T, dX, dds, ws, nb)
        torch.cuda.synchronize()
        return dX, dds


    def fwd_keep(self, X_bits, ds=None):
        torch, peqa = self.torch, self.peqa
        X = to_dev(X_bits) if isinstance(X_bits, np.ndarray) else X_bits
        T = X.shape[0]
        Y = torch.empty((T, self.N), dtype=torch.int16, device="cuda")
        P = torch.empty((T, self.N), dtype=torch.float32, device="cuda")
        dsd = to_dev(np.ascontiguousarray(ds, np.float32)) if isinstance(ds, np.ndarray) else ds
        ws, nb = self.workspace(T, peqa.PEQA_OP_FWD_KEEP)
        peqa.linear_fwd_keep(self.L, self.packed, self.s0, dsd, self.z0, X, T, Y, P, ws, nb)
        torch.cuda.synchronize()
        return Y, P

    def bwd_kept(self, P, dY_bits, ds=None, want_dX=True, want_dds=True):
        torch, peqa = self.torch, self.peqa
        dY = to_dev(dY_bits) if isinstance(dY_bits, np.ndarray) else dY_bits
        T = dY.shape[0]
        dX = torch.empty((T, self.K), dtype=torch.int16, device="cuda") if want_dX else None
        dds = torch.empty((self.N, self.G), dtype=torch.float32, device="cuda") if want_dds else None
        dsd = to_dev(np.ascontiguousarray(ds, np.float32)) if isinstance(ds, np.ndarray) else ds
        ws, nb = self.workspace(T, peqa.PEQA_OP_BWD_KEPT)
        peqa.linear_bwd_kept(self.L, self.packed, self.s0, dsd, self.z0, P, dY, T, dX, dds, ws, nb)
        torch.cuda.synchronize()
        return dX, dds


    def fwd_z(self, X_bits, ds=None, dz=None):
        torch, peqa = self.torch, self.peqa
        X = to_dev(X_bits) if isinstance(X_bits, np.ndarray) else X_bits
        T = X.shape[0]
        Y = torch.empty((T, self.N), dtype=torch.int16, device="cuda")
        dsd = to_dev(np.ascontiguousarray(ds, np.float32)) if isinstance(ds, np.ndarray) else ds
        dzd = to_dev(np.ascontiguousarray(dz, np.float32)) if isinstance(dz, np.ndarray) else dz
        ws, nb = self.workspace(T, peqa.PEQA_OP_FWD_Z)
        peqa.linear_fwd_z(self.L, self.packed, self.s0, dsd, self.z0, dzd, X, T, Y, ws, nb)
        torch.cuda.synchronize()
        return Y

    def bwd_z(self, X_bits, dY_bits, ds=None, dz=None, want_dX=True, want_dds=True, want_ddz=True):
        torch, peqa = self.torch, self.peqa
        X = to_dev(X_bits) if isinstance(X_bits, np.ndarray) else X_bits
        dY = to_dev(dY_bits) if isinstance(dY_bits, np.ndarray) else dY_bits
        T = dY.shape[0]
        dX = torch.empty((T, self.K), dtype=torch.int16, device="cuda") if want_dX else None
        dds = torch.empty((self.N, self.G), dtype=torch.float32, device="cuda") if want_dds else None
        ddz = torch.empty((self.N, self.G), dtype=torch.float32, device="cuda") if want_ddz else None
        dsd = to_dev(np.ascontiguousarray(ds, np.float32)) if isinstance(ds, np.ndarray) else ds
        dzd = to_dev(np.ascontiguousarray(dz, np.float32)) if isinstance(dz, np.ndarray) else dz
        ws, nb = self.workspace(T, peqa.PEQA_OP_BWD_Z)
        peqa.linear_bwd_z(self.L, self.packed, self.s0, dsd, self.z0, dzd, X, dY, T, dX, dds, ddz, ws, nb)
        torch.cuda.synchronize()
        return dX, dds, ddz


def assert_scale_grad_close(g, gref, what="d_ds"):
    """The two bounds every scale (or zero-point) gradient is held to: relative L2 error at most 1e-3 (the stated
    tolerance), and, element by element, |g - ref| <= 1e-3 |ref| + 5e-5 rms(ref), so that a single wrong channel
    or group of small magnitude cannot hide under the norm.  Returns (relative L2 error, worst element's share of
    its bound)."""
    g = np.asarray(g, np.float64)
    gref = np.asarray(gref, np.float64)
    assert g.shape == gref.shape, (what, g.shape, gref.shape)
    nref = np.linalg.norm(gref)
    l2 = np.linalg.norm(g - gref) / nref if nref > 0 else float(np.abs(g).max())
    assert l2 <= 1e-3, "%s: relative L2 error %.3e" % (what, l2)
    bound = 1e-3 * np.abs(gref) + 5e-5 * nref / np.sqrt(gref.size)
    ratio = np.abs(g - gref) / np.maximum(bound, 1e-300)
    worst = float(ratio.max())
    assert worst <= 1.0, "%s: element %s off by %.3e (bound %.3e)" % (
        what, np.unravel_index(int(ratio.argmax()), ratio.shape), float(np.abs(g - gref).ravel()[ratio.argmax()]),
        float(bound.ravel()[ratio.argmax()]))
    return l2, worst


def bf16_dev_to_f64(t):
    from paper_2305_14152_amd import synth
    return synth.bf16_bits_to_f32(to_host(t).view(np.uint16)).astype(np.float64)
