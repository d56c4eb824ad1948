"""Thin ctypes binding over the C-ABI library (include/peqa.h), same names, argument
marshalling only.  PyTorch supplies device memory and the HIP stream; every step of the
computation runs inside libpeqa_hip.so.  There is no fallback: a missing library raises."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpeqa_hip.so")

PEQA_OK = 0
PEQA_ERR_NULL, PEQA_ERR_SHAPE, PEQA_ERR_BITS, PEQA_ERR_GROUP = 1, 2, 3, 4
PEQA_ERR_ALIGN, PEQA_ERR_WORKSPACE, PEQA_ERR_DEVICE, PEQA_ERR_PARAM = 5, 6, 7, 8
PEQA_OP_FWD, PEQA_OP_BWD, PEQA_OP_FWD_KEEP, PEQA_OP_BWD_KEPT, PEQA_OP_FWD_Z, PEQA_OP_BWD_Z = 0, 1, 2, 3, 4, 5
PEQA_OPT_GEMM_WAVES, PEQA_OPT_BWD_PAIR, PEQA_OPT_GROUPED_DDS = 0, 1, 2

EXPORTS = ["peqa_check_layout", "peqa_packed_words", "peqa_num_scales", "peqa_workspace_bytes",
           "peqa_status_string", "peqa_bit_location", "peqa_quantize", "peqa_linear_fwd",
           "peqa_linear_bwd", "peqa_scale_update", "peqa_trace_begin", "peqa_trace_end",
           "peqa_workspace_bytes_fused", "peqa_linear_fwd_fused", "peqa_linear_fwd_keep", "peqa_linear_bwd_kept",
           "peqa_linear_fwd_z", "peqa_linear_bwd_z", "peqa_quantize_search",
           "peqa_scale_update_multi", "peqa_device_info",
           "peqa_row_sums", "peqa_linear_fwd_fused_rs", "peqa_linear_bwd_rs",
           "peqa_set_option", "peqa_get_option", "peqa_linear_fwd_static",
           "peqa_block_workspace_bytes", "peqa_block_fwd", "peqa_block_bwd", "peqa_trace_select"]


class Layout(ctypes.Structure):
    _fields_ = [("n_out", ctypes.c_int32), ("k_in", ctypes.c_int32),
                ("bits", ctypes.c_int32), ("group_size", ctypes.c_int32)]

    @property
    def groups(self):
        return self.k_in // self.group_size if self.group_size else 1


class AdamW(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float), ("step", ctypes.c_int32)]


class PeqaError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s (status %d)" % (what, status_string(status), status))


_lib = None


def lib():
    """Loads libpeqa_hip.so; raises if it has not been built (python -m paper_2305_14152_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libpeqa_hip.so is missing: build it with __graft_entry__.build() "
                              "or `python paper_2305_14152_amd/build.py`; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        LP = ctypes.POINTER(Layout)
        L.peqa_check_layout.argtypes = [LP]
        L.peqa_check_layout.restype = i32
        L.peqa_packed_words.argtypes = [LP]
        L.peqa_packed_words.restype = sz
        L.peqa_num_scales.argtypes = [LP]
        L.peqa_num_scales.restype = sz
        L.peqa_workspace_bytes.argtypes = [LP, i32, i32]
        L.peqa_workspace_bytes.restype = sz
        L.peqa_status_string.argtypes = [i32]
        L.peqa_status_string.restype = ctypes.c_char_p
        L.peqa_bit_location.argtypes = [LP, i32, i32, i32, ctypes.POINTER(sz), ctypes.POINTER(i32)]
        L.peqa_bit_location.restype = i32
        L.peqa_quantize.argtypes = [LP, vp, vp, vp, vp, vp]
        L.peqa_quantize.restype = i32
        L.peqa_quantize_search.argtypes = [LP, vp, i32, ctypes.c_float, vp, vp, vp, vp]
        L.peqa_quantize_search.restype = i32
        L.peqa_linear_fwd.argtypes = [LP, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.peqa_linear_fwd.restype = i32
        L.peqa_linear_fwd_static.argtypes = [LP, vp, vp, vp, vp, vp, i32, vp, vp]
        L.peqa_linear_fwd_static.restype = i32
        L.peqa_linear_bwd.argtypes = [LP, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
        L.peqa_linear_bwd.restype = i32
        L.peqa_linear_fwd_keep.argtypes = [LP, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
        L.peqa_linear_fwd_keep.restype = i32
        L.peqa_linear_bwd_kept.argtypes = [LP, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
        L.peqa_linear_bwd_kept.restype = i32
        L.peqa_linear_fwd_z.argtypes = [LP, vp, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.peqa_linear_fwd_z.restype = i32
        L.peqa_linear_bwd_z.argtypes = [LP, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, sz, vp]
        L.peqa_linear_bwd_z.restype = i32
        L.peqa_scale_update.argtypes = [sz, vp, vp, vp, vp, vp, ctypes.POINTER(AdamW), vp]
        L.peqa_scale_update.restype = i32
        L.peqa_scale_update_multi.argtypes = [i32, vp, ctypes.POINTER(AdamW), vp]
        L.peqa_scale_update_multi.restype = i32
        L.peqa_row_sums.argtypes = [vp, i32, i32, vp, vp]
        L.peqa_row_sums.restype = i32
        L.peqa_linear_fwd_fused_rs.argtypes = [i32, vp, vp, vp, i32, vp, sz, vp]
        L.peqa_linear_fwd_fused_rs.restype = i32
        L.peqa_linear_bwd_rs.argtypes = [LP, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
        L.peqa_linear_bwd_rs.restype = i32
        L.peqa_workspace_bytes_fused.argtypes = [i32, vp, i32]
        L.peqa_workspace_bytes_fused.restype = sz
        L.peqa_linear_fwd_fused.argtypes = [i32, vp, vp, i32, vp, sz, vp]
        L.peqa_linear_fwd_fused.restype = i32
        L.peqa_set_option.argtypes = [i32, i32]
        L.peqa_set_option.restype = i32
        L.peqa_get_option.argtypes = [i32]
        L.peqa_get_option.restype = i32
        L.peqa_block_workspace_bytes.argtypes = [i32, vp, i32, i32]
        L.peqa_block_workspace_bytes.restype = sz
        L.peqa_block_fwd.argtypes = [i32, vp, i32, vp, sz, vp]
        L.peqa_block_fwd.restype = i32
        L.peqa_block_bwd.argtypes = [i32, vp, i32, vp, sz, vp]
        L.peqa_block_bwd.restype = i32
        L.peqa_trace_select.argtypes = [ctypes.c_char_p]
        L.peqa_trace_select.restype = i32
        L.peqa_trace_begin.argtypes = [i32]
        L.peqa_trace_begin.restype = i32
        L.peqa_trace_end.argtypes = [i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(i32),
                                     ctypes.POINTER(ctypes.c_float)]
        L.peqa_trace_end.restype = i32
        _lib = L
    return _lib


def status_string(status):
    return lib().peqa_status_string(int(status)).decode()


def _check(status, what):
    if status != PEQA_OK:
        raise PeqaError(status, what)


def _ptr(t):
    """Device (or raw integer) pointer of a torch tensor; None -> NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors must be contiguous"
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def layout(n_out, k_in, bits, group_size=0):
    return Layout(int(n_out), int(k_in), int(bits), int(group_size))


def check_layout(L):
    return int(lib().peqa_check_layout(ctypes.byref(L)))


def packed_words(L):
    return int(lib().peqa_packed_words(ctypes.byref(L)))


def num_scales(L):
    return int(lib().peqa_num_scales(ctypes.byref(L)))


def workspace_bytes(L, T, op):
    return int(lib().peqa_workspace_bytes(ctypes.byref(L), int(T), int(op)))


def bit_location(L, i, k, t):
    w, b = ctypes.c_size_t(), ctypes.c_int32()
    _check(lib().peqa_bit_location(ctypes.byref(L), i, k, t, ctypes.byref(w), ctypes.byref(b)), "peqa_bit_location")
    return int(w.value), int(b.value)


def quantize(L, W0, packed, s0, z0, stream=None):
    _check(lib().peqa_quantize(ctypes.byref(L), _ptr(W0), _ptr(packed), _ptr(s0), _ptr(z0), _stream(stream)),
           "peqa_quantize")


class UpdateItem(ctypes.Structure):
    _fields_ = [("n_scales", ctypes.c_size_t), ("ds", ctypes.c_void_p), ("d_ds", ctypes.c_void_p),
                ("m", ctypes.c_void_p), ("v", ctypes.c_void_p), ("s0", ctypes.c_void_p)]


def scale_update_multi(tensors, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, step=1, stream=None):
    """tensors: sequence of (n_scales, ds, d_ds, m, v, s0)."""
    arr = (UpdateItem * len(tensors))()
    for i, (n, ds, d_ds, m, v, s0) in enumerate(tensors):
        arr[i] = UpdateItem(int(n), _ptr(ds), _ptr(d_ds), _ptr(m), _ptr(v), _ptr(s0))
    opt = AdamW(lr, beta1, beta2, eps, weight_decay, int(step))
    _check(lib().peqa_scale_update_multi(len(tensors), ctypes.addressof(arr), ctypes.byref(opt), _stream(stream)),
           "peqa_scale_update_multi")


def device_info():
    """(compute units, peak engine clock in kHz) of the current device."""
    cus, khz = ctypes.c_int32(0), ctypes.c_int32(0)
    f = lib().peqa_device_info
    f.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
    f.restype = ctypes.c_int32
    _check(f(ctypes.byref(cus), ctypes.byref(khz)), "peqa_device_info")
    return cus.value, khz.value


def row_sums(X, T, K, rs, stream=None):
    _check(lib().peqa_row_sums(_ptr(X), int(T), int(K), _ptr(rs), _stream(stream)), "peqa_row_sums")


def linear_fwd_fused_rs(layers, X, rs, T, workspace, workspace_bytes_, stream=None):
    arr = _items(layers)
    _check(lib().peqa_linear_fwd_fused_rs(len(layers), ctypes.addressof(arr), _ptr(X), _ptr(rs), int(T),
                                          _ptr(workspace), int(workspace_bytes_), _stream(stream)),
           "peqa_linear_fwd_fused_rs")


def linear_bwd_rs(L, packed, s0, ds, z0, X, rs, dY, T, dX, d_ds, workspace, workspace_bytes_, stream=None):
    _check(lib().peqa_linear_bwd_rs(ctypes.byref(L), _ptr(packed), _ptr(s0), _ptr(ds), _ptr(z0), _ptr(X), _ptr(rs),
                                    _ptr(dY), int(T), _ptr(dX), _ptr(d_ds), _ptr(workspace), int(workspace_bytes_),
                                    _stream(stream)), "peqa_linear_bwd_rs")


def quantize_search(L, W0, n_ratios, min_ratio, packed, s0, z0, stream=None):
    _check(lib().peqa_quantize_search(ctypes.byref(L), _ptr(W0), int(n_ratios), float(min_ratio), _ptr(packed),
                                      _ptr(s0), _ptr(z0), _stream(stream)), "peqa_quantize_search")


def linear_fwd(L, packed, s0, ds, z0, X, T, Y, workspace, workspace_bytes_, stream=None):
    _check(lib().peqa_linear_fwd(ctypes.byref(L), _ptr(packed), _ptr(s0), _ptr(ds), _ptr(z0), _ptr(X), int(T),
                                 _ptr(Y), _ptr(workspace), int(workspace_bytes_), _stream(stream)),
           "peqa_linear_fwd")


STATIC_SCRATCH_BYTES = 16 << 20


def linear_fwd_static(L, packed, s0, ds, z0, X, T, Y, stream=None):
    _check(lib().peqa_linear_fwd_static(ctypes.byref(L), _ptr(packed), _ptr(s0), _ptr(ds), _ptr(z0), _ptr(X), int(T),
                                        _ptr(Y), _stream(stream)), "peqa_linear_fwd_static")


class FwdItem(ctypes.Structure):
    _fields_ = [("layout", Layout), ("packed", ctypes.c_void_p), ("s0", ctypes.c_void_p), ("ds", ctypes.c_void_p),
                ("z0", ctypes.c_void_p), ("Y", ctypes.c_void_p)]


def _items(layers):
    """layers: sequence of (L, packed, s0, ds, z0, Y)."""
    arr = (FwdItem * len(layers))()
    for i, (L, packed, s0, ds, z0, Y) in enumerate(layers):
        arr[i] = FwdItem(L, _ptr(packed), _ptr(s0), _ptr(ds), _ptr(z0), _ptr(Y))
    return arr


def workspace_bytes_fused(layers, T):
    arr = _items(layers)
    return int(lib().peqa_workspace_bytes_fused(len(layers), ctypes.addressof(arr), int(T)))


def linear_fwd_fused(layers, X, T, workspace, workspace_bytes_, stream=None):
    arr = _items(layers)
    _check(lib().peqa_linear_fwd_fused(len(layers), ctypes.addressof(arr), _ptr(X), int(T), _ptr(workspace),
                                       int(workspace_bytes_), _stream(stream)), "peqa_linear_fwd_fused")


def linear_bwd(L, packed, s0, ds, z0, X, dY, T, dX, d_ds, workspace, workspace_bytes_, stream=None):
    _check(lib().peqa_linear_bwd(ctypes.byref(L), _ptr(packed), _ptr(s0), _ptr(ds), _ptr(z0), _ptr(X), _ptr(dY),
                                 int(T), _ptr(dX), _ptr(d_ds), _ptr(workspace), int(workspace_bytes_),
                                 _stream(stream)), "peqa_linear_bwd")


def linear_fwd_keep(L, packed, s0, ds, z0, X, T, Y, P, workspace, workspace_bytes_, stream=None):
    _check(lib().peqa_linear_fwd_keep(ctypes.byref(L), _ptr(packed), _ptr(s0), _ptr(ds), _ptr(z0), _ptr(X), int(T),
                                      _ptr(Y), _ptr(P), _ptr(workspace), int(workspace_bytes_), _stream(stream)),
           "peqa_linear_fwd_keep")


def linear_bwd_kept(L, packed, s0, ds, z0, P, dY, T, dX, d_ds, workspace, workspace_bytes_, stream=None):
    _check(lib().peqa_linear_bwd_kept(ctypes.byref(L), _ptr(packed), _ptr(s0), _ptr(ds), _ptr(z0), _ptr(P), _ptr(dY),
                                      int(T), _ptr(dX), _ptr(d_ds), _ptr(workspace), int(workspace_bytes_),
                                      _stream(stream)), "peqa_linear_bwd_kept")


def linear_fwd_z(L, packed, s0, ds, z0, dz, X, T, Y, workspace, workspace_bytes_, stream=None):
    _check(lib().peqa_linear_fwd_z(ctypes.byref(L), _ptr(packed), _ptr(s0), _ptr(ds), _ptr(z0), _ptr(dz), _ptr(X),
                                   int(T), _ptr(Y), _ptr(workspace), int(workspace_bytes_), _stream(stream)),
           "peqa_linear_fwd_z")


def linear_bwd_z(L, packed, s0, ds, z0, dz, X, dY, T, dX, d_ds, d_dz, workspace, workspace_bytes_, stream=None):
    _check(lib().peqa_linear_bwd_z(ctypes.byref(L), _ptr(packed), _ptr(s0), _ptr(ds), _ptr(z0), _ptr(dz), _ptr(X),
                                   _ptr(dY), int(T), _ptr(dX), _ptr(d_ds), _ptr(d_dz), _ptr(workspace),
                                   int(workspace_bytes_), _stream(stream)), "peqa_linear_bwd_z")


def scale_update(n_scales, ds, d_ds, m, v, s0, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, step=1,
                 stream=None):
    opt = AdamW(lr, beta1, beta2, eps, weight_decay, int(step))
    _check(lib().peqa_scale_update(int(n_scales), _ptr(ds), _ptr(d_ds), _ptr(m), _ptr(v), _ptr(s0),
                                   ctypes.byref(opt), _stream(stream)), "peqa_scale_update")


class BlockItem(ctypes.Structure):
    _fields_ = [("layout", Layout), ("packed", ctypes.c_void_p), ("s0", ctypes.c_void_p), ("ds", ctypes.c_void_p),
                ("z0", ctypes.c_void_p), ("X", ctypes.c_void_p), ("Y", ctypes.c_void_p), ("dY", ctypes.c_void_p),
                ("dX", ctypes.c_void_p), ("d_ds", ctypes.c_void_p), ("row_sums", ctypes.c_void_p)]


def block_items(layers):
    """layers: sequence of dicts with keys L, packed, s0, z0 and optionally ds, X, Y, dY, dX, d_ds, row_sums."""
    arr = (BlockItem * len(layers))()
    for i, d in enumerate(layers):
        arr[i] = BlockItem(d["L"], _ptr(d["packed"]), _ptr(d["s0"]), _ptr(d.get("ds")), _ptr(d["z0"]), _ptr(d.get("X")),
                           _ptr(d.get("Y")), _ptr(d.get("dY")), _ptr(d.get("dX")), _ptr(d.get("d_ds")),
                           _ptr(d.get("row_sums")))
    return arr


def block_workspace_bytes(items, T, op):
    return int(lib().peqa_block_workspace_bytes(len(items), ctypes.addressof(items), int(T), int(op)))


def block_fwd(items, T, workspace, workspace_bytes_, stream=None):
    _check(lib().peqa_block_fwd(len(items), ctypes.addressof(items), int(T), _ptr(workspace), int(workspace_bytes_),
                                _stream(stream)), "peqa_block_fwd")


def block_bwd(items, T, workspace, workspace_bytes_, stream=None):
    _check(lib().peqa_block_bwd(len(items), ctypes.addressof(items), int(T), _ptr(workspace), int(workspace_bytes_),
                                _stream(stream)), "peqa_block_bwd")


def set_option(option, value):
    _check(lib().peqa_set_option(int(option), int(value)), "peqa_set_option")


def get_option(option):
    return int(lib().peqa_get_option(int(option)))


def trace_begin(max_launches, prefix=None):
    """Brackets the library's launches with HIP events until trace_end(); `prefix` restricts it to kernels whose
    name starts with it."""
    _check(lib().peqa_trace_select(prefix.encode() if prefix else None), "peqa_trace_select")
    _check(lib().peqa_trace_begin(int(max_launches)), "peqa_trace_begin")


def trace_end(max_kernels=32):
    names = (ctypes.c_char_p * max_kernels)()
    launches = (ctypes.c_int32 * max_kernels)()
    total_ms = (ctypes.c_float * max_kernels)()
    n = lib().peqa_trace_end(max_kernels, names, launches, total_ms)
    return {names[i].decode(): (int(launches[i]), float(total_ms[i])) for i in range(n)}
