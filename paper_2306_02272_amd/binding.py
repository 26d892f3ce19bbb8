"""ctypes binding of include/owq.h: argument marshalling only.

Every function has the name and meaning of the C entry point.  Arrays cross
the boundary as raw pointers: numpy arrays for HOST arguments, integer device
addresses (torch `tensor.data_ptr()`) for DEVICE arguments.  There is no
fallback: if libowq.so is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libowq.so")

OWQ_OK = 0
STATUS_NAMES = ["OWQ_OK", "OWQ_ERR_NULL", "OWQ_ERR_SHAPE", "OWQ_ERR_BITS", "OWQ_ERR_GROUP",
                "OWQ_ERR_CODE_RANGE", "OWQ_ERR_INDEX", "OWQ_ERR_BUFFER", "OWQ_ERR_BATCH",
                "OWQ_ERR_HANDLE", "OWQ_ERR_HIP", "OWQ_ERR_UNSUPPORTED", "OWQ_ERR_LAYOUT", "OWQ_ERR_SCRATCH"]
(OWQ_ERR_NULL, OWQ_ERR_SHAPE, OWQ_ERR_BITS, OWQ_ERR_GROUP, OWQ_ERR_CODE_RANGE, OWQ_ERR_INDEX,
 OWQ_ERR_BUFFER, OWQ_ERR_BATCH, OWQ_ERR_HANDLE, OWQ_ERR_HIP, OWQ_ERR_UNSUPPORTED,
 OWQ_ERR_LAYOUT, OWQ_ERR_SCRATCH) = range(1, 14)
OWQ_STATIC_SCRATCH_BYTES = 32 << 20
OWQ_LAYOUT_GEMV, OWQ_LAYOUT_TILE, OWQ_LAYOUT_COMPACT = 0, 1, 2

# every symbol include/owq.h declares
EXPORTS = ["owq_geometry", "owq_packed_bytes", "owq_pack_host", "owq_unpack_codes", "owq_pack_layer",
           "owq_open_packed", "owq_linear", "owq_free_layer", "owq_layer_info", "owq_export_packed", "owq_set_launch",
           "owq_update_weak", "owq_weak_set_bytes", "owq_pack_weak_set", "owq_linear_multi", "owq_search_config",
           "owq_backward_workspace_bytes", "owq_linear_backward", "owq_probe_read", "owq_probe_read_write", "owq_probe_empty", "owq_probe_alu", "owq_probe_mfma", "owq_workspace_bytes", "owq_linear_ws", "owq_linear_static",
           "owq_status_str"]


class OwqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__(f"{where}: {name}")


class LayerDesc(C.Structure):
    _fields_ = [("d_out", C.c_int32), ("d_in", C.c_int32), ("bits", C.c_int32),
                ("group_size", C.c_int32), ("k", C.c_int32),
                ("codes", C.c_void_p), ("scale", C.c_void_p), ("zero", C.c_void_p),
                ("weak_idx", C.c_void_p), ("weak_w", C.c_void_p), ("layout", C.c_int32)]


class SearchDesc(C.Structure):
    _fields_ = [("d_out", C.c_int32), ("d_in", C.c_int32), ("bits", C.c_int32), ("group_size", C.c_int32),
                ("k", C.c_int32), ("n_lo", C.c_int32), ("n_hi", C.c_int32), ("shrink", C.c_float)]


class LayerInfo(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("format_version", "d_out", "d_in", "bits", "group_size", "k", "nblk", "cw", "r",
                 "nact", "nslab", "n_rt", "d_out_pad", "chunks", "n_groups", "kp")] + \
               [(n, C.c_uint64) for n in
                ("off_codes", "off_sz", "off_weak_w", "off_weak_idx", "total_bytes")] + \
               [("layout", C.c_int32), ("nbp", C.c_int32), ("off_wmask", C.c_uint64),
                ("off_scratch", C.c_uint64)] + \
               [(n, C.c_int32) for n in
                ("row_tiles_per_wg", "row_splits", "waves_per_wg", "prefetch_depth", "workgroups",
                 "lds_bytes", "last_hip_error", "reserved")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


_lib = None


def lib():
    """The loaded shared library (raises if it was never built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: run `python -m paper_2306_02272_amd.build` "
                              "(or __graft_entry__.build()) first")
        L = C.CDLL(LIB_PATH)
        P, I32, SZ = C.c_void_p, C.c_int32, C.c_size_t
        L.owq_geometry.argtypes = [C.POINTER(LayerDesc), C.POINTER(LayerInfo)]
        L.owq_packed_bytes.argtypes = [C.POINTER(LayerDesc), C.POINTER(SZ)]
        L.owq_pack_host.argtypes = [C.POINTER(LayerDesc), P, SZ]
        L.owq_unpack_codes.argtypes = [P, C.POINTER(LayerInfo), P]
        L.owq_pack_layer.argtypes = [C.POINTER(LayerDesc), P, SZ, P, C.POINTER(P)]
        L.owq_open_packed.argtypes = [C.POINTER(LayerDesc), P, SZ, C.POINTER(P)]
        L.owq_linear.argtypes = [P, P, P, I32, P]
        L.owq_free_layer.argtypes = [P]
        L.owq_layer_info.argtypes = [P, C.POINTER(LayerInfo)]
        L.owq_export_packed.argtypes = [P, P, SZ]
        L.owq_set_launch.argtypes = [P, I32, I32, I32, I32]
        L.owq_update_weak.argtypes = [P, P, P]
        L.owq_weak_set_bytes.argtypes = [P, C.POINTER(SZ)]
        L.owq_pack_weak_set.argtypes = [P, P, P, SZ, P]
        L.owq_linear_multi.argtypes = [P, P, I32, P, P, P, I32, P]
        L.owq_search_config.argtypes = [C.POINTER(SearchDesc), P, P, P, P, P, P, P, P]
        L.owq_backward_workspace_bytes.argtypes = [P, I32, C.POINTER(SZ)]
        L.owq_linear_backward.argtypes = [P, P, P, P, P, I32, P, SZ, P]
        L.owq_workspace_bytes.argtypes = [P, C.POINTER(SZ)]
        L.owq_linear_ws.argtypes = [P, P, P, I32, P, SZ, P]
        L.owq_linear_static.argtypes = [P, P, P, I32, P]
        L.owq_probe_read.argtypes = [P, SZ, I32, P]
        L.owq_probe_read_write.argtypes = [P, SZ, I32, P, SZ, P]
        L.owq_probe_empty.argtypes = [P]
        L.owq_probe_alu.argtypes = [P, C.c_int32, C.c_int32, P]
        L.owq_probe_mfma.argtypes = [P, C.c_int32, C.c_int32, P]
        for n in EXPORTS:
            getattr(L, n).restype = C.c_int
        L.owq_status_str.argtypes = [C.c_int]
        L.owq_status_str.restype = C.c_char_p
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != OWQ_OK:
        raise OwqError(status, where)


def _ptr(a):
    return None if a is None else a.ctypes.data


def make_desc(d_out, d_in, bits, group_size, k, codes=None, scale=None, zero=None,
              weak_idx=None, weak_w=None, layout=0):
    """LayerDesc over numpy arrays (kept alive on the returned object)."""
    def prep(a, dt):
        if a is None:
            return None
        a = np.ascontiguousarray(a)
        if dt is np.uint16 and a.dtype == np.float16:
            a = a.view(np.uint16)
        assert a.dtype == dt, (a.dtype, dt)
        return a
    keep = [prep(codes, np.uint8), prep(scale, np.uint16), prep(zero, np.uint16),
            prep(weak_idx, np.int32), prep(weak_w, np.uint16)]
    d = LayerDesc(d_out, d_in, bits, group_size, k, *[_ptr(a) for a in keep], layout)
    d._keep = keep
    return d


def desc_from_layer(layer, layout=0):
    """LayerDesc for a synth.Layer-like object (numpy fields)."""
    return make_desc(layer.d_out, layer.d_in, layer.bits, layer.group_size, layer.k,
                     layer.codes, layer.scale, layer.zero, layer.weak_idx, layer.weak_w, layout)


def owq_geometry(desc) -> LayerInfo:
    info = LayerInfo()
    _check(lib().owq_geometry(C.byref(desc), C.byref(info)), "owq_geometry")
    return info


def owq_packed_bytes(desc) -> int:
    n = C.c_size_t(0)
    _check(lib().owq_packed_bytes(C.byref(desc), C.byref(n)), "owq_packed_bytes")
    return int(n.value)


def owq_pack_host(desc) -> np.ndarray:
    n = owq_packed_bytes(desc)
    out = np.empty(n, dtype=np.uint8)
    _check(lib().owq_pack_host(C.byref(desc), out.ctypes.data, n), "owq_pack_host")
    return out


def owq_unpack_codes(blob: np.ndarray, info: LayerInfo) -> np.ndarray:
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    codes = np.empty((info.d_out, info.d_in), dtype=np.uint8)
    _check(lib().owq_unpack_codes(blob.ctypes.data, C.byref(info), codes.ctypes.data), "owq_unpack_codes")
    return codes


def owq_pack_layer(desc, dev_ptr: int, dev_bytes: int, stream: int = 0) -> int:
    h = C.c_void_p(None)
    _check(lib().owq_pack_layer(C.byref(desc), C.c_void_p(dev_ptr), dev_bytes,
                                C.c_void_p(stream), C.byref(h)), "owq_pack_layer")
    return h.value


def owq_open_packed(desc, dev_ptr: int, dev_bytes: int) -> int:
    h = C.c_void_p(None)
    _check(lib().owq_open_packed(C.byref(desc), C.c_void_p(dev_ptr), dev_bytes, C.byref(h)),
           "owq_open_packed")
    return h.value


def owq_linear(handle: int, x_ptr: int, y_ptr: int, batch: int, stream: int = 0) -> None:
    _check(lib().owq_linear(C.c_void_p(handle), C.c_void_p(x_ptr), C.c_void_p(y_ptr), batch,
                            C.c_void_p(stream)), "owq_linear")


def owq_workspace_bytes(handle: int) -> int:
    n = C.c_size_t(0)
    _check(lib().owq_workspace_bytes(C.c_void_p(handle), C.byref(n)), "owq_workspace_bytes")
    return int(n.value)


def owq_linear_ws(handle: int, x_ptr: int, y_ptr: int, batch: int, workspace_ptr: int, workspace_bytes: int,
                  stream: int = 0) -> None:
    _check(lib().owq_linear_ws(C.c_void_p(handle), C.c_void_p(x_ptr), C.c_void_p(y_ptr), batch,
                               C.c_void_p(workspace_ptr), workspace_bytes, C.c_void_p(stream)), "owq_linear_ws")


def owq_linear_static(handle: int, x_ptr: int, y_ptr: int, batch: int, stream: int = 0) -> None:
    _check(lib().owq_linear_static(C.c_void_p(handle), C.c_void_p(x_ptr), C.c_void_p(y_ptr), batch,
                                   C.c_void_p(stream)), "owq_linear_static")


def owq_probe_read(dev_ptr: int, nbytes: int, workgroups: int, stream: int = 0) -> None:
    _check(lib().owq_probe_read(C.c_void_p(dev_ptr), nbytes, workgroups, C.c_void_p(stream)), "owq_probe_read")


def owq_probe_read_write(dev_ptr: int, nbytes: int, workgroups: int, out_ptr: int, out_bytes: int, stream: int = 0) -> None:
    _check(lib().owq_probe_read_write(C.c_void_p(dev_ptr), nbytes, workgroups, C.c_void_p(out_ptr), out_bytes,
                                      C.c_void_p(stream)), "owq_probe_read_write")


def owq_probe_empty(stream: int = 0) -> None:
    _check(lib().owq_probe_empty(C.c_void_p(stream)), "owq_probe_empty")


def owq_probe_mfma(dev_word: int, workgroups: int, trips: int, stream: int = 0) -> None:
    _check(lib().owq_probe_mfma(C.c_void_p(dev_word), workgroups, trips, C.c_void_p(stream)), "owq_probe_mfma")


def owq_probe_alu(dev_word: int, workgroups: int, trips: int, stream: int = 0) -> None:
    _check(lib().owq_probe_alu(C.c_void_p(dev_word), workgroups, trips, C.c_void_p(stream)), "owq_probe_alu")


def owq_free_layer(handle: int) -> None:
    _check(lib().owq_free_layer(C.c_void_p(handle)), "owq_free_layer")


def owq_layer_info(handle: int) -> LayerInfo:
    info = LayerInfo()
    _check(lib().owq_layer_info(C.c_void_p(handle), C.byref(info)), "owq_layer_info")
    return info


def owq_export_packed(handle: int) -> np.ndarray:
    info = owq_layer_info(handle)
    out = np.empty(info.total_bytes, dtype=np.uint8)
    _check(lib().owq_export_packed(C.c_void_p(handle), out.ctypes.data, out.size), "owq_export_packed")
    return out


def owq_set_launch(handle: int, row_tiles_per_wg=0, row_splits=0, waves_per_wg=0, prefetch_depth=0):
    _check(lib().owq_set_launch(C.c_void_p(handle), row_tiles_per_wg, row_splits, waves_per_wg,
                                prefetch_depth), "owq_set_launch")


def _weak_host(weak_w):
    a = np.ascontiguousarray(weak_w)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def owq_update_weak(handle: int, weak_w, stream: int = 0) -> None:
    a = _weak_host(weak_w)
    _check(lib().owq_update_weak(C.c_void_p(handle), a.ctypes.data if a.size else None, C.c_void_p(stream)),
           "owq_update_weak")


def owq_weak_set_bytes(handle: int) -> int:
    n = C.c_size_t(0)
    _check(lib().owq_weak_set_bytes(C.c_void_p(handle), C.byref(n)), "owq_weak_set_bytes")
    return int(n.value)


def owq_pack_weak_set(handle: int, weak_w, dev_ptr: int, dev_bytes: int, stream: int = 0) -> None:
    a = _weak_host(weak_w)
    _check(lib().owq_pack_weak_set(C.c_void_p(handle), a.ctypes.data if a.size else None, C.c_void_p(dev_ptr),
                                   dev_bytes, C.c_void_p(stream)), "owq_pack_weak_set")


def owq_linear_multi(handle: int, weak_sets_ptr: int, n_sets: int, task_id_ptr: int, x_ptr: int, y_ptr: int,
                     batch: int, stream: int = 0) -> None:
    _check(lib().owq_linear_multi(C.c_void_p(handle), C.c_void_p(weak_sets_ptr), n_sets, C.c_void_p(task_id_ptr),
                                  C.c_void_p(x_ptr), C.c_void_p(y_ptr), batch, C.c_void_p(stream)),
           "owq_linear_multi")


def owq_search_config(desc: SearchDesc, w_ptr: int, weak_idx_ptr: int, scale_ptr: int, zero_ptr: int,
                      codes_ptr: int, err_ptr: int = 0, choice_ptr: int = 0, stream: int = 0) -> None:
    """Every pointer is a DEVICE address (0 = NULL where the header allows it)."""
    _check(lib().owq_search_config(C.byref(desc), C.c_void_p(w_ptr), C.c_void_p(weak_idx_ptr), C.c_void_p(scale_ptr),
                                   C.c_void_p(zero_ptr), C.c_void_p(codes_ptr), C.c_void_p(err_ptr),
                                   C.c_void_p(choice_ptr), C.c_void_p(stream)), "owq_search_config")


def search_config(w, weak_idx, bits, group_size, n_lo, n_hi, shrink, want_err=True):
    """owq_search_config on CUDA tensors: w fp16 [d_out, d_in], weak_idx int32 [k] (or None).
    Allocates the outputs with torch and returns (scale, zero, codes, err, choice) on the GPU."""
    import torch
    assert w.dtype == torch.float16 and w.is_cuda and w.is_contiguous() and w.dim() == 2
    d_out, d_in = w.shape
    k = 0 if weak_idx is None else int(weak_idx.numel())
    if k:
        assert weak_idx.dtype == torch.int32 and weak_idx.is_cuda and weak_idx.is_contiguous()
    n_g = 1 if group_size == 0 or group_size >= d_in else -(-d_in // group_size)
    dev = w.device
    scale = torch.empty((d_out, n_g), dtype=torch.float16, device=dev)
    zero = torch.empty((d_out, n_g), dtype=torch.float16, device=dev)
    codes = torch.empty((d_out, d_in), dtype=torch.uint8, device=dev)
    err = torch.empty((d_out, n_g), dtype=torch.float32, device=dev) if want_err else None
    choice = torch.empty((d_out, n_g), dtype=torch.int32, device=dev) if want_err else None
    desc = SearchDesc(d_out, d_in, bits, group_size, k, n_lo, n_hi, shrink)
    owq_search_config(desc, w.data_ptr(), weak_idx.data_ptr() if k else 0, scale.data_ptr(), zero.data_ptr(),
                      codes.data_ptr(), err.data_ptr() if want_err else 0, choice.data_ptr() if want_err else 0,
                      torch.cuda.current_stream().cuda_stream)
    return scale, zero, codes, err, choice


def owq_backward_workspace_bytes(handle: int, batch: int) -> int:
    n = C.c_size_t(0)
    _check(lib().owq_backward_workspace_bytes(C.c_void_p(handle), batch, C.byref(n)), "owq_backward_workspace_bytes")
    return int(n.value)


def owq_linear_backward(handle: int, dy_ptr: int, x_ptr: int, dx_ptr: int, dww_ptr: int, batch: int,
                        workspace_ptr: int, workspace_bytes: int, stream: int = 0) -> None:
    """Every pointer is a DEVICE address (0 = NULL where the header allows it)."""
    _check(lib().owq_linear_backward(C.c_void_p(handle), C.c_void_p(dy_ptr), C.c_void_p(x_ptr), C.c_void_p(dx_ptr),
                                     C.c_void_p(dww_ptr), batch, C.c_void_p(workspace_ptr), workspace_bytes,
                                     C.c_void_p(stream)), "owq_linear_backward")


def owq_status_str(status: int) -> str:
    return lib().owq_status_str(status).decode()


class OwqLinear:
    """A packed layer resident on the current GPU (torch owns the memory, nothing else)."""

    def __init__(self, layer, device="cuda", packed=None, layout=0):
        """Pack `layer` onto the GPU; with `packed` (a uint8 CUDA tensor holding a blob of the
        same shape) only a handle is opened over a private copy of it."""
        import torch
        self.torch = torch
        self.desc = desc_from_layer(layer, layout)
        nbytes = owq_packed_bytes(self.desc)
        if packed is None:
            self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
            assert self.buf.data_ptr() % 256 == 0
            self.handle = owq_pack_layer(self.desc, self.buf.data_ptr(), nbytes,
                                         torch.cuda.current_stream().cuda_stream)
        else:
            assert packed.numel() == nbytes and packed.dtype == torch.uint8 and packed.is_cuda
            self.buf = packed.clone()
            assert self.buf.data_ptr() % 256 == 0
            self.handle = owq_open_packed(self.desc, self.buf.data_ptr(), nbytes)
        self.d_in, self.d_out = layer.d_in, layer.d_out

    def info(self) -> LayerInfo:
        return owq_layer_info(self.handle)

    def __call__(self, x, out=None):
        torch = self.torch
        assert x.dtype == torch.float16 and x.is_cuda and x.is_contiguous() and x.shape[-1] == self.d_in
        batch = x.numel() // self.d_in
        if out is None:
            out = torch.empty((batch, self.d_out), dtype=torch.float16, device=x.device)
        owq_linear(self.handle, x.data_ptr(), out.data_ptr(), batch,
                   torch.cuda.current_stream().cuda_stream)
        return out

    def add_weak_sets(self, sets):
        """Upload further sets of weak columns ([d_out, k] fp16 each); returns (pointer table, buffers)."""
        torch = self.torch
        nbytes = max(16, owq_weak_set_bytes(self.handle))
        bufs = []
        for wset in sets:
            b = torch.empty(nbytes, dtype=torch.uint8, device=self.buf.device)
            owq_pack_weak_set(self.handle, wset, b.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream)
            bufs.append(b)
        table = torch.tensor([b.data_ptr() for b in bufs], dtype=torch.int64, device=self.buf.device)
        return table, bufs

    def multi(self, x, table, task_id, out=None):
        """owq_linear_multi: task_id an int32 CUDA tensor [batch], table from add_weak_sets."""
        torch = self.torch
        assert x.dtype == torch.float16 and x.is_cuda and x.is_contiguous() and x.shape[-1] == self.d_in
        batch = x.numel() // self.d_in
        assert task_id.dtype == torch.int32 and task_id.is_cuda and task_id.numel() == batch
        if out is None:
            out = torch.empty((batch, self.d_out), dtype=torch.float16, device=x.device)
        owq_linear_multi(self.handle, table.data_ptr(), int(table.numel()), task_id.data_ptr(), x.data_ptr(),
                         out.data_ptr(), batch, torch.cuda.current_stream().cuda_stream)
        return out

    def backward(self, dy, x=None, want_dx=True, want_dww=True, workspace=None):
        """owq_linear_backward on CUDA tensors; returns (dx fp16 [batch, d_in] or None, dww fp32 [d_out, k] or None)."""
        torch = self.torch
        assert dy.dtype == torch.float16 and dy.is_cuda and dy.is_contiguous() and dy.shape[-1] == self.d_out
        batch = dy.numel() // self.d_out
        k = self.desc.k
        dx = torch.empty((batch, self.d_in), dtype=torch.float16, device=dy.device) if want_dx else None
        dww = torch.empty((self.d_out, k), dtype=torch.float32, device=dy.device) if want_dww else None
        if want_dww and k > 0:
            assert x is not None and x.dtype == torch.float16 and x.is_contiguous() and x.numel() == batch * self.d_in
        if workspace is None:
            workspace = torch.empty(owq_backward_workspace_bytes(self.handle, batch), dtype=torch.uint8, device=dy.device)
        owq_linear_backward(self.handle, dy.data_ptr(), x.data_ptr() if x is not None else 0,
                            dx.data_ptr() if want_dx else 0, dww.data_ptr() if (want_dww and k > 0) else 0, batch,
                            workspace.data_ptr() if workspace is not None else 0,
                            int(workspace.numel()) if workspace is not None else 0,
                            torch.cuda.current_stream().cuda_stream)
        return dx, dww

    def close(self):
        if self.handle:
            owq_free_layer(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
