"""Thin ctypes binding of libvarco.so: argument marshalling only. Every step of the hot path runs in the
library's HIP kernels; torch tensors serve as device memory and torch streams as hipStream_t handles.

The library must have been built (python -m paper_2406_17611_amd.build, or __graft_entry__.build());
loading fails loudly otherwise - there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvarco.so")

OK, ERR_INVALID_ARG, ERR_SHAPE, ERR_STATE, ERR_UNSUPPORTED, ERR_HIP = range(6)
CONV_GCN, CONV_SAGE = 0, 1
ACT_IDENTITY, ACT_RELU = 0, 1
ORDER_AGGREGATE_FIRST, ORDER_TRANSFORM_FIRST = 0, 1
F32 = 0
BF16 = 1
MAX_LAYERS = 16

EXPORTS = [
    "varco_partition_build", "varco_partition_view", "varco_partition_free",
    "varco_create", "varco_destroy", "varco_register_partition", "varco_prepare", "varco_last_error",
    "varco_begin_step", "varco_set_ratio", "varco_set_matmul_terms", "varco_set_layer_order", "varco_get_keep",
    "varco_compress", "varco_decompress", "varco_layer_fwd", "varco_layer_bwd",
    "varco_accumulate_returned", "varco_get_stats", "varco_reset_stats", "varco_profile_enable", "varco_profile_read",
    "varco_calibration_copy", "varco_sum_gradients", "varco_softmax_xent", "varco_sgd_step", "varco_schedule_ratio",
    "varco_step_table_enable", "varco_set_step", "varco_advance_step",
    "varco_aggregate_fwd", "varco_aggregate_bwd", "varco_transform_fwd", "varco_transform_bwd_weight",
    "varco_transform_bwd_input", "varco_transform_bwd_weight_static",
]
KERNEL_CLASSES = ["compress", "decompress", "agg_fwd", "gemm_fwd", "gemm_wgrad", "gemm_dgrad", "agg_bwd_local",
                  "agg_bwd_halo", "reduce", "agg_bwd_halo_sum"]


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_partitions", C.c_int32), ("conv", C.c_int32), ("dtype", C.c_int32),
                ("mask_key", C.c_uint64), ("widths", C.POINTER(C.c_int32)), ("act", C.POINTER(C.c_int32))]


_DESC_ARRAYS = [("rowptr", np.int32), ("colidx", np.int32), ("vals", np.float32), ("t_rowptr", np.int32),
                ("t_colidx", np.int32), ("t_vals", np.float32), ("local_gid", np.int32), ("halo_gid", np.int32),
                ("halo_owner_ptr", np.int32), ("boundary_rows", np.int32), ("halo_src_row", np.int32),
                ("halo_zrow", np.int32), ("ret_ptr", np.int32), ("ret_src", np.int32)]


class PartitionDesc(C.Structure):
    _fields_ = ([("n_local", C.c_int32), ("n_halo", C.c_int32), ("n_boundary", C.c_int32),
                 ("z_row_offset", C.c_int32), ("nnz", C.c_int64), ("halo_row_offset", C.c_int32),
                 ("n_returned", C.c_int32)] + [(name, C.c_void_p) for name, _ in _DESC_ARRAYS])


class Stats(C.Structure):
    _fields_ = [("fwd_elems", C.c_int64 * MAX_LAYERS), ("bwd_elems", C.c_int64 * MAX_LAYERS),
                ("full_fwd_elems", C.c_int64 * MAX_LAYERS), ("full_bwd_elems", C.c_int64 * MAX_LAYERS),
                ("bytes_per_elem", C.c_int32)]


class Profile(C.Structure):
    _fields_ = [("launches", C.c_int64 * 10), ("ms", C.c_double * 10), ("bytes", C.c_double * 10),
                ("flops", C.c_double * 10), ("stream_bytes", C.c_double * 10)]


class VarcoError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"varco status {code}: {text}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2406_17611_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u32, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64
        L.varco_partition_build.argtypes = [i32, vp, vp, vp, vp, i32, C.POINTER(vp)]
        L.varco_partition_view.argtypes = [vp, i32, C.POINTER(PartitionDesc)]
        L.varco_partition_free.argtypes = [vp]
        L.varco_partition_free.restype = None
        L.varco_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
        L.varco_destroy.argtypes = [vp]
        L.varco_register_partition.argtypes = [vp, i32, C.POINTER(PartitionDesc)]
        L.varco_prepare.argtypes = [vp, vp]
        L.varco_last_error.argtypes = [vp]
        L.varco_last_error.restype = C.c_char_p
        L.varco_begin_step.argtypes = [vp, u64]
        L.varco_set_matmul_terms.argtypes = [vp, C.c_int32]
        L.varco_set_layer_order.argtypes = [vp, i32, i32]
        L.varco_set_ratio.argtypes = [vp, i32, u32, u32]
        L.varco_get_keep.argtypes = [vp, i32, C.POINTER(i32)]
        L.varco_compress.argtypes = [vp, i32, vp, vp, i64, vp, i64, vp, vp]
        L.varco_decompress.argtypes = [vp, i32, vp, vp, i64, vp, vp, i64, i32, vp]
        L.varco_layer_fwd.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.varco_layer_bwd.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.varco_accumulate_returned.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp]
        L.varco_get_stats.argtypes = [vp, C.POINTER(Stats)]
        L.varco_reset_stats.argtypes = [vp]
        L.varco_calibration_copy.argtypes = [vp, vp, i64, vp]
        L.varco_sum_gradients.argtypes = [vp, vp, i64, vp]
        L.varco_softmax_xent.argtypes = [vp, vp, i64, vp, i64, i32, C.c_float, vp, i64, vp, vp, vp, vp]
        L.varco_sgd_step.argtypes = [vp, vp, i64, C.c_float, vp]
        L.varco_schedule_ratio.argtypes = [i32, i64, i64, C.c_uint32, C.c_uint32, C.c_uint32, C.POINTER(C.c_uint32),
                                           C.POINTER(C.c_uint32)]
        L.varco_step_table_enable.argtypes = [vp, vp]
        L.varco_set_step.argtypes = [vp, u64, vp]
        L.varco_advance_step.argtypes = [vp, vp]
        L.varco_aggregate_fwd.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.varco_aggregate_bwd.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.varco_transform_fwd.argtypes = [vp, i32, i64, vp, vp, vp, i32, i32, vp]
        L.varco_transform_bwd_weight.argtypes = [vp, i32, i64, vp, vp, vp, vp, vp]
        L.varco_transform_bwd_input.argtypes = [vp, i32, i64, vp, vp, vp, vp, i32, vp]
        L.varco_transform_bwd_weight_static.argtypes = [vp, i32, i64, vp, vp, vp, vp, vp]
        L.varco_profile_enable.argtypes = [vp, i32]
        L.varco_profile_read.argtypes = [vp, C.POINTER(Profile), i32]
        for name in EXPORTS:
            if name not in ("varco_partition_free", "varco_last_error"):
                getattr(L, name).restype = i32
        _lib = L
    return _lib


def _check(code: int, ctx=None):
    if code != OK:
        text = lib().varco_last_error(ctx)
        raise VarcoError(code, text.decode() if text else "")


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array, None -> NULL."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else stream


def calibration_copy(dst, src, stream=None):
    """Copies the bytes of tensor `src` into `dst` with the library's plain copy kernel."""
    _check(lib().varco_calibration_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream(stream)))


SCHED_LINEAR, SCHED_FIXED_INCREMENT, SCHED_EXPONENTIAL = 0, 1, 2


def tap(layer: int, hop: int) -> int:
    """Address of hop `hop` of a K-tap layer (VARCO_TAP of the header)."""
    return layer + MAX_LAYERS * hop


def schedule_ratio(kind: int, step: int, n_steps: int, c_max: int, c_min: int, param: int):
    """(num, den) of the compression ratio at iteration `step` (host only)."""
    num, den = C.c_uint32(), C.c_uint32()
    _check(lib().varco_schedule_ratio(kind, step, n_steps, c_max, c_min, param, C.byref(num), C.byref(den)))
    return num.value, den.value


def sgd_step(w, dw, lr: float, stream=None):
    """w -= lr * dw (fp32 device tensors of equal size)."""
    assert w.numel() == dw.numel() and w.dtype == dw.dtype
    _check(lib().varco_sgd_step(_ptr(w), _ptr(dw), w.numel(), lr, _stream(stream)))


def sum_gradients(dst, src, stream=None):
    """dst += src (fp32 device tensors of equal size)."""
    assert dst.numel() == src.numel() and dst.dtype == src.dtype
    _check(lib().varco_sum_gradients(_ptr(dst), _ptr(src), dst.numel(), _stream(stream)))


# ---------------------------------------------------------------------------------------------------------
# host-side partition builder
# ---------------------------------------------------------------------------------------------------------

class HostPartition:
    """numpy copies of one partition's index structures, as built by varco_partition_build."""

    def __init__(self, desc: PartitionDesc):
        self.n_local, self.n_halo, self.n_boundary = desc.n_local, desc.n_halo, desc.n_boundary
        self.z_row_offset, self.nnz = desc.z_row_offset, desc.nnz
        self.halo_row_offset, self.n_returned = desc.halo_row_offset, desc.n_returned
        sizes = {"rowptr": self.n_local + 1, "colidx": self.nnz, "vals": self.nnz,
                 "t_rowptr": self.n_local + self.n_halo + 1, "t_colidx": self.nnz, "t_vals": self.nnz,
                 "local_gid": self.n_local, "halo_gid": self.n_halo, "halo_owner_ptr": None,
                 "boundary_rows": self.n_boundary, "halo_src_row": self.n_halo, "halo_zrow": self.n_halo,
                 "ret_ptr": self.n_boundary + 1, "ret_src": self.n_returned}
        self._sizes = sizes

    def _fill(self, desc, n_parts):
        self._sizes["halo_owner_ptr"] = n_parts + 1
        for name, dt in _DESC_ARRAYS:
            n = self._sizes[name]
            addr = getattr(desc, name)
            if n == 0 or not addr:
                arr = np.empty(0, dtype=dt)
            else:
                arr = np.ctypeslib.as_array(C.cast(addr, C.POINTER(np.ctypeslib.as_ctypes_type(dt))), shape=(n,)).copy()
            setattr(self, name, arr)


def partition_build(n: int, rowptr: np.ndarray, colidx: np.ndarray, vals: np.ndarray, part: np.ndarray,
                    n_parts: int) -> list[HostPartition]:
    """Runs the library's host-side builder and returns numpy copies of every partition's arrays."""
    L = lib()
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    part = np.ascontiguousarray(part, dtype=np.int32)
    if rowptr.shape[0] != n + 1 or part.shape[0] != n or colidx.shape[0] != vals.shape[0]:
        raise VarcoError(ERR_SHAPE, "partition_build: array lengths do not match n")
    h = C.c_void_p()
    _check(L.varco_partition_build(n, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data, part.ctypes.data,
                                   n_parts, C.byref(h)))
    try:
        out = []
        for q in range(n_parts):
            d = PartitionDesc()
            _check(L.varco_partition_view(h, q, C.byref(d)))
            hp = HostPartition(d)
            hp._fill(d, n_parts)
            out.append(hp)
        return out
    finally:
        L.varco_partition_free(h)


# ---------------------------------------------------------------------------------------------------------
# context
# ---------------------------------------------------------------------------------------------------------

class Context:
    def __init__(self, widths, act, conv: int, n_partitions: int, mask_key: int, dtype: int = F32):
        L = lib()
        self._widths = (C.c_int32 * len(widths))(*widths)
        self._act = (C.c_int32 * len(act))(*act)
        cfg = Config(len(act), n_partitions, conv, dtype, mask_key, self._widths, self._act)
        self._h = C.c_void_p()
        _check(L.varco_create(C.byref(cfg), C.byref(self._h)))
        self.widths = list(widths)
        self.n_layers = len(act)
        self.n_partitions = n_partitions
        self.step_on_device = False
        self._keep = {}          # device tensors of registered partitions (kept alive)
        self.parts = {}

    def close(self):
        if self._h:
            lib().varco_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def register_partition(self, q: int, hp: HostPartition, device="cuda"):
        """Uploads a HostPartition's arrays (torch tensors, kept alive by this object) and registers them."""
        import torch
        dev = {}
        d = PartitionDesc()
        d.n_local, d.n_halo, d.n_boundary = hp.n_local, hp.n_halo, hp.n_boundary
        d.z_row_offset, d.nnz = hp.z_row_offset, hp.nnz
        d.halo_row_offset, d.n_returned = hp.halo_row_offset, hp.n_returned
        for name, _ in _DESC_ARRAYS:
            t = torch.from_numpy(getattr(hp, name)).to(device)
            dev[name] = t
            setattr(d, name, t.data_ptr() if t.numel() else None)
        _check(lib().varco_register_partition(self._h, q, C.byref(d)), self._h)
        self._keep[q] = dev
        self.parts[q] = hp
        return dev

    def register_raw(self, q: int, desc: PartitionDesc):
        _check(lib().varco_register_partition(self._h, q, C.byref(desc)), self._h)

    def prepare(self, stream=None):
        """Workspace set of `stream` (torch's current stream when None) and the tables of the kept positions."""
        _check(lib().varco_prepare(self._h, _stream(stream)), self._h)

    def begin_step(self, step: int):
        _check(lib().varco_begin_step(self._h, step), self._h)

    def step_table_enable(self, stream=None):
        _check(lib().varco_step_table_enable(self._h, _stream(stream)), self._h)
        self.step_on_device = True

    def set_step(self, step: int, stream=None):
        _check(lib().varco_set_step(self._h, step, _stream(stream)), self._h)

    def advance_step(self, stream=None):
        _check(lib().varco_advance_step(self._h, _stream(stream)), self._h)

    def set_matmul_terms(self, terms: int):
        _check(lib().varco_set_matmul_terms(self._h, terms), self._h)

    def set_layer_order(self, layer: int, order: int):
        _check(lib().varco_set_layer_order(self._h, layer, order), self._h)

    def set_ratio(self, layer: int, num: int, den: int = 1):
        _check(lib().varco_set_ratio(self._h, layer, num, den), self._h)

    def keep(self, layer: int) -> int:
        k = C.c_int32()
        _check(lib().varco_get_keep(self._h, layer, C.byref(k)), self._h)
        return k.value

    def compress(self, layer, gids, rows, n_rows, x, ldx, z, stream=None):
        _check(lib().varco_compress(self._h, layer, _ptr(gids), _ptr(rows), n_rows, _ptr(x), ldx, _ptr(z),
                                    _stream(stream)), self._h)

    def decompress(self, layer, gids, rows, n_rows, z, x, ldx, accumulate, stream=None):
        _check(lib().varco_decompress(self._h, layer, _ptr(gids), _ptr(rows), n_rows, _ptr(z), _ptr(x), ldx,
                                      int(accumulate), _stream(stream)), self._h)

    def layer_fwd(self, layer, q, x_local, z_in, h1, h0, x_out, z_out, m_saved, stream=None):
        _check(lib().varco_layer_fwd(self._h, layer, q, _ptr(x_local), _ptr(z_in), _ptr(h1), _ptr(h0), _ptr(x_out),
                                     _ptr(z_out), _ptr(m_saved), _stream(stream)), self._h)

    def layer_bwd(self, layer, q, dx_out, x_out, x_local, m_saved, h1, h0, dh1, dh0, dx_local, dz_halo, stream=None):
        _check(lib().varco_layer_bwd(self._h, layer, q, _ptr(dx_out), _ptr(x_out), _ptr(x_local), _ptr(m_saved),
                                     _ptr(h1), _ptr(h0), _ptr(dh1), _ptr(dh0), _ptr(dx_local), _ptr(dz_halo),
                                     _stream(stream)), self._h)

    def accumulate_returned(self, layer, p, ret_ptr, ret_src, returned, dx_local, stream=None):
        _check(lib().varco_accumulate_returned(self._h, layer, p, _ptr(ret_ptr), _ptr(ret_src), _ptr(returned),
                                               _ptr(dx_local), _stream(stream)), self._h)

    def aggregate_fwd(self, tap, q, y_local, z_in, y_out, stream=None):
        _check(lib().varco_aggregate_fwd(self._h, tap, q, _ptr(y_local), _ptr(z_in), _ptr(y_out), _stream(stream)), self._h)

    def aggregate_bwd(self, tap, q, g_out, g_local, dz_halo, stream=None):
        _check(lib().varco_aggregate_bwd(self._h, tap, q, _ptr(g_out), _ptr(g_local), _ptr(dz_halo), _stream(stream)),
               self._h)

    def transform_fwd(self, layer, y, h, c, accumulate, apply_act, stream=None):
        _check(lib().varco_transform_fwd(self._h, layer, y.shape[0], _ptr(y), _ptr(h), _ptr(c), int(accumulate),
                                         int(apply_act), _stream(stream)), self._h)

    def transform_bwd_weight(self, layer, y, dx_out, x_out, dh, stream=None):
        _check(lib().varco_transform_bwd_weight(self._h, layer, y.shape[0], _ptr(y), _ptr(dx_out), _ptr(x_out), _ptr(dh),
                                                _stream(stream)), self._h)

    def transform_bwd_weight_static(self, layer, y, dx_out, x_out, dh, stream=None):
        _check(lib().varco_transform_bwd_weight_static(self._h, layer, y.shape[0], _ptr(y), _ptr(dx_out), _ptr(x_out),
                                                       _ptr(dh), _stream(stream)), self._h)

    def transform_bwd_input(self, layer, dx_out, x_out, h, g_out, accumulate, stream=None):
        _check(lib().varco_transform_bwd_input(self._h, layer, dx_out.shape[0], _ptr(dx_out), _ptr(x_out), _ptr(h),
                                               _ptr(g_out), int(accumulate), _stream(stream)), self._h)

    def softmax_xent(self, logits, labels, n_classes, scale, dlogits, row_loss, row_correct, totals, stream=None):
        n_rows = logits.shape[0]
        _check(lib().varco_softmax_xent(self._h, _ptr(logits), logits.stride(0) if n_rows else n_classes, _ptr(labels),
                                        n_rows, n_classes, scale, _ptr(dlogits),
                                        dlogits.stride(0) if dlogits is not None and n_rows else n_classes,
                                        _ptr(row_loss), _ptr(row_correct), _ptr(totals), _stream(stream)), self._h)

    def stats(self) -> dict:
        s = Stats()
        _check(lib().varco_get_stats(self._h, C.byref(s)), self._h)
        n = self.n_layers
        return dict(fwd_elems=list(s.fwd_elems)[:n], bwd_elems=list(s.bwd_elems)[:n],
                    full_fwd_elems=list(s.full_fwd_elems)[:n], full_bwd_elems=list(s.full_bwd_elems)[:n],
                    bytes_per_elem=s.bytes_per_elem)

    def reset_stats(self):
        _check(lib().varco_reset_stats(self._h), self._h)

    def profile_enable(self, on: bool):
        _check(lib().varco_profile_enable(self._h, int(on)), self._h)

    def profile_read(self, reset: bool = True) -> dict:
        """Per kernel class: launches, total ms, algorithmic bytes and flops of the bracketed launches."""
        p = Profile()
        _check(lib().varco_profile_read(self._h, C.byref(p), int(reset)), self._h)
        return {name: dict(launches=p.launches[i], ms=p.ms[i], bytes=p.bytes[i], flops=p.flops[i],
                           stream_bytes=p.stream_bytes[i])
                for i, name in enumerate(KERNEL_CLASSES)}
