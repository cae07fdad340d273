"""ctypes binding of include/splitzip.h.  Same names as the C entry points
(without the ``splitzip_`` prefix); torch tensors supply device pointers and
the current HIP stream, nothing else."""
from __future__ import annotations

import ctypes as C
import os

import torch

BF16 = 0
FP8_E5M2 = 1
FP8_E4M3 = 2   # accepted by the variant_* calls only
ESC_POS, ESC_SENTINEL, ESC_ABS32 = 0, 1, 2

STATUS_OVERFLOW = 1
STATUS_BAD_STREAM = 2
STATUS_INTERNAL = 4

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "libsplitzip.so")


class SplitZipError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {lib().splitzip_strerror(code).decode()} ({code})")


class _CCodebook(C.Structure):
    _fields_ = [("dec", C.c_uint8 * 16), ("enc", C.c_uint8 * 256), ("member", C.c_uint8 * 256),
                ("dtype", C.c_uint32)]


class _CSizes(C.Structure):
    _fields_ = [("total_bytes", C.c_uint64), ("n_escapes", C.c_uint64), ("status", C.c_uint32),
                ("reserved", C.c_uint32)]


class _CItem(C.Structure):
    _fields_ = [("d_in", C.c_void_p), ("n_elems", C.c_uint64), ("d_out", C.c_void_p), ("out_capacity", C.c_size_t),
                ("cb", C.POINTER(_CCodebook))]


class _CDItem(C.Structure):
    _fields_ = [("d_comp", C.c_void_p), ("comp_bytes", C.c_size_t), ("n_elems", C.c_uint64), ("d_out", C.c_void_p),
                ("cb", C.POINTER(_CCodebook))]


class _CPaged(C.Structure):
    _fields_ = [("d_pool", C.c_void_p), ("d_block_table", C.c_void_p), ("n_blocks", C.c_uint32),
                ("n_pool_blocks", C.c_uint32), ("block_elems", C.c_uint32), ("reserved", C.c_uint32),
                ("page_stride_bytes", C.c_uint64), ("offset_bytes", C.c_uint64)]


class Variant(C.Structure):
    """splitzip_variant: one of the formats of the paper's ablations"""
    _fields_ = [("dtype", C.c_uint32), ("code_bits", C.c_uint32), ("k", C.c_uint32), ("escape_mode", C.c_uint32),
                ("chunk_elems", C.c_uint32), ("value_bits", C.c_uint32)]

    def __repr__(self):
        return (f"Variant(dtype={self.dtype}, code_bits={self.code_bits}, k={self.k}, "
                f"escape_mode={self.escape_mode}, chunk_elems={self.chunk_elems}, value_bits={self.value_bits})")


_lib = None


def lib():
    """The loaded C library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(
                f"{path} is missing: build it with `python -m paper_2605_01708_amd.build` "
                "(or __graft_entry__.build()); there is no CPU fallback")
        L = C.CDLL(path)
        vp, u64, sz, i = C.c_void_p, C.c_uint64, C.c_size_t, C.c_int
        cbp = C.POINTER(_CCodebook)
        L.splitzip_version.restype = i
        L.splitzip_strerror.restype = C.c_char_p
        L.splitzip_strerror.argtypes = [i]
        L.splitzip_calibrate.restype = i
        L.splitzip_calibrate.argtypes = [vp, u64, i, cbp, C.POINTER(C.c_uint64)]
        L.splitzip_codebook_from_dec.restype = i
        L.splitzip_codebook_from_dec.argtypes = [C.POINTER(C.c_uint8), i, cbp]
        for f in (L.splitzip_fixed_bytes, L.splitzip_compress_bound, L.splitzip_workspace_bytes):
            f.restype = sz
            f.argtypes = [u64, i]
        L.splitzip_total_bytes.restype = sz
        L.splitzip_total_bytes.argtypes = [u64, u64, i]
        L.splitzip_workspace_init.restype = i
        L.splitzip_workspace_init.argtypes = [vp, sz, vp]
        L.splitzip_compress.restype = i
        L.splitzip_compress.argtypes = [vp, u64, i, cbp, vp, sz, vp, sz, vp, vp]
        L.splitzip_decompress.restype = i
        L.splitzip_decompress.argtypes = [vp, sz, u64, i, cbp, vp, vp, vp]
        L.splitzip_codebook_from_hist.restype = i
        L.splitzip_codebook_from_hist.argtypes = [C.POINTER(C.c_uint64), i, cbp]
        L.splitzip_histogram.restype = i
        L.splitzip_histogram.argtypes = [vp, u64, i, vp, vp]
        L.splitzip_codebook_device.restype = i
        L.splitzip_codebook_device.argtypes = [vp, i, vp, vp]
        L.splitzip_compress_dcb.restype = i
        L.splitzip_compress_dcb.argtypes = [vp, u64, i, vp, vp, sz, vp, sz, vp, vp]
        L.splitzip_decompress_dcb.restype = i
        L.splitzip_decompress_dcb.argtypes = [vp, sz, u64, i, vp, vp, vp, vp]
        L.splitzip_compress_batch.restype = i
        L.splitzip_compress_batch.argtypes = [C.POINTER(_CItem), C.c_uint32, i, vp, sz, vp, vp]
        L.splitzip_decompress_batch.restype = i
        L.splitzip_decompress_batch.argtypes = [C.POINTER(_CDItem), C.c_uint32, i, vp, vp]
        L.splitzip_calibrate_batch_device.restype = i
        L.splitzip_calibrate_batch_device.argtypes = [C.POINTER(_CItem), C.c_uint32, i, vp, vp, vp]
        L.splitzip_compress_batch_dcb.restype = i
        L.splitzip_compress_batch_dcb.argtypes = [C.POINTER(_CItem), C.c_uint32, i, vp, vp, sz, vp, vp]
        L.splitzip_decompress_batch_dcb.restype = i
        L.splitzip_decompress_batch_dcb.argtypes = [C.POINTER(_CDItem), C.c_uint32, i, vp, vp, vp]
        L.splitzip_decompress_own.restype = i
        L.splitzip_decompress_own.argtypes = [vp, sz, u64, i, vp, vp, vp]
        L.splitzip_decompress_batch_own.restype = i
        L.splitzip_decompress_batch_own.argtypes = [C.POINTER(_CDItem), C.c_uint32, i, vp, vp]
        L.splitzip_noalloc_max_elems.restype = u64
        L.splitzip_noalloc_max_elems.argtypes = []
        L.splitzip_compress_noalloc.restype = i
        L.splitzip_compress_noalloc.argtypes = [vp, u64, i, cbp, vp, sz, vp, vp]
        L.splitzip_internal_test_hooks.restype = None
        L.splitzip_internal_test_hooks.argtypes = [u64, u64, C.c_uint32, u64]
        L.splitzip_traffic_probe.restype = i
        L.splitzip_traffic_probe.argtypes = [vp, sz, vp, sz, vp]
        L.splitzip_traffic_probe_shape.restype = i
        L.splitzip_traffic_probe_shape.argtypes = [vp, sz, vp, sz, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, vp]
        pgp = C.POINTER(_CPaged)
        L.splitzip_compress_paged.restype = i
        L.splitzip_compress_paged.argtypes = [pgp, u64, i, cbp, vp, sz, vp, sz, vp, vp]
        L.splitzip_decompress_paged.restype = i
        L.splitzip_decompress_paged.argtypes = [vp, sz, u64, i, cbp, pgp, vp, vp]
        L.splitzip_compress_batch_paged.restype = i
        L.splitzip_compress_batch_paged.argtypes = [C.POINTER(_CItem), C.c_uint32, i, pgp, vp, sz, vp, vp]
        L.splitzip_decompress_batch_paged.restype = i
        L.splitzip_decompress_batch_paged.argtypes = [C.POINTER(_CDItem), C.c_uint32, i, pgp, vp, vp]
        vrp = C.POINTER(Variant)
        L.splitzip_variant_supported.restype = i
        L.splitzip_variant_supported.argtypes = [vrp]
        L.splitzip_variant_total_bytes.restype = sz
        L.splitzip_variant_total_bytes.argtypes = [u64, u64, vrp]
        for f in (L.splitzip_variant_compress_bound, L.splitzip_variant_workspace_bytes):
            f.restype = sz
            f.argtypes = [u64, vrp]
        L.splitzip_variant_calibrate.restype = i
        L.splitzip_variant_calibrate.argtypes = [vp, u64, vrp, cbp, C.POINTER(C.c_uint64)]
        L.splitzip_variant_codebook_from_dec.restype = i
        L.splitzip_variant_codebook_from_dec.argtypes = [C.POINTER(C.c_uint8), vrp, cbp]
        L.splitzip_variant_compress.restype = i
        L.splitzip_variant_compress.argtypes = [vp, u64, vrp, cbp, vp, sz, vp, sz, vp, vp]
        L.splitzip_variant_decompress.restype = i
        L.splitzip_variant_decompress.argtypes = [vp, sz, u64, vrp, cbp, vp, vp, vp]
        _lib = L
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise SplitZipError(rc, what)


class Codebook:
    """Host-side calibration tables (a splitzip_codebook)."""

    def __init__(self, c: _CCodebook):
        self.c = c

    @property
    def dtype(self) -> int:
        return int(self.c.dtype)

    @property
    def dec(self):
        return list(self.c.dec)

    @property
    def enc(self):
        return list(self.c.enc)

    @property
    def member(self):
        return list(self.c.member)


def _elem_size(dtype: int) -> int:
    return 2 if dtype == BF16 else 1


def calibrate(sample: torch.Tensor, dtype: int, return_hist: bool = False):
    """splitzip_calibrate on a HOST tensor of raw words (any 2-byte dtype for BF16, 1-byte for E5M2)."""
    if sample.device.type != "cpu":
        raise ValueError("calibration runs on the host: pass a CPU tensor")
    s = sample.contiguous()
    if s.element_size() != _elem_size(dtype):
        raise ValueError("sample element size does not match dtype")
    cb = _CCodebook()
    hist = (C.c_uint64 * 256)()
    _check(lib().splitzip_calibrate(s.data_ptr(), s.numel(), dtype, C.byref(cb), hist), "splitzip_calibrate")
    return (Codebook(cb), list(hist)) if return_hist else Codebook(cb)


def codebook_from_dec(dec, dtype: int) -> Codebook:
    arr = (C.c_uint8 * 16)(*[int(v) for v in dec])
    cb = _CCodebook()
    _check(lib().splitzip_codebook_from_dec(arr, dtype, C.byref(cb)), "splitzip_codebook_from_dec")
    return Codebook(cb)


def codebook_from_hist(hist, dtype: int) -> Codebook:
    """splitzip_codebook_from_hist on a host list / tensor of 256 exponent counts."""
    vals = [int(v) for v in (hist.tolist() if hasattr(hist, "tolist") else hist)]
    arr = (C.c_uint64 * 256)(*vals)
    cb = _CCodebook()
    _check(lib().splitzip_codebook_from_hist(arr, dtype, C.byref(cb)), "splitzip_codebook_from_hist")
    return Codebook(cb)


def histogram(x: torch.Tensor, dtype: int, hist: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """splitzip_histogram: adds the exponent counts of the device words x to hist (256 x int64 on the
    device; a zeroed one is made if none is given) and returns it."""
    if x.element_size() != _elem_size(dtype) or not x.is_contiguous():
        raise ValueError("x must be a contiguous tensor of raw words of the dtype")
    if hist is None:
        hist = torch.zeros(256, dtype=torch.int64, device=x.device)
    _check(lib().splitzip_histogram(x.data_ptr(), x.numel(), dtype, hist.data_ptr(), _stream_ptr(stream)), "splitzip_histogram")
    return hist


class DeviceCodebook:
    """A splitzip_codebook in device memory, written by splitzip_codebook_device."""

    def __init__(self, dtype: int, device="cuda"):
        self.dtype = dtype
        self.buf = torch.zeros((C.sizeof(_CCodebook) + 7) // 8, dtype=torch.int64, device=device)

    def to_host(self) -> Codebook:
        """Copy of the tables on the host (synchronises)."""
        raw = self.buf.cpu().numpy().tobytes()[: C.sizeof(_CCodebook)]
        return Codebook(_CCodebook.from_buffer_copy(raw))


def codebook_device(hist: torch.Tensor, dtype: int, out: DeviceCodebook | None = None, stream=None) -> DeviceCodebook:
    """splitzip_codebook_device: the tables for 256 device counts, written to device memory."""
    out = DeviceCodebook(dtype, hist.device) if out is None else out
    _check(lib().splitzip_codebook_device(hist.data_ptr(), dtype, out.buf.data_ptr(), _stream_ptr(stream)), "splitzip_codebook_device")
    return out


def compress_dcb(x: torch.Tensor, d_cb: DeviceCodebook, out: torch.Tensor, workspace: "Workspace", sizes: torch.Tensor,
                 stream=None, capacity: int | None = None) -> None:
    """splitzip_compress_dcb: splitzip_compress with a codebook in device memory."""
    if x.element_size() != _elem_size(d_cb.dtype) or not x.is_contiguous():
        raise ValueError("x must be a contiguous tensor of raw words of the codebook's dtype")
    cap = out.numel() * out.element_size() if capacity is None else capacity
    _check(lib().splitzip_compress_dcb(x.data_ptr(), x.numel(), d_cb.dtype, d_cb.buf.data_ptr(), out.data_ptr(), cap,
                                       workspace.buf.data_ptr(), workspace.nbytes, sizes.data_ptr(), _stream_ptr(stream)),
           "splitzip_compress_dcb")


def decompress_dcb(comp: torch.Tensor, comp_bytes: int, n_elems: int, d_cb: DeviceCodebook, out: torch.Tensor,
                   sizes: torch.Tensor | None = None, stream=None) -> None:
    """splitzip_decompress_dcb: splitzip_decompress with a codebook in device memory."""
    if out.numel() < n_elems or out.element_size() != _elem_size(d_cb.dtype) or not out.is_contiguous():
        raise ValueError("out must be a contiguous tensor of at least n_elems raw words")
    _check(lib().splitzip_decompress_dcb(comp.data_ptr(), comp_bytes, n_elems, d_cb.dtype, d_cb.buf.data_ptr(), out.data_ptr(),
                                         sizes.data_ptr() if sizes is not None else None, _stream_ptr(stream)),
           "splitzip_decompress_dcb")


def fixed_bytes(n: int, dtype: int) -> int:
    return int(lib().splitzip_fixed_bytes(n, dtype))


def total_bytes(n: int, m: int, dtype: int) -> int:
    return int(lib().splitzip_total_bytes(n, m, dtype))


def compress_bound(n: int, dtype: int) -> int:
    return int(lib().splitzip_compress_bound(n, dtype))


def workspace_bytes(n: int, dtype: int) -> int:
    return int(lib().splitzip_workspace_bytes(n, dtype))


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


class Workspace:
    """Device scratch for compress calls of up to n_elems; initialised once."""

    def __init__(self, n_elems: int, dtype: int, device="cuda", stream=None):
        self.n_elems = n_elems
        self.nbytes = workspace_bytes(n_elems, dtype)
        self.buf = torch.empty(self.nbytes, dtype=torch.uint8, device=device)
        _check(lib().splitzip_workspace_init(self.buf.data_ptr(), self.nbytes, _stream_ptr(stream)),
               "splitzip_workspace_init")


def new_sizes(device="cuda") -> torch.Tensor:
    """Zeroed device splitzip_sizes record (24 bytes as 3 x int64)."""
    return torch.zeros(3, dtype=torch.int64, device=device)


def read_sizes(sizes: torch.Tensor):
    """(total_bytes, n_escapes, status) -- copies the record to the host (synchronises)."""
    h = sizes.cpu()
    return int(h[0]), int(h[1]), int(h[2]) & 0xFFFFFFFF


def compress(x: torch.Tensor, cb: Codebook, out: torch.Tensor, workspace: Workspace,
             sizes: torch.Tensor, stream=None, capacity: int | None = None) -> None:
    """splitzip_compress: x (device words) -> out (device uint8), sizes written on the stream."""
    n = x.numel()
    if x.element_size() != _elem_size(cb.dtype) or not x.is_contiguous():
        raise ValueError("x must be a contiguous tensor of raw words of the codebook's dtype")
    cap = out.numel() * out.element_size() if capacity is None else capacity
    _check(lib().splitzip_compress(x.data_ptr(), n, cb.dtype, C.byref(cb.c), out.data_ptr(), cap,
                                   workspace.buf.data_ptr(), workspace.nbytes, sizes.data_ptr(),
                                   _stream_ptr(stream)), "splitzip_compress")


def internal_test_hooks(stage_bytes: int = 0, status_bytes: int = 0, finish_groups: int = 0, direct_bytes: int = 0) -> None:
    """What the tests of the rarely taken paths turn (not part of splitzip.h): a staging area and a status area smaller
    than the workspace has, the groups of tiles per workgroup of the finishing pass (1, 2 or 4), and the bytes of tile
    counts a launch's finishing pass may read directly (beyond: sums of 64 counts).  0 = as built."""
    lib().splitzip_internal_test_hooks(stage_bytes, status_bytes, finish_groups, direct_bytes)


def noalloc_max_elems() -> int:
    return int(lib().splitzip_noalloc_max_elems())


def compress_noalloc(x: torch.Tensor, cb: Codebook, out: torch.Tensor, sizes: torch.Tensor, stream=None,
                     capacity: int | None = None) -> None:
    """splitzip_compress_noalloc: splitzip_compress on the library's own per-GPU scratch array instead of a workspace."""
    n = x.numel()
    if x.element_size() != _elem_size(cb.dtype) or not x.is_contiguous():
        raise ValueError("x must be a contiguous tensor of raw words of the codebook's dtype")
    cap = out.numel() * out.element_size() if capacity is None else capacity
    _check(lib().splitzip_compress_noalloc(x.data_ptr(), n, cb.dtype, C.byref(cb.c), out.data_ptr(), cap,
                                           sizes.data_ptr(), _stream_ptr(stream)), "splitzip_compress_noalloc")


def decompress(comp: torch.Tensor, comp_bytes: int, n_elems: int, cb: Codebook, out: torch.Tensor,
               sizes: torch.Tensor | None = None, stream=None) -> None:
    """splitzip_decompress: comp (device uint8 stream) -> out (device words)."""
    if out.numel() < n_elems or out.element_size() != _elem_size(cb.dtype) or not out.is_contiguous():
        raise ValueError("out must be a contiguous tensor of at least n_elems raw words")
    _check(lib().splitzip_decompress(comp.data_ptr(), comp_bytes, n_elems, cb.dtype, C.byref(cb.c),
                                     out.data_ptr(), sizes.data_ptr() if sizes is not None else None,
                                     _stream_ptr(stream)), "splitzip_decompress")


def new_sizes_array(n: int, device="cuda") -> torch.Tensor:
    """n zeroed device splitzip_sizes records, one row of 3 x int64 each."""
    return torch.zeros(n, 3, dtype=torch.int64, device=device)


def read_sizes_array(sizes: torch.Tensor):
    """[(total_bytes, n_escapes, status), ...] -- copies to the host (synchronises)."""
    h = sizes.cpu().tolist()
    return [(int(r[0]), int(r[1]), int(r[2]) & 0xFFFFFFFF) for r in h]


class CompressBatch:
    """The marshalled item list of a splitzip_compress_batch call; build once, launch many times."""

    def __init__(self, xs, cbs, outs, capacities=None):
        if not (len(xs) == len(cbs) == len(outs)):
            raise ValueError("xs, cbs and outs must have the same length")
        self.n = len(xs)
        self.dtype = cbs[0].dtype if cbs else BF16
        self.items = (_CItem * max(self.n, 1))()
        self._keep = (list(xs), list(cbs), list(outs))
        for k, (x, cb, out) in enumerate(zip(xs, cbs, outs)):
            if x.element_size() != _elem_size(cb.dtype) or not x.is_contiguous() or cb.dtype != self.dtype:
                raise ValueError("every x must be a contiguous tensor of raw words of one dtype")
            cap = out.numel() * out.element_size() if capacities is None else capacities[k]
            self.items[k] = _CItem(x.data_ptr(), x.numel(), out.data_ptr(), cap, C.pointer(cb.c))

    def launch(self, workspace: "Workspace", sizes: torch.Tensor, stream=None) -> None:
        _check(lib().splitzip_compress_batch(self.items, self.n, self.dtype, workspace.buf.data_ptr(), workspace.nbytes,
                                             sizes.data_ptr(), _stream_ptr(stream)), "splitzip_compress_batch")


class DecompressBatch:
    """The marshalled item list of a splitzip_decompress_batch call."""

    def __init__(self, comps, comp_bytes, n_elems, cbs, outs):
        if not (len(comps) == len(comp_bytes) == len(n_elems) == len(cbs) == len(outs)):
            raise ValueError("all lists must have the same length")
        self.n = len(comps)
        self.dtype = cbs[0].dtype if cbs else BF16
        self.items = (_CDItem * max(self.n, 1))()
        self._keep = (list(comps), list(cbs), list(outs))
        for k, (c, cbytes, n, cb, out) in enumerate(zip(comps, comp_bytes, n_elems, cbs, outs)):
            if out.numel() < n or out.element_size() != _elem_size(cb.dtype) or not out.is_contiguous() or cb.dtype != self.dtype:
                raise ValueError("every out must be a contiguous tensor of at least n_elems raw words of one dtype")
            self.items[k] = _CDItem(c.data_ptr(), cbytes, n, out.data_ptr(), C.pointer(cb.c))

    def launch(self, sizes: torch.Tensor | None = None, stream=None) -> None:
        _check(lib().splitzip_decompress_batch(self.items, self.n, self.dtype,
                                               sizes.data_ptr() if sizes is not None else None, _stream_ptr(stream)),
               "splitzip_decompress_batch")


class DeviceCodebooks:
    """n splitzip_codebook in device memory, written by splitzip_calibrate_batch_device, and the counts they come from."""

    def __init__(self, n: int, dtype: int, device="cuda"):
        self.n, self.dtype = n, dtype
        self.buf = torch.zeros(max(n, 1) * C.sizeof(_CCodebook) // 4, dtype=torch.int32, device=device)
        self.hists = torch.zeros((max(n, 1), 256), dtype=torch.int64, device=device)

    def to_host(self, k: int) -> Codebook:
        """Copy of the k-th codebook on the host (synchronises)."""
        w = C.sizeof(_CCodebook) // 4
        raw = self.buf[k * w:(k + 1) * w].cpu().numpy().tobytes()
        return Codebook(_CCodebook.from_buffer_copy(raw))


def _null_cb():
    return C.POINTER(_CCodebook)()


class CalibrateBatchDevice:
    """splitzip_calibrate_batch_device: a codebook per tensor, counted and ranked on the device."""

    def __init__(self, xs, dcbs: DeviceCodebooks):
        self.n, self.dcbs = len(xs), dcbs
        self.items = (_CItem * max(self.n, 1))()
        self._keep = list(xs)
        for k, x in enumerate(xs):
            if x.element_size() != _elem_size(dcbs.dtype) or not x.is_contiguous():
                raise ValueError("every x must be a contiguous tensor of raw words of the codebooks' dtype")
            self.items[k] = _CItem(x.data_ptr(), x.numel(), None, 0, _null_cb())

    def launch(self, stream=None) -> None:
        _check(lib().splitzip_calibrate_batch_device(self.items, self.n, self.dcbs.dtype, self.dcbs.hists.data_ptr(),
                                                     self.dcbs.buf.data_ptr(), _stream_ptr(stream)), "splitzip_calibrate_batch_device")


class CompressBatchDcb:
    """splitzip_compress_batch_dcb: tensor k under the k-th codebook of a DeviceCodebooks."""

    def __init__(self, xs, dcbs: DeviceCodebooks, outs, capacities=None):
        if not (len(xs) == len(outs)) or len(xs) > dcbs.n:
            raise ValueError("xs and outs must have the same length, at most the number of codebooks")
        self.n, self.dcbs = len(xs), dcbs
        self.items = (_CItem * max(self.n, 1))()
        self._keep = (list(xs), list(outs))
        for k, (x, out) in enumerate(zip(xs, outs)):
            if x.element_size() != _elem_size(dcbs.dtype) or not x.is_contiguous():
                raise ValueError("every x must be a contiguous tensor of raw words of the codebooks' dtype")
            cap = out.numel() * out.element_size() if capacities is None else capacities[k]
            self.items[k] = _CItem(x.data_ptr(), x.numel(), out.data_ptr(), cap, _null_cb())

    def launch(self, workspace: "Workspace", sizes: torch.Tensor, stream=None) -> None:
        _check(lib().splitzip_compress_batch_dcb(self.items, self.n, self.dcbs.dtype, self.dcbs.buf.data_ptr(),
                                                 workspace.buf.data_ptr(), workspace.nbytes, sizes.data_ptr(),
                                                 _stream_ptr(stream)), "splitzip_compress_batch_dcb")


class DecompressBatchDcb:
    """splitzip_decompress_batch_dcb: stream k under the k-th codebook of a DeviceCodebooks."""

    def __init__(self, comps, comp_bytes, n_elems, dcbs: DeviceCodebooks, outs):
        if not (len(comps) == len(comp_bytes) == len(n_elems) == len(outs)) or len(comps) > dcbs.n:
            raise ValueError("all lists must have the same length, at most the number of codebooks")
        self.n, self.dcbs = len(comps), dcbs
        self.items = (_CDItem * max(self.n, 1))()
        self._keep = (list(comps), list(outs))
        for k, (c, cbytes, n, out) in enumerate(zip(comps, comp_bytes, n_elems, outs)):
            if out.numel() < n or out.element_size() != _elem_size(dcbs.dtype) or not out.is_contiguous():
                raise ValueError("every out must be a contiguous tensor of at least n_elems raw words of the codebooks' dtype")
            self.items[k] = _CDItem(c.data_ptr(), cbytes, n, out.data_ptr(), _null_cb())

    def launch(self, sizes: torch.Tensor | None = None, stream=None) -> None:
        _check(lib().splitzip_decompress_batch_dcb(self.items, self.n, self.dcbs.dtype, self.dcbs.buf.data_ptr(),
                                                   sizes.data_ptr() if sizes is not None else None, _stream_ptr(stream)),
               "splitzip_decompress_batch_dcb")


def decompress_own(comp: torch.Tensor, comp_bytes: int, n_elems: int, dtype: int, out: torch.Tensor,
                   sizes: torch.Tensor | None = None, stream=None) -> None:
    """splitzip_decompress_own: decompress with the codebook the stream carries in its header."""
    if out.numel() < n_elems or out.element_size() != _elem_size(dtype) or not out.is_contiguous():
        raise ValueError("out must be a contiguous tensor of at least n_elems raw words of the dtype")
    _check(lib().splitzip_decompress_own(comp.data_ptr(), comp_bytes, n_elems, dtype, out.data_ptr(),
                                         sizes.data_ptr() if sizes is not None else None, _stream_ptr(stream)),
           "splitzip_decompress_own")


class DecompressBatchOwn:
    """splitzip_decompress_batch_own: every stream under the codebook of its own header."""

    def __init__(self, comps, comp_bytes, n_elems, dtype: int, outs):
        if not (len(comps) == len(comp_bytes) == len(n_elems) == len(outs)):
            raise ValueError("all lists must have the same length")
        self.n, self.dtype = len(comps), dtype
        self.items = (_CDItem * max(self.n, 1))()
        self._keep = (list(comps), list(outs))
        for k, (c, cbytes, n, out) in enumerate(zip(comps, comp_bytes, n_elems, outs)):
            if out.numel() < n or out.element_size() != _elem_size(dtype) or not out.is_contiguous():
                raise ValueError("every out must be a contiguous tensor of at least n_elems raw words of the dtype")
            self.items[k] = _CDItem(c.data_ptr(), cbytes, n, out.data_ptr(), _null_cb())

    def launch(self, sizes: torch.Tensor | None = None, stream=None) -> None:
        _check(lib().splitzip_decompress_batch_own(self.items, self.n, self.dtype,
                                                   sizes.data_ptr() if sizes is not None else None, _stream_ptr(stream)),
               "splitzip_decompress_batch_own")


def compress_batch(xs, cbs, outs, workspace: Workspace, sizes: torch.Tensor, stream=None, capacities=None) -> None:
    """splitzip_compress_batch: xs[k] -> outs[k] with codebook cbs[k]; sizes = new_sizes_array(len(xs))."""
    CompressBatch(xs, cbs, outs, capacities).launch(workspace, sizes, stream)


def decompress_batch(comps, comp_bytes, n_elems, cbs, outs, sizes: torch.Tensor | None = None, stream=None) -> None:
    """splitzip_decompress_batch: comps[k] (comp_bytes[k] bytes, n_elems[k] words) -> outs[k]."""
    DecompressBatch(comps, comp_bytes, n_elems, cbs, outs).launch(sizes, stream)


def traffic_probe(src: torch.Tensor, read_bytes: int, dst: torch.Tensor, write_bytes: int, stream=None) -> None:
    _check(lib().splitzip_traffic_probe(src.data_ptr(), read_bytes, dst.data_ptr(), write_bytes,
                                        _stream_ptr(stream)), "splitzip_traffic_probe")


def traffic_probe_shape(src: torch.Tensor, read_bytes: int, dst: torch.Tensor, write_bytes: int, reads_per_step: int,
                        writes_per_step: int, wgs_per_cu: int, flags: int = 3, stream=None) -> None:
    _check(lib().splitzip_traffic_probe_shape(src.data_ptr(), read_bytes, dst.data_ptr(), write_bytes, reads_per_step,
                                              writes_per_step, wgs_per_cu, flags, _stream_ptr(stream)),
           "splitzip_traffic_probe_shape")


# ---- format variants of the ablations -----------------------------------------------------------

def variant(dtype: int, code_bits: int = 4, k: int = 16, escape_mode: int = 0, chunk_elems: int = 1024,
            value_bits: int = 0) -> Variant:
    return Variant(dtype, code_bits, k, escape_mode, chunk_elems, value_bits)


def variant_supported(v: Variant) -> bool:
    return bool(lib().splitzip_variant_supported(C.byref(v)))


def variant_total_bytes(n: int, m: int, v: Variant) -> int:
    return int(lib().splitzip_variant_total_bytes(n, m, C.byref(v)))


def variant_compress_bound(n: int, v: Variant) -> int:
    return int(lib().splitzip_variant_compress_bound(n, C.byref(v)))


def variant_workspace_bytes(n: int, v: Variant) -> int:
    return int(lib().splitzip_variant_workspace_bytes(n, C.byref(v)))


def variant_calibrate(sample: torch.Tensor, v: Variant, return_hist: bool = False):
    """splitzip_variant_calibrate on a HOST tensor of raw words."""
    if sample.device.type != "cpu":
        raise ValueError("calibration runs on the host: pass a CPU tensor")
    s = sample.contiguous()
    if s.element_size() != _elem_size(v.dtype):
        raise ValueError("sample element size does not match dtype")
    cb = _CCodebook()
    hist = (C.c_uint64 * 256)()
    _check(lib().splitzip_variant_calibrate(s.data_ptr(), s.numel(), C.byref(v), C.byref(cb), hist),
           "splitzip_variant_calibrate")
    return (Codebook(cb), list(hist)) if return_hist else Codebook(cb)


def variant_codebook_from_dec(dec, v: Variant) -> Codebook:
    vals = [int(x) for x in dec][:16]
    arr = (C.c_uint8 * 16)(*(vals + [0] * (16 - len(vals))))
    cb = _CCodebook()
    _check(lib().splitzip_variant_codebook_from_dec(arr, C.byref(v), C.byref(cb)), "splitzip_variant_codebook_from_dec")
    return Codebook(cb)


def variant_compress(x: torch.Tensor, v: Variant, cb: Codebook, out: torch.Tensor, workspace: torch.Tensor,
                     sizes: torch.Tensor, stream=None, capacity: int | None = None) -> None:
    """splitzip_variant_compress; workspace is a device uint8 tensor of variant_workspace_bytes."""
    if x.element_size() != _elem_size(v.dtype) or not x.is_contiguous():
        raise ValueError("x must be a contiguous tensor of raw words of the variant's dtype")
    cap = out.numel() * out.element_size() if capacity is None else capacity
    _check(lib().splitzip_variant_compress(x.data_ptr(), x.numel(), C.byref(v), C.byref(cb.c), out.data_ptr(), cap,
                                           workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                           sizes.data_ptr(), _stream_ptr(stream)), "splitzip_variant_compress")


def variant_decompress(comp: torch.Tensor, comp_bytes: int, n_elems: int, v: Variant, cb: Codebook, out: torch.Tensor,
                       sizes: torch.Tensor | None = None, stream=None) -> None:
    if out.numel() < n_elems or out.element_size() != _elem_size(v.dtype) or not out.is_contiguous():
        raise ValueError("out must be a contiguous tensor of at least n_elems raw words")
    _check(lib().splitzip_variant_decompress(comp.data_ptr(), comp_bytes, n_elems, C.byref(v), C.byref(cb.c),
                                             out.data_ptr(), sizes.data_ptr() if sizes is not None else None,
                                             _stream_ptr(stream)), "splitzip_variant_decompress")


# ---- paged / strided tensors ------------------------------------------------------------------------

class Paged:
    """splitzip_paged: a tensor whose words sit in pages of a pool, found through a block table.

    pool: device tensor (any dtype) holding the pages; block_table: device int32/uint32 tensor of page indices;
    block_elems: elements of this tensor per page; page_stride_bytes / offset_bytes as in include/splitzip.h."""

    def __init__(self, pool: torch.Tensor, block_table: torch.Tensor, block_elems: int, page_stride_bytes: int,
                 offset_bytes: int = 0, n_pool_blocks: int | None = None):
        if block_table.element_size() != 4 or not block_table.is_contiguous():
            raise ValueError("block_table must be a contiguous tensor of 32-bit page indices")
        self.pool, self.block_table = pool, block_table            # keep the tensors alive
        pool_bytes = pool.numel() * pool.element_size()
        npool = pool_bytes // page_stride_bytes if n_pool_blocks is None else n_pool_blocks
        self.c = _CPaged(pool.data_ptr(), block_table.data_ptr(), block_table.numel(), npool, block_elems, 0,
                         page_stride_bytes, offset_bytes)


def compress_paged(src: Paged, n_elems: int, cb: Codebook, out: torch.Tensor, workspace: Workspace,
                   sizes: torch.Tensor, stream=None, capacity: int | None = None) -> None:
    cap = out.numel() * out.element_size() if capacity is None else capacity
    _check(lib().splitzip_compress_paged(C.byref(src.c), n_elems, cb.dtype, C.byref(cb.c), out.data_ptr(), cap,
                                         workspace.buf.data_ptr(), workspace.nbytes, sizes.data_ptr(),
                                         _stream_ptr(stream)), "splitzip_compress_paged")


def decompress_paged(comp: torch.Tensor, comp_bytes: int, n_elems: int, cb: Codebook, dst: Paged,
                     sizes: torch.Tensor | None = None, stream=None) -> None:
    _check(lib().splitzip_decompress_paged(comp.data_ptr(), comp_bytes, n_elems, cb.dtype, C.byref(cb.c),
                                           C.byref(dst.c), sizes.data_ptr() if sizes is not None else None,
                                           _stream_ptr(stream)), "splitzip_decompress_paged")


class CompressBatchPaged:
    """splitzip_compress_batch_paged: tensors k = 0.. in pools that share one block table.  pools[k] is a device tensor
    whose first byte is the tensor's first word in page 0 (a view into the pool at the tensor's offset); n_elems[k] its
    logical length; paging a Paged that carries the table and the page geometry."""

    def __init__(self, pools, n_elems, cbs, outs, paging: Paged, capacities=None):
        if not (len(pools) == len(n_elems) == len(cbs) == len(outs)):
            raise ValueError("all lists must have the same length")
        self.n = len(pools)
        self.dtype = cbs[0].dtype if cbs else BF16
        self.paging = paging
        self.items = (_CItem * max(self.n, 1))()
        self._keep = (list(pools), list(cbs), list(outs))
        for k, (pool, n, cb, out) in enumerate(zip(pools, n_elems, cbs, outs)):
            cap = out.numel() * out.element_size() if capacities is None else capacities[k]
            self.items[k] = _CItem(pool.data_ptr(), n, out.data_ptr(), cap, C.pointer(cb.c))

    def launch(self, workspace: "Workspace", sizes: torch.Tensor, stream=None) -> None:
        _check(lib().splitzip_compress_batch_paged(self.items, self.n, self.dtype, C.byref(self.paging.c),
                                                   workspace.buf.data_ptr(), workspace.nbytes, sizes.data_ptr(),
                                                   _stream_ptr(stream)), "splitzip_compress_batch_paged")


class DecompressBatchPaged:
    """splitzip_decompress_batch_paged: the reverse, into pools that share one block table."""

    def __init__(self, comps, comp_bytes, n_elems, cbs, pools, paging: Paged):
        if not (len(comps) == len(comp_bytes) == len(n_elems) == len(cbs) == len(pools)):
            raise ValueError("all lists must have the same length")
        self.n = len(comps)
        self.dtype = cbs[0].dtype if cbs else BF16
        self.paging = paging
        self.items = (_CDItem * max(self.n, 1))()
        self._keep = (list(comps), list(cbs), list(pools))
        for k, (c, cbytes, n, cb, pool) in enumerate(zip(comps, comp_bytes, n_elems, cbs, pools)):
            self.items[k] = _CDItem(c.data_ptr(), cbytes, n, pool.data_ptr(), C.pointer(cb.c))

    def launch(self, sizes: torch.Tensor | None = None, stream=None) -> None:
        _check(lib().splitzip_decompress_batch_paged(self.items, self.n, self.dtype, C.byref(self.paging.c),
                                                     sizes.data_ptr() if sizes is not None else None, _stream_ptr(stream)),
               "splitzip_decompress_batch_paged")
