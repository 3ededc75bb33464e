"""Thin ctypes binding of the HIP codec library (include/zc.h).

Argument marshalling only: every step of the codec runs in the library's
kernels.  PyTorch supplies device memory and the current stream.  There is no
fallback: if libzc.so is not built (see __graft_entry__.build) importing the
library handle raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libzc.so")

FMT_BF16, FMT_FP8_E4M3, FMT_FP4_E2M1_MX, FMT_FP8_E4M3_BYTES, FMT_FP4_E2M1_MX_BYTES, FMT_FP4_E2M1_NV, FMT_FP8_E5M2 = 1, 2, 3, 4, 5, 6, 7
POLICY_HUFF_ALL, POLICY_AUTO = 0, 1
FLAG_HOST_CODES = 1
FLAG_REVERSE_FIELDS = 2
NOALLOC_SCRATCH_BYTES = 4 << 20
MODE_EMPTY, MODE_HUFF, MODE_RAW, MODE_CONST = 0, 1, 2, 3
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_BUFFER_TOO_SMALL, ERR_CORRUPT, ERR_DEVICE = range(6)

EXPORTS = ["zc_compress_bound", "zc_workspace_bytes", "zc_compress", "zc_compress_batch", "zc_read_info",
           "zc_decompress", "zc_decompress_chunks", "zc_decompress_batch", "zc_decompress_batch_plan",
           "zc_decompress_batch_run", "zc_stats", "zc_build_code", "zc_train_code", "zc_compress_with_code",
           "zc_compress_batch_with_code", "zc_compress_batch_with_code_async", "zc_compress_batch_async", "zc_code_stale",
           "zc_validate_container", "zc_release_host_buffers", "zc_compress_noalloc", "zc_copy_reference", "zc_status_string"]


class Params(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("format", C.c_uint32), ("chunk_bytes", C.c_uint32),
                ("max_code_len", C.c_uint32 * 3), ("streams_per_chunk", C.c_uint32), ("policy", C.c_uint32),
                ("flags", C.c_uint32)]


class Info(C.Structure):
    _fields_ = [("format", C.c_uint32), ("policy", C.c_uint32), ("streams", C.c_uint32), ("n_fields", C.c_uint32),
                ("xor_delta", C.c_uint32), ("chunk_bytes", C.c_uint32), ("n_chunks", C.c_uint32), ("payload_order", C.c_uint32),
                ("n_elems", C.c_uint64), ("total_bytes", C.c_uint64), ("payload_offset", C.c_uint64),
                ("table_offset", C.c_uint64 * 3), ("index_offset", C.c_uint64 * 3),
                ("mode", C.c_uint8 * 3), ("sym_bits", C.c_uint8 * 3), ("max_len", C.c_uint8 * 3), ("const_symbol", C.c_uint8 * 3),
                ("code_len", (C.c_uint8 * 256) * 3)]


class FieldStats(C.Structure):
    _fields_ = [("alphabet", C.c_uint32), ("distinct", C.c_uint32), ("mode", C.c_uint32), ("max_len", C.c_uint32),
                ("n_symbols", C.c_uint64), ("hist", C.c_uint64 * 256), ("code_len", C.c_uint8 * 256),
                ("entropy_bits", C.c_double), ("mean_code_len", C.c_double), ("payload_bits", C.c_uint64),
                ("stream_bytes", C.c_uint64), ("ratio_payload", C.c_double)]


class StatsOut(C.Structure):
    _fields_ = [("n_fields", C.c_uint32), ("reserved", C.c_uint32), ("raw_bytes", C.c_uint64),
                ("container_bytes", C.c_uint64), ("ratio_payload_total", C.c_double),
                ("ratio_container_total", C.c_double), ("field", FieldStats * 3)]


class Tensor(C.Structure):
    _fields_ = [("d_src", C.c_void_p), ("d_xor_base", C.c_void_p), ("d_scales", C.c_void_p), ("n_elems", C.c_uint64),
                ("d_comp", C.c_void_p), ("comp_capacity", C.c_uint64), ("d_dst", C.c_void_p), ("d_scales_out", C.c_void_p),
                ("d_chunk_ids", C.c_void_p), ("n_chunk_ids", C.c_uint32), ("reserved", C.c_uint32),
                ("out_bytes", C.c_uint64), ("info", Info)]


class BatchPlan(C.Structure):
    _fields_ = [("format", C.c_uint32), ("streams", C.c_uint32), ("n_tensors", C.c_uint32), ("n_fast_work", C.c_uint32),
                ("n_work", C.c_uint32), ("fast_kernel", C.c_uint32), ("fast_exp_kind", C.c_uint32), ("fast_sm_kind", C.c_uint32),
                ("n_rings", C.c_uint32), ("xor_delta", C.c_uint32), ("scattered", C.c_uint32), ("tail_kernel", C.c_uint32),
                ("fast_work_offset", C.c_uint64), ("work_offset", C.c_uint64)]


class ZcError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        RuntimeError.__init__(self, "%s: %s" % (what, status_string(status)))


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        vp, u64, u32 = C.c_void_p, C.c_uint64, C.c_uint32
        L.zc_status_string.restype = C.c_char_p
        L.zc_status_string.argtypes = [C.c_int]
        L.zc_compress_bound.restype = u64
        L.zc_compress_bound.argtypes = [u64, C.POINTER(Params)]
        L.zc_workspace_bytes.restype = u64
        L.zc_workspace_bytes.argtypes = [C.POINTER(u64), u32, C.POINTER(Params)]
        L.zc_compress.restype = C.c_int
        L.zc_compress.argtypes = [vp, u64, C.POINTER(Params), vp, vp, vp, u64, C.POINTER(u64), C.POINTER(Info), vp, u64, vp]
        L.zc_compress_batch.restype = C.c_int
        L.zc_compress_batch.argtypes = [C.POINTER(Tensor), u32, C.POINTER(Params), vp, u64, vp]
        L.zc_compress_noalloc.restype = C.c_int
        L.zc_compress_noalloc.argtypes = [vp, u64, C.POINTER(Params), vp, vp, vp, u64, vp]
        L.zc_copy_reference.restype = C.c_int
        L.zc_copy_reference.argtypes = [vp, vp, u64, u32, vp]
        L.zc_code_stale.restype = C.c_int
        L.zc_code_stale.argtypes = [C.POINTER(Info), C.POINTER(Info), C.c_double]
        L.zc_train_code.restype = C.c_int
        L.zc_train_code.argtypes = [vp, u64, C.POINTER(Params), vp, vp, C.POINTER(Info), vp, u64, vp]
        L.zc_compress_with_code.restype = C.c_int
        L.zc_compress_with_code.argtypes = [vp, u64, C.POINTER(Params), C.POINTER(Info), vp, vp, vp, u64, C.POINTER(u64), C.POINTER(Info), vp, u64, vp]
        L.zc_compress_batch_with_code.restype = C.c_int
        L.zc_compress_batch_with_code.argtypes = [C.POINTER(Tensor), u32, C.POINTER(Params), C.POINTER(Info), vp, u64, vp]
        L.zc_compress_batch_with_code_async.restype = C.c_int
        L.zc_compress_batch_with_code_async.argtypes = [C.POINTER(Tensor), u32, C.POINTER(Params), C.POINTER(Info), vp, u64, vp]
        L.zc_compress_batch_async.restype = C.c_int
        L.zc_compress_batch_async.argtypes = [C.POINTER(Tensor), u32, C.POINTER(Params), vp, u64, vp]
        L.zc_read_info.restype = C.c_int
        L.zc_read_info.argtypes = [vp, u64, C.c_int, C.POINTER(Info), vp]
        L.zc_decompress.restype = C.c_int
        L.zc_decompress.argtypes = [vp, u64, C.POINTER(Info), vp, u64, vp, vp, vp]
        L.zc_decompress_chunks.restype = C.c_int
        L.zc_decompress_chunks.argtypes = [vp, u64, C.POINTER(Info), vp, u32, vp, u64, vp, vp, vp]
        L.zc_decompress_batch.restype = C.c_int
        L.zc_decompress_batch.argtypes = [C.POINTER(Tensor), u32, vp, u64, vp]
        L.zc_decompress_batch_plan.restype = C.c_int
        L.zc_decompress_batch_plan.argtypes = [C.POINTER(Tensor), u32, vp, u64, C.POINTER(BatchPlan), vp]
        L.zc_decompress_batch_run.restype = C.c_int
        L.zc_decompress_batch_run.argtypes = [C.POINTER(BatchPlan), vp, vp]
        L.zc_stats.restype = C.c_int
        L.zc_stats.argtypes = [vp, u64, C.POINTER(Params), vp, vp, C.POINTER(StatsOut), vp, u64, vp]
        L.zc_validate_container.restype = C.c_int
        L.zc_validate_container.argtypes = [vp, u64, u64, C.c_int, C.POINTER(Info)]
        L.zc_release_host_buffers.restype = C.c_int
        L.zc_release_host_buffers.argtypes = []
        L.zc_build_code.restype = C.c_int
        L.zc_build_code.argtypes = [C.POINTER(u64), u32, u32, C.POINTER(C.c_uint8), C.POINTER(C.c_uint16)]
        _lib = L
    return _lib


def status_string(status):
    return lib().zc_status_string(status).decode()


def params(fmt, chunk_bytes, max_code_len=(0, 0, 0), streams=0, policy=POLICY_HUFF_ALL, flags=0):
    p = Params()
    p.struct_size = C.sizeof(Params)
    p.format, p.chunk_bytes, p.streams_per_chunk, p.policy, p.flags = fmt, chunk_bytes, streams, policy, flags
    for i in range(3):
        p.max_code_len[i] = max_code_len[i]
    return p


def elem_bits(fmt):
    return {FMT_BF16: 16, FMT_FP8_E4M3: 8, FMT_FP4_E2M1_MX: 4, FMT_FP8_E4M3_BYTES: 8, FMT_FP4_E2M1_MX_BYTES: 4, FMT_FP4_E2M1_NV: 4, FMT_FP8_E5M2: 8}[fmt]


def scale_block(fmt):
    """Elements that share one scale byte (0: the format has none)."""
    return {FMT_FP4_E2M1_MX: 32, FMT_FP4_E2M1_MX_BYTES: 32, FMT_FP4_E2M1_NV: 16}.get(fmt, 0)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, what):
    if status != OK:
        raise ZcError(status, what)


def compress_bound(n_elems, p):
    return int(lib().zc_compress_bound(n_elems, C.byref(p)))


def workspace_bytes(n_elems_list, p):
    arr = (C.c_uint64 * len(n_elems_list))(*n_elems_list)
    return int(lib().zc_workspace_bytes(arr, len(n_elems_list), C.byref(p)))


def build_code(hist, limit):
    """Host-only: (lengths, codes) of the library's code construction for a histogram."""
    n = len(hist)
    h = (C.c_uint64 * n)(*[int(v) for v in hist])
    ln = (C.c_uint8 * n)()
    cd = (C.c_uint16 * n)()
    _check(lib().zc_build_code(h, n, limit, ln, cd), "zc_build_code")
    return list(ln), list(cd)


def _workspace(n_elems_list, p, device):
    need = workspace_bytes(n_elems_list, p)
    if need == 0:
        raise ZcError(ERR_INVALID_ARG, "zc_workspace_bytes")
    return torch.empty(need, dtype=torch.uint8, device=device)


def compress(src, n_elems, p, xor_base=None, scales=None, dst=None, ws=None):
    """src/xor_base/scales/dst/ws: CUDA tensors (any dtype, contiguous).  Returns (container view, Info)."""
    dev = src.device
    if dst is None:
        dst = torch.empty(max(compress_bound(n_elems, p), 16), dtype=torch.uint8, device=dev)
    if ws is None:
        ws = _workspace([n_elems], p, dev)
    size = C.c_uint64(0)
    info = Info()
    st = lib().zc_compress(_ptr(src), n_elems, C.byref(p), _ptr(xor_base), _ptr(scales), _ptr(dst), dst.numel() * dst.element_size(),
                           C.byref(size), C.byref(info), _ptr(ws), ws.numel(), _stream())
    _check(st, "zc_compress")
    return dst.view(torch.uint8).reshape(-1)[:size.value], info


def compress_noalloc(src, n_elems, p, dst, xor_base=None, scales=None):
    """Queue the compression of one tensor into dst (at least compress_bound bytes) without a workspace and
    without any allocation; the container's size is in its header once the stream gets there (read_info)."""
    st = lib().zc_compress_noalloc(_ptr(src), n_elems, C.byref(p), _ptr(xor_base), _ptr(scales), _ptr(dst),
                                   dst.numel() * dst.element_size(), _stream())
    _check(st, "zc_compress_noalloc")


def train_code(src, n_elems, p, xor_base=None, scales=None, ws=None):
    """Static dictionary (an Info whose mode/code_len fields are meaningful) from a representative tensor."""
    if ws is None:
        ws = _workspace([n_elems], p, src.device)
    code = Info()
    st = lib().zc_train_code(_ptr(src), n_elems, C.byref(p), _ptr(xor_base), _ptr(scales), C.byref(code), _ptr(ws), ws.numel(), _stream())
    _check(st, "zc_train_code")
    return code


def code_stale(code, written, slack=0.02):
    """Refresh test for a static dictionary: True when `written` (the Info of a compress_with_code call) is
    larger relative to its raw size than the training tensor was, by more than `slack`."""
    r = lib().zc_code_stale(C.byref(code), C.byref(written), slack)
    if r < 0:
        raise ZcError(ERR_INVALID_ARG, "zc_code_stale")
    return bool(r)


def compress_with_code(src, n_elems, p, code, xor_base=None, scales=None, dst=None, ws=None):
    dev = src.device
    if dst is None:
        dst = torch.empty(max(compress_bound(n_elems, p), 16), dtype=torch.uint8, device=dev)
    if ws is None:
        ws = _workspace([n_elems], p, dev)
    size = C.c_uint64(0)
    info = Info()
    st = lib().zc_compress_with_code(_ptr(src), n_elems, C.byref(p), C.byref(code), _ptr(xor_base), _ptr(scales), _ptr(dst),
                                     dst.numel() * dst.element_size(), C.byref(size), C.byref(info), _ptr(ws), ws.numel(), _stream())
    _check(st, "zc_compress_with_code")
    return dst.view(torch.uint8).reshape(-1)[:size.value], info


def read_info(comp, check_index=False):
    info = Info()
    _check(lib().zc_read_info(_ptr(comp), comp.numel(), 1 if check_index else 0, C.byref(info), _stream()), "zc_read_info")
    return info


def validate_container(host_bytes, check_index=True, container_bytes=None):
    """Host only: validate a container held in host memory (bytes, bytearray or a numpy uint8 array); returns its
    Info.  container_bytes: size of the whole container when host_bytes is only its beginning."""
    buf = (C.c_uint8 * len(host_bytes)).from_buffer_copy(bytes(host_bytes))
    info = Info()
    total = len(host_bytes) if container_bytes is None else container_bytes
    _check(lib().zc_validate_container(buf, len(host_bytes), total, 1 if check_index else 0, C.byref(info)), "zc_validate_container")
    return info


def copy_reference(src, dst, chunk_bytes=0):
    """Queue the library's plain copy kernel (the bandwidth yardstick) from src to dst, both CUDA tensors of equal size;
    chunk_bytes != 0: one wavefront per chunk, as the 64-lane codec kernels walk through memory."""
    _check(lib().zc_copy_reference(_ptr(src), _ptr(dst), src.numel() * src.element_size(), chunk_bytes, _stream()), "zc_copy_reference")


def release_host_buffers():
    _check(lib().zc_release_host_buffers(), "zc_release_host_buffers")


def decompress(comp, info=None, out=None, scales_out=None, xor_base=None, read_header_in_call=False):
    """Returns (elements as uint8 tensor, scales or None).  read_header_in_call: pass no Info to the library, which
    then reads the header itself (a blocking copy) before it queues the decode."""
    if info is None:
        info = read_info(comp)
    raw = (info.n_elems * elem_bits(info.format) + 7) // 8
    if out is None:
        out = torch.empty(raw, dtype=torch.uint8, device=comp.device)
    if info.n_fields == 3 and scales_out is None:
        scales_out = torch.empty(max(info.n_elems // scale_block(info.format), 1), dtype=torch.uint8, device=comp.device)
    st = lib().zc_decompress(_ptr(comp), comp.numel(), None if read_header_in_call else C.byref(info), _ptr(out),
                             out.numel() * out.element_size(), _ptr(scales_out), _ptr(xor_base), _stream())
    _check(st, "zc_decompress")
    return out, scales_out


def decompress_chunks(comp, info, ids, out=None, scales_out=None, xor_base=None):
    """ids: int32/uint32 CUDA tensor of chunk ids; chunk ids[i] lands at out[i*chunk_bytes:]."""
    n = ids.numel()
    if out is None:
        out = torch.empty(n * info.chunk_bytes, dtype=torch.uint8, device=comp.device)
    if info.n_fields == 3 and scales_out is None:
        scales_out = torch.empty(max(n * info.chunk_bytes * 2 // scale_block(info.format), 1), dtype=torch.uint8, device=comp.device)
    st = lib().zc_decompress_chunks(_ptr(comp), comp.numel(), C.byref(info), _ptr(ids), n, _ptr(out),
                                    out.numel() * out.element_size(), _ptr(scales_out), _ptr(xor_base), _stream())
    _check(st, "zc_decompress_chunks")
    return out, scales_out


def stats(src, n_elems, p, xor_base=None, scales=None, ws=None):
    if ws is None:
        ws = _workspace([n_elems], p, src.device)
    out = StatsOut()
    st = lib().zc_stats(_ptr(src), n_elems, C.byref(p), _ptr(xor_base), _ptr(scales), C.byref(out), _ptr(ws), ws.numel(), _stream())
    _check(st, "zc_stats")
    return out


class Batch:
    """A set of tensors compressed / decompressed with one launch sequence.

    Holds the host array of zc_tensor descriptors plus the torch tensors that own the
    device memory, so that repeated calls allocate nothing."""

    def __init__(self, srcs, n_elems, p, xor_bases=None, scales=None):
        self.p = p
        self.n = len(srcs)
        self.srcs, self.bases, self.scales = list(srcs), xor_bases, scales
        dev = srcs[0].device
        self.arr = (Tensor * self.n)()
        self.caps = [max(compress_bound(n, p), 16) for n in n_elems]
        # one arena for all containers, each slot 256-byte aligned
        offs, total = [], 0
        for c in self.caps:
            offs.append(total)
            total += (c + 255) // 256 * 256
        self.arena = torch.empty(total, dtype=torch.uint8, device=dev)
        self.comp = [self.arena[o:o + c] for o, c in zip(offs, self.caps)]
        self.ws = _workspace(list(n_elems), p, dev)
        # the decode plan lives in a workspace of its own: compress() rewrites self.ws
        self.ws_plan = torch.empty(self.ws.numel(), dtype=torch.uint8, device=dev)
        for i in range(self.n):
            a = self.arr[i]
            a.d_src = srcs[i].data_ptr()
            a.d_xor_base = xor_bases[i].data_ptr() if xor_bases else None
            a.d_scales = scales[i].data_ptr() if scales else None
            a.n_elems = n_elems[i]
            a.d_comp = self.comp[i].data_ptr()
            a.comp_capacity = self.caps[i]
        self.out = None
        self.scales_out = None

    def compress(self, code=None):
        """code: a static dictionary from train_code() (then no histogram pass), or None."""
        if code is None:
            _check(lib().zc_compress_batch(self.arr, self.n, C.byref(self.p), _ptr(self.ws), self.ws.numel(), _stream()), "zc_compress_batch")
        else:
            _check(lib().zc_compress_batch_with_code(self.arr, self.n, C.byref(self.p), C.byref(code), _ptr(self.ws), self.ws.numel(), _stream()),
                   "zc_compress_batch_with_code")
        return [int(self.arr[i].out_bytes) for i in range(self.n)]

    def compress_async(self, code=None):
        """Queue the compression (with a static dictionary if one is given, else with codes built on the device)
        and return without waiting; call refresh_info() (which waits) before container(), decompress() or
        plan_decompress()."""
        if code is None:
            _check(lib().zc_compress_batch_async(self.arr, self.n, C.byref(self.p), _ptr(self.ws), self.ws.numel(), _stream()),
                   "zc_compress_batch_async")
        else:
            _check(lib().zc_compress_batch_with_code_async(self.arr, self.n, C.byref(self.p), C.byref(code), _ptr(self.ws), self.ws.numel(), _stream()),
                   "zc_compress_batch_with_code_async")

    def refresh_info(self):
        """Read every container's header back (blocking) after compress_async()."""
        for i in range(self.n):
            info = read_info(self.comp[i])
            self.arr[i].info = info
            self.arr[i].out_bytes = info.total_bytes
        return [int(self.arr[i].out_bytes) for i in range(self.n)]

    def container(self, i):
        return self.comp[i][:int(self.arr[i].out_bytes)]

    def prepare_outputs(self):
        dev = self.arena.device
        eb = elem_bits(self.p.format)
        self.out = [torch.empty(max((int(self.arr[i].n_elems) * eb + 7) // 8, 16), dtype=torch.uint8, device=dev) for i in range(self.n)]
        if scale_block(self.p.format):
            self.scales_out = [torch.empty(max(int(self.arr[i].n_elems) // scale_block(self.p.format), 16), dtype=torch.uint8, device=dev) for i in range(self.n)]
        for i in range(self.n):
            self.arr[i].d_dst = self.out[i].data_ptr()
            self.arr[i].d_scales_out = self.scales_out[i].data_ptr() if self.scales_out else None

    def set_outputs(self, outs, scales_out=None):
        """Decode into the caller's buffers (one uint8 CUDA tensor per tensor, each large enough) from the next plan on."""
        self.out, self.scales_out = list(outs), scales_out
        for i in range(self.n):
            self.arr[i].d_dst = self.out[i].data_ptr()
            self.arr[i].d_scales_out = scales_out[i].data_ptr() if scales_out else None

    def set_chunk_ids(self, ids):
        """ids: one int32 CUDA tensor of chunk ids per tensor (or None to decode whole tensors again).
        The next plan/decompress decodes only those chunks, densely, into fresh output buffers."""
        dev = self.arena.device
        self.ids = ids
        if ids is None:
            self.out = None
            for i in range(self.n):
                self.arr[i].d_chunk_ids = None
                self.arr[i].n_chunk_ids = 0
            return
        self.out = [torch.empty(max(ids[i].numel() * self.p.chunk_bytes, 16), dtype=torch.uint8, device=dev) for i in range(self.n)]
        for i in range(self.n):
            self.arr[i].d_chunk_ids = ids[i].data_ptr()
            self.arr[i].n_chunk_ids = ids[i].numel()
            self.arr[i].d_dst = self.out[i].data_ptr()

    def decompress(self):
        if self.out is None:
            self.prepare_outputs()
        _check(lib().zc_decompress_batch(self.arr, self.n, _ptr(self.ws), self.ws.numel(), _stream()), "zc_decompress_batch")
        return self.out

    def plan_decompress(self):
        """Queue the upload of descriptors and work lists on the current stream; returns the plan."""
        if self.out is None:
            self.prepare_outputs()
        self.plan = BatchPlan()
        _check(lib().zc_decompress_batch_plan(self.arr, self.n, _ptr(self.ws_plan), self.ws_plan.numel(), C.byref(self.plan), _stream()),
               "zc_decompress_batch_plan")
        return self.plan

    def run_decompress(self):
        """Enqueue the decode kernels on the plan left in the workspace by plan_decompress()."""
        _check(lib().zc_decompress_batch_run(C.byref(self.plan), _ptr(self.ws_plan), _stream()), "zc_decompress_batch_run")
        return self.out
