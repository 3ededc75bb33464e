"""ctypes binding of the CPU oracle (oracle/zc_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU
baseline may import this module; the product package never does.  Nothing here
computes anything: it marshals numpy arrays into the C functions.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zc_oracle.c")
_LIB = os.path.join(_HERE, "libzc_oracle.so")

BF16, FP8_E4M3, FP4_E2M1_MX, FP8_E4M3_BYTES, FP4_E2M1_MX_BYTES, FP4_E2M1_NV, FP8_E5M2 = 1, 2, 3, 4, 5, 6, 7
MODE_EMPTY, MODE_HUFF, MODE_RAW, MODE_CONST = 0, 1, 2, 3
POLICY_HUFF_ALL, POLICY_AUTO = 0, 1
OK, ERR_ARG, ERR_UNSUPPORTED, ERR_SMALL, ERR_CORRUPT = 0, 1, 2, 3, 4


def build(force=False):
    """Compile the oracle with gcc (plain C99, -O2, single thread)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Params(C.Structure):
    _fields_ = [("format", C.c_uint32), ("chunk_bytes", C.c_uint32), ("max_code_len", C.c_uint32 * 3),
                ("streams_per_chunk", C.c_uint32), ("policy", C.c_uint32), ("payload_order", C.c_uint32)]


class FieldStats(C.Structure):
    _fields_ = [("alphabet", C.c_uint32), ("distinct", C.c_uint32), ("mode", C.c_uint32), ("max_len", C.c_uint32),
                ("n_symbols", C.c_uint64), ("hist", C.c_uint64 * 256), ("code_len", C.c_uint8 * 256),
                ("entropy_bits", C.c_double), ("mean_code_len", C.c_double), ("payload_bits", C.c_uint64),
                ("stream_bytes", C.c_uint64), ("ratio_payload", C.c_double)]


class StatsOut(C.Structure):
    _fields_ = [("n_fields", C.c_uint32), ("pad", C.c_uint32), ("raw_bytes", C.c_uint64),
                ("container_bytes", C.c_uint64), ("ratio_payload_total", C.c_double),
                ("ratio_container_total", C.c_double), ("field", FieldStats * 3)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        u8p, u64 = C.c_void_p, C.c_uint64
        _lib.zco_num_fields.restype = C.c_int
        _lib.zco_sym_bits.restype = C.c_int
        for name in ("zco_exponent_of", "zco_signmant_of"):
            getattr(_lib, name).restype = C.c_uint
            getattr(_lib, name).argtypes = [C.c_int, C.c_uint]
        _lib.zco_rebuild.restype = C.c_uint
        _lib.zco_rebuild.argtypes = [C.c_int, C.c_uint, C.c_uint]
        _lib.zco_split.argtypes = [C.c_int, u8p, u8p, u64, u8p, u8p]
        _lib.zco_join.argtypes = [C.c_int, u8p, u8p, u8p, u64, u8p]
        _lib.zco_histogram.argtypes = [u8p, u64, u8p]
        _lib.zco_group_values.argtypes = [C.c_int, C.c_int, u8p, u64, u8p]
        _lib.zco_ungroup_symbols.argtypes = [C.c_int, C.c_int, u8p, u64, u8p]
        _lib.zco_code_lengths.restype = C.c_int
        _lib.zco_code_lengths.argtypes = [u8p, C.c_int, C.c_int, u8p]
        _lib.zco_canonical_codes.argtypes = [u8p, C.c_int, u8p]
        _lib.zco_stream_bound.restype = u64
        _lib.zco_stream_bound.argtypes = [u64, C.c_int, C.c_int]
        _lib.zco_encode_stream.restype = u64
        _lib.zco_encode_stream.argtypes = [u8p, u64, u8p, u8p, C.c_int, C.c_int, C.c_int, u8p]
        _lib.zco_decode_stream.restype = u64
        _lib.zco_decode_stream.argtypes = [u8p, u64, u64, u8p, C.c_int, C.c_int, C.c_int, u8p]
        _lib.zco_compress_bound.restype = u64
        _lib.zco_compress_bound.argtypes = [u64, C.POINTER(Params)]
        _lib.zco_compress.restype = C.c_int
        _lib.zco_compress.argtypes = [u8p, u64, C.POINTER(Params), u8p, u8p, u8p, u64, C.POINTER(u64)]
        _lib.zco_compress_with_code.restype = C.c_int
        _lib.zco_compress_with_code.argtypes = [u8p, u64, C.POINTER(Params), u8p, u8p, u8p, u8p, u8p, u64, C.POINTER(u64)]
        _lib.zco_train_code.restype = C.c_int
        _lib.zco_train_code.argtypes = [u8p, u64, C.POINTER(Params), u8p, u8p, u8p, u8p]
        _lib.zco_decompress.restype = C.c_int
        _lib.zco_decompress.argtypes = [u8p, u64, u8p, u8p, u64, u8p]
        _lib.zco_decompress_chunk.restype = C.c_int
        _lib.zco_decompress_chunk.argtypes = [u8p, u64, u64, u8p, u8p, u64, u8p]
        _lib.zco_stats.restype = C.c_int
        _lib.zco_stats.argtypes = [u8p, u64, C.POINTER(Params), u8p, u8p, C.POINTER(StatsOut)]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _bytes(a):
    """Any array viewed as contiguous bytes (None stays None)."""
    if a is None:
        return None
    return np.ascontiguousarray(a).view(np.uint8).reshape(-1)


def params(fmt, chunk_bytes, max_code_len=(0, 0, 0), streams=0, policy=POLICY_HUFF_ALL, payload_order=0):
    p = Params()
    p.format, p.chunk_bytes, p.streams_per_chunk, p.policy, p.payload_order = fmt, chunk_bytes, streams, policy, payload_order
    for i in range(3):
        p.max_code_len[i] = max_code_len[i]
    return p


def elem_bits(fmt):
    return {BF16: 16, FP8_E4M3: 8, FP4_E2M1_MX: 4, FP8_E4M3_BYTES: 8, FP4_E2M1_MX_BYTES: 4, FP4_E2M1_NV: 4, FP8_E5M2: 8}[fmt]


def group_of(fmt):
    """Field values per coded symbol."""
    return {FP8_E4M3_BYTES: 2, FP4_E2M1_MX_BYTES: 4}.get(fmt, 1)


def group_values(fmt, f, values, n_elems):
    """Coded symbols of field f from its per-element field values (byte-grouped formats)."""
    out = np.zeros((n_elems + group_of(fmt) - 1) // group_of(fmt), np.uint8)
    lib().zco_group_values(fmt, f, _p(np.ascontiguousarray(values, np.uint8)), n_elems, _p(out))
    return out


def ungroup_symbols(fmt, f, syms, n_elems):
    out = np.zeros(n_elems, np.uint8)
    lib().zco_ungroup_symbols(fmt, f, _p(np.ascontiguousarray(syms, np.uint8)), n_elems, _p(out))
    return out


def split(fmt, src, n_elems, base=None):
    src, base = _bytes(src), _bytes(base)
    e = np.empty(n_elems, np.uint8)
    m = np.empty(n_elems, np.uint8)
    lib().zco_split(fmt, _p(src), _p(base), n_elems, _p(e), _p(m))
    return e, m


def join(fmt, e, m, base=None):
    n = len(e)
    out = np.zeros((n * elem_bits(fmt) + 7) // 8, np.uint8)
    lib().zco_join(fmt, _p(np.ascontiguousarray(e)), _p(np.ascontiguousarray(m)), _p(_bytes(base)), n, _p(out))
    return out


def histogram(syms):
    syms = np.ascontiguousarray(syms, np.uint8)
    h = np.zeros(256, np.uint64)
    lib().zco_histogram(_p(syms), len(syms), _p(h))
    return h


def code_lengths(hist, limit):
    """hist: sequence of counts (its length is the alphabet). Returns uint8 lengths."""
    h = np.zeros(256, np.uint64)
    h[:len(hist)] = np.asarray(hist, np.uint64)
    out = np.zeros(256, np.uint8)
    rc = lib().zco_code_lengths(_p(h), len(hist), limit, _p(out))
    if rc:
        raise ValueError("limit too small for the alphabet")
    return out[:len(hist)].copy()


def canonical_codes(lengths):
    ln = np.zeros(256, np.uint8)
    ln[:len(lengths)] = lengths
    out = np.zeros(256, np.uint16)
    lib().zco_canonical_codes(_p(ln), len(lengths), _p(out))
    return out[:len(lengths)].copy()


def encode_stream(syms, lengths, G, S):
    syms = np.ascontiguousarray(syms, np.uint8)
    ln = np.zeros(256, np.uint8)
    ln[:len(lengths)] = lengths
    codes = np.zeros(256, np.uint16)
    codes[:len(lengths)] = canonical_codes(lengths)
    lmax = int(ln.max())
    out = np.zeros(int(lib().zco_stream_bound(len(syms), S, lmax)), np.uint8)
    n = lib().zco_encode_stream(_p(syms), len(syms), _p(ln), _p(codes), lmax, G, S, _p(out))
    return out[:n].copy()


def decode_stream(stream, n, lengths, G, S):
    """Returns (symbols, bytes consumed); consumed == 0 flags a malformed stream."""
    stream = np.ascontiguousarray(stream, np.uint8)
    ln = np.zeros(256, np.uint8)
    ln[:len(lengths)] = lengths
    out = np.zeros(n, np.uint8)
    used = lib().zco_decode_stream(_p(stream), len(stream), n, _p(ln), len(lengths), G, S, _p(out))
    return out, int(used)


def compress_bound(n_elems, p):
    return int(lib().zco_compress_bound(n_elems, C.byref(p)))


def compress(src, n_elems, p, xor_base=None, scales=None):
    """Returns the container as a uint8 array; raises on a non-zero status."""
    src, xor_base, scales = _bytes(src), _bytes(xor_base), _bytes(scales)
    cap = compress_bound(n_elems, p)
    if cap == 0:
        raise ValueError("invalid parameters")
    dst = np.zeros(cap, np.uint8)
    size = C.c_uint64(0)
    rc = lib().zco_compress(_p(src), n_elems, C.byref(p), _p(xor_base), _p(scales), _p(dst), cap, C.byref(size))
    if rc:
        raise ValueError("zco_compress status %d" % rc)
    return dst[:size.value].copy()


def train_code(src, n_elems, p, xor_base=None, scales=None):
    """Static dictionary from representative data: (lengths uint8[3,256], modes uint8[3])."""
    ln = np.zeros((3, 256), np.uint8)
    md = np.zeros(3, np.uint8)
    rc = lib().zco_train_code(_p(_bytes(src)), n_elems, C.byref(p), _p(_bytes(xor_base)), _p(_bytes(scales)), _p(ln), _p(md))
    if rc:
        raise ValueError("zco_train_code status %d" % rc)
    return ln, md


def compress_with_code(src, n_elems, p, lengths, modes, xor_base=None, scales=None):
    src, xor_base, scales = _bytes(src), _bytes(xor_base), _bytes(scales)
    cap = compress_bound(n_elems, p)
    dst = np.zeros(cap, np.uint8)
    size = C.c_uint64(0)
    ln = np.ascontiguousarray(lengths, np.uint8)
    md = np.ascontiguousarray(modes, np.uint8)
    rc = lib().zco_compress_with_code(_p(src), n_elems, C.byref(p), _p(xor_base), _p(scales), _p(ln), _p(md), _p(dst), cap, C.byref(size))
    if rc:
        raise ValueError("zco_compress_with_code status %d" % rc)
    return dst[:size.value].copy()


def decompress(comp, out_bytes, xor_base=None, n_scales=0):
    """Returns (status, element bytes, scale bytes or None)."""
    comp = _bytes(comp)
    dst = np.zeros(out_bytes, np.uint8)
    sc = np.zeros(n_scales, np.uint8) if n_scales else None
    rc = lib().zco_decompress(_p(comp), len(comp), _p(_bytes(xor_base)), _p(dst), out_bytes, _p(sc))
    return rc, dst, sc


def decompress_chunk(comp, chunk, chunk_bytes, xor_base_chunk=None, n_scales=0):
    comp = _bytes(comp)
    dst = np.zeros(chunk_bytes, np.uint8)
    sc = np.zeros(n_scales, np.uint8) if n_scales else None
    rc = lib().zco_decompress_chunk(_p(comp), len(comp), chunk, _p(_bytes(xor_base_chunk)), _p(dst), chunk_bytes, _p(sc))
    return rc, dst, sc


def stats(src, n_elems, p, xor_base=None, scales=None):
    out = StatsOut()
    rc = lib().zco_stats(_p(_bytes(src)), n_elems, C.byref(p), _p(_bytes(xor_base)), _p(_bytes(scales)), C.byref(out))
    if rc:
        raise ValueError("zco_stats status %d" % rc)
    return out
