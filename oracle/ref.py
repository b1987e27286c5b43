"""ctypes access to the CPU oracle (oracle/kvc_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The GPU library never imports or calls anything here.
Arrays are numpy; 16-bit floats travel as uint16 bit patterns.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libkvc_ref.so")

F16, BF16 = 1, 2


def build(force=False):
    """Compile the oracle with gcc; every fp32 operation stays one rounded operation."""
    src = os.path.join(_HERE, "kvc_ref.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", _SO, src, "-lm"])
    return _SO


class Config(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("layers", C.c_int32), ("heads", C.c_int32),
                ("head_dim", C.c_int32), ("bits_k", C.c_int32), ("bits_v", C.c_int32),
                ("group_k", C.c_int32), ("group_v", C.c_int32), ("codec", C.c_int32),
                ("transform", C.c_int32), ("anchor_period", C.c_int32),
                ("head_bits_k", C.c_void_p), ("head_bits_v", C.c_void_p)]


class Layout(C.Structure):
    _fields_ = [("stride_layer", C.c_int64), ("stride_head", C.c_int64),
                ("stride_token", C.c_int64), ("stride_block", C.c_int64),
                ("block_tokens", C.c_int32), ("block_table", C.POINTER(C.c_int32))]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        L = _lib
        L.ref_f16_to_f32.restype = C.c_float
        L.ref_f16_to_f32.argtypes = [C.c_uint16]
        L.ref_f32_to_f16.restype = C.c_uint16
        L.ref_f32_to_f16.argtypes = [C.c_float]
        L.ref_bf16_to_f32.restype = C.c_float
        L.ref_bf16_to_f32.argtypes = [C.c_uint16]
        L.ref_f32_to_bf16.restype = C.c_uint16
        L.ref_f32_to_bf16.argtypes = [C.c_float]
        L.ref_dequantize.restype = C.c_uint16
        L.ref_dequantize.argtypes = [C.c_int, C.c_uint16, C.c_uint16, C.c_int]
        L.ref_huff_encode_chunk.restype = C.c_int64
        L.ref_encode_chunk_at.restype = C.c_int64
        L.ref_chunks_per_head.restype = C.c_int64
        L.ref_chunks_per_head.argtypes = [C.c_int64]
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def config(dtype=F16, layers=1, heads=1, head_dim=128, bits_k=4, bits_v=4, group_k=32, group_v=32,
           codec=0, transform=0, head_bits_k=None, head_bits_v=None, anchor_period=0):
    """transform 2 (delta against an anchor token) needs anchor_period.  head_bits_k / head_bits_v: optional uint8 arrays of layers*heads widths (the uniform width of
    that tensor is then 0); the arrays are kept alive by the returned object."""
    keep = []
    ptrs = []
    for t in (head_bits_k, head_bits_v):
        if t is None:
            ptrs.append(None)
        else:
            a = np.ascontiguousarray(t, dtype=np.uint8).reshape(-1)
            assert a.size == layers * heads
            keep.append(a)
            ptrs.append(a.ctypes.data)
    cfg = Config(dtype, layers, heads, head_dim, 0 if head_bits_k is not None else bits_k,
                 0 if head_bits_v is not None else bits_v, group_k, group_v, codec, transform, anchor_period,
                 ptrs[0], ptrs[1])
    cfg._keep = keep
    return cfg


def contiguous_layout(heads, tokens, head_dim):
    """Element strides of one tensor stored [layer][kv][head][token][dim]; K and V are passed
    as separate base pointers half a layer apart."""
    return Layout(2 * heads * tokens * head_dim, tokens * head_dim, head_dim, 0, 0, None)


def paged_layout(heads, head_dim, block_tokens, num_phys_blocks, table):
    """[layer][kv][phys_block][block_tokens][head][dim] with a block table shared by all layers."""
    table = np.ascontiguousarray(table, dtype=np.int32)
    lay = Layout(2 * num_phys_blocks * block_tokens * heads * head_dim, head_dim,
                 heads * head_dim, block_tokens * heads * head_dim, block_tokens,
                 table.ctypes.data_as(C.POINTER(C.c_int32)))
    lay._keep = table
    return lay


# ---- scalar and group level -------------------------------------------------------------

def f16_to_f32(h):
    return lib().ref_f16_to_f32(int(h))


def f32_to_f16(f):
    return lib().ref_f32_to_f16(float(np.float32(f)))


def bf16_to_f32(h):
    return lib().ref_bf16_to_f32(int(h))


def f32_to_bf16(f):
    return lib().ref_f32_to_bf16(float(np.float32(f)))


def group_meta(x, bits):
    x = np.ascontiguousarray(x, dtype=np.float32)
    s, z = C.c_uint16(), C.c_uint16()
    lib().ref_group_meta(_p(x), C.c_int(x.size), C.c_int(bits), C.byref(s), C.byref(z))
    return s.value, z.value


def group_quantize(x, bits, scale_h, zero_h):
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.size, dtype=np.uint8)
    lib().ref_group_quantize(_p(x), C.c_int(x.size), C.c_int(bits), C.c_uint16(scale_h),
                             C.c_uint16(zero_h), _p(q))
    return q


def dequantize(q, scale_h, zero_h, dtype=F16):
    return lib().ref_dequantize(int(q), int(scale_h), int(zero_h), int(dtype))


def pack(q, bits):
    q = np.ascontiguousarray(q, dtype=np.uint8)
    out = np.empty(q.size * bits // 8, dtype=np.uint8)
    lib().ref_pack(_p(q), C.c_int64(q.size), C.c_int(bits), _p(out))
    return out


def unpack(buf, n, bits):
    buf = np.ascontiguousarray(buf, dtype=np.uint8)
    q = np.empty(n, dtype=np.uint8)
    lib().ref_unpack(_p(buf), C.c_int64(n), C.c_int(bits), _p(q))
    return q


def hadamard_row(row_u16, dtype=F16, inverse=False):
    """ref_hadamard_row on one row of 16-bit patterns (length = a power of two)."""
    row = np.ascontiguousarray(row_u16, dtype=np.uint16)
    out = np.empty_like(row)
    lib().ref_hadamard_row(_p(row), _p(out), C.c_int(row.size), C.c_int(dtype), C.c_int(1 if inverse else 0))
    return out


def delta_row(row_u16, anchor_u16, dtype=F16, inverse=False):
    """ref_delta_row: row - anchor (or row + anchor), rounded to the type, on 16-bit patterns."""
    row = np.ascontiguousarray(row_u16, dtype=np.uint16)
    anchor = np.ascontiguousarray(anchor_u16, dtype=np.uint16)
    assert row.size == anchor.size
    out = np.empty_like(row)
    lib().ref_delta_row(_p(row), _p(anchor), _p(out), C.c_int(row.size), C.c_int(dtype),
                        C.c_int(1 if inverse else 0))
    return out


def huff_lengths(hist):
    hist = np.ascontiguousarray(hist, dtype=np.uint32)
    assert hist.size == 256
    out = np.empty(256, dtype=np.uint8)
    lib().ref_huff_lengths(_p(hist), _p(out))
    return out


def huff_codes(lengths):
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    out = np.zeros(256, dtype=np.uint16)
    lib().ref_huff_codes(_p(lengths), _p(out))
    return out


def huff_encode_chunk(raw, rows, row_bytes, lengths):
    raw = np.ascontiguousarray(raw, dtype=np.uint8)
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    body = np.zeros(rows * row_bytes + 512, dtype=np.uint8)
    n = lib().ref_huff_encode_chunk(_p(raw), C.c_int(rows), C.c_int(row_bytes), _p(lengths), _p(body))
    return body[:n].copy()


def huff_decode_chunk(body, rows, row_bytes, lengths):
    body = np.ascontiguousarray(body, dtype=np.uint8)
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    raw = np.zeros(rows * row_bytes, dtype=np.uint8)
    rc = lib().ref_huff_decode_chunk(_p(body), C.c_int64(body.size), C.c_int(rows),
                                     C.c_int(row_bytes), _p(lengths), _p(raw))
    return rc, raw


# ---- tensor level -----------------------------------------------------------------------

def payload_size(cfg, tokens):
    n, ex = C.c_uint64(), C.c_int()
    rc = lib().ref_payload_size(C.byref(cfg), C.c_int64(tokens), C.byref(n), C.byref(ex))
    if rc:
        raise ValueError("ref_payload_size: %d" % rc)
    return n.value, bool(ex.value)


def chunks_per_head(tokens):
    return lib().ref_chunks_per_head(tokens)


def compress_head(cfg, is_v, src, lay, tokens, l, h):
    """src: uint16 array holding the tensor; returns (packed codes, meta pairs as uint16)."""
    bits = cfg.bits_v if is_v else cfg.bits_k
    D = cfg.head_dim
    codes = np.zeros(tokens * D * bits // 8, dtype=np.uint8)
    if bits == 16:
        pairs = 0
    elif is_v:
        pairs = tokens * (D // cfg.group_v)
    else:
        pairs = -(-tokens // cfg.group_k) * D
    meta = np.zeros(2 * pairs, dtype=np.uint16)
    rc = lib().ref_compress_head(C.byref(cfg), C.c_int(is_v), _p(src), C.byref(lay),
                                 C.c_int64(tokens), C.c_int(l), C.c_int(h), _p(codes), _p(meta))
    if rc:
        raise ValueError("ref_compress_head: %d" % rc)
    return codes, meta


def decompress_head(cfg, is_v, codes, meta, tokens, l, h, dst, lay, anchors=None):
    """anchors: this head's anchor rows (uint16, [runs][head_dim]) when cfg.transform == 2."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    meta = np.ascontiguousarray(meta, dtype=np.uint16)
    if anchors is not None:
        anchors = np.ascontiguousarray(anchors, dtype=np.uint16)
    rc = lib().ref_decompress_head(C.byref(cfg), C.c_int(is_v), _p(codes), _p(meta),
                                   _p(anchors) if anchors is not None else None, C.c_int64(tokens), C.c_int(l), C.c_int(h), _p(dst), C.byref(lay))
    if rc:
        raise ValueError("ref_decompress_head: %d" % rc)


def huff_tables(cfg, k, v, lay, tokens):
    lk = np.zeros(256, dtype=np.uint8)
    lv = np.zeros(256, dtype=np.uint8)
    rc = lib().ref_huff_tables(C.byref(cfg), _p(k), _p(v), C.byref(lay), C.c_int64(tokens),
                               _p(lk), _p(lv))
    if rc:
        raise ValueError("ref_huff_tables: %d" % rc)
    return lk, lv


def encode_chunk_at(cfg, is_v, src, lay, tokens, chunk, lengths):
    bits = cfg.bits_v if is_v else cfg.bits_k
    body = np.zeros(128 * cfg.head_dim * bits // 8 + 512, dtype=np.uint8)
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    n = lib().ref_encode_chunk_at(C.byref(cfg), C.c_int(is_v), _p(src), C.byref(lay),
                                  C.c_int64(tokens), C.c_int64(chunk), _p(lengths), _p(body))
    if n < 0:
        raise ValueError("ref_encode_chunk_at: %d" % n)
    return body[:n].copy()


def compress(cfg, k, v, lay, tokens):
    """k, v: uint16 numpy views whose element 0 is the tensor base. Returns payload bytes."""
    cap, _ = payload_size(cfg, tokens)
    payload = np.zeros(cap, dtype=np.uint8)
    out = C.c_uint64()
    rc = lib().ref_compress(C.byref(cfg), _p(k), _p(v), C.byref(lay), C.c_int64(tokens),
                            _p(payload), C.c_uint64(cap), C.byref(out))
    if rc:
        raise ValueError("ref_compress: %d" % rc)
    return payload[:out.value].copy()


def decompress(payload, k_out, v_out, lay, expect=None):
    payload = np.ascontiguousarray(payload, dtype=np.uint8)
    rc = lib().ref_decompress(_p(payload), C.c_uint64(payload.size), _p(k_out), _p(v_out),
                              C.byref(lay), C.byref(expect) if expect is not None else None)
    return rc


def inspect(header):
    header = np.ascontiguousarray(header[:128], dtype=np.uint8)
    cfg = Config()
    tokens, total = C.c_int64(), C.c_uint64()
    sec = (C.c_uint64 * 10)()
    rc = lib().ref_inspect(_p(header), C.byref(cfg), C.byref(tokens), C.byref(total), sec)
    return rc, cfg, tokens.value, total.value, list(sec)
