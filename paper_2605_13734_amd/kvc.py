"""Thin ctypes binding of libkvc (include/kvc.h): argument marshalling only.

Every step of the path runs in the HIP kernels of the library; PyTorch appears here only as
the owner of device memory and streams.  There is no CPU fallback: `load()` raises if the
library has not been built (python __graft_entry__.py, or build.py in this directory).
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvc.so")

F16, BF16 = 1, 2
CODEC_NONE, CODEC_HUFF8 = 0, 1
OK = 0
DEV_BAD_BLOCK, DEV_BAD_HEADER, DEV_BAD_CHUNK, DEV_BAD_TABLE, DEV_SCAN_TIMEOUT = 1, 2, 4, 8, 16

SYMBOLS = ["kvc_plan", "kvc_plan_free", "kvc_payload_size", "kvc_workspace_size", "kvc_compress",
           "kvc_decompress", "kvc_payload_inspect", "kvc_check_block_table", "kvc_status_string",
           "kvc_trace", "kvc_selftest", "kvc_table_bytes", "kvc_workspace_init", "kvc_compress_static", "kvc_stream_probe", "kvc_profile_throughput", "kvc_benefit_threshold", "kvc_policy_build",
           "kvc_policy_lookup"]


class Strategy(C.Structure):
    _fields_ = [("bits_k", C.c_uint8), ("bits_v", C.c_uint8), ("group_k", C.c_uint16),
                ("group_v", C.c_uint16), ("codec", C.c_uint8), ("transform", C.c_uint8),
                ("anchor_period", C.c_uint16), ("head_bits_k", C.c_void_p), ("head_bits_v", C.c_void_p)]


class Profile(C.Structure):
    _fields_ = [("cr", C.c_double), ("s_enc", C.c_double), ("s_dec", C.c_double)]


class PolicySegment(C.Structure):
    _fields_ = [("x_from", C.c_double), ("profile", C.c_int32)]


class Model(C.Structure):
    _fields_ = [("dtype", C.c_uint8), ("layers", C.c_int32), ("kv_heads", C.c_int32),
                ("head_dim", C.c_int32)]


class Request(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("tokens", C.c_int64),
                ("stride_layer", C.c_int64), ("stride_head", C.c_int64),
                ("stride_token", C.c_int64), ("stride_block", C.c_int64),
                ("block_table", C.c_void_p), ("block_tokens", C.c_int32),
                ("num_phys_blocks", C.c_int32)]


class KvcError(RuntimeError):
    def __init__(self, where, status):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, status_string(status), status))


_lib = None


def load():
    """Load libkvc.so; fails loudly when it is missing (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libkvc.so is not built: run `python __graft_entry__.py` "
                               "(hipcc --offload-arch=gfx950) first; there is no CPU fallback")
        # PyTorch ships its own HIP runtime under the same soname; it has to be in the process
        # first so that libkvc binds to the runtime that owns torch's streams and memory.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.kvc_plan.argtypes = [C.POINTER(Model), C.POINTER(Strategy), C.c_int64, C.c_int32,
                               C.POINTER(C.c_void_p)]
        L.kvc_plan_free.argtypes = [C.c_void_p]
        L.kvc_plan_free.restype = None
        L.kvc_payload_size.argtypes = [C.c_void_p, C.c_int64, C.POINTER(C.c_uint64), C.POINTER(C.c_int)]
        L.kvc_workspace_size.argtypes = [C.c_void_p]
        L.kvc_workspace_size.restype = C.c_size_t
        L.kvc_compress.argtypes = [C.c_void_p, C.POINTER(Request), C.c_int32, C.c_void_p,
                                   C.POINTER(C.c_uint64), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvc_compress_static.argtypes = [C.c_void_p, C.POINTER(Request), C.c_int32, C.c_void_p,
                                          C.POINTER(C.c_uint64), C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvc_decompress.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(Request),
                                     C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvc_payload_inspect.argtypes = [C.c_void_p, C.POINTER(Model), C.POINTER(Strategy),
                                          C.POINTER(C.c_int64), C.POINTER(C.c_uint64),
                                          C.POINTER(C.c_uint64)]
        L.kvc_check_block_table.argtypes = [C.c_void_p, C.c_int64, C.c_int32]
        L.kvc_trace.argtypes = [C.c_void_p, C.c_void_p, C.c_int32]
        L.kvc_table_bytes.argtypes = [C.c_void_p]
        L.kvc_table_bytes.restype = C.c_size_t
        L.kvc_workspace_init.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvc_stream_probe.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]
        L.kvc_selftest.argtypes = [C.c_void_p, C.c_void_p]
        L.kvc_profile_throughput.argtypes = [C.POINTER(Profile)]
        L.kvc_profile_throughput.restype = C.c_double
        L.kvc_benefit_threshold.argtypes = [C.POINTER(Profile)]
        L.kvc_benefit_threshold.restype = C.c_double
        L.kvc_policy_build.argtypes = [C.POINTER(Profile), C.c_int32, C.POINTER(PolicySegment), C.c_int32,
                                       C.POINTER(C.c_int32)]
        L.kvc_policy_lookup.argtypes = [C.POINTER(PolicySegment), C.c_int32, C.c_double, C.POINTER(C.c_int32),
                                        C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.kvc_status_string.argtypes = [C.c_int]
        L.kvc_status_string.restype = C.c_char_p
        _lib = L
    return _lib


def status_string(status):
    return load().kvc_status_string(int(status)).decode()


class Plan:
    """kvc_plan / kvc_plan_free, kvc_payload_size, kvc_workspace_size."""

    def __init__(self, dtype, layers, kv_heads, head_dim=128, bits_k=4, bits_v=4, group_k=32,
                 group_v=32, codec=0, max_tokens=0, max_batch=1, transform=0, head_bits_k=None, head_bits_v=None,
                 anchor_period=0):
        """transform 2 (difference from an anchor token) needs anchor_period.  head_bits_k / head_bits_v: optional sequences of layers * kv_heads widths (the uniform
        width of that tensor is then passed as 0)."""
        self.model = Model(dtype, layers, kv_heads, head_dim)
        tabs = []
        for t in (head_bits_k, head_bits_v):
            if t is None:
                tabs.append(None)
            else:
                tabs.append((C.c_uint8 * (layers * kv_heads))(*[int(b) for b in t]))
        self._tables = tabs
        self.strategy = Strategy(0 if tabs[0] is not None else bits_k, 0 if tabs[1] is not None else bits_v,
                                 group_k, group_v, codec, transform, anchor_period,
                                 C.cast(tabs[0], C.c_void_p) if tabs[0] is not None else None,
                                 C.cast(tabs[1], C.c_void_p) if tabs[1] is not None else None)
        self.max_tokens, self.max_batch = max_tokens, max_batch
        self._h = C.c_void_p()
        rc = load().kvc_plan(C.byref(self.model), C.byref(self.strategy), max_tokens, max_batch,
                             C.byref(self._h))
        if rc != OK:
            raise KvcError("kvc_plan", rc)

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.kvc_plan_free(self._h)
            self._h = None

    def payload_size(self, tokens):
        n, ex = C.c_uint64(), C.c_int()
        rc = load().kvc_payload_size(self._h, tokens, C.byref(n), C.byref(ex))
        if rc != OK:
            raise KvcError("kvc_payload_size", rc)
        return n.value, bool(ex.value)

    def workspace_size(self):
        return load().kvc_workspace_size(self._h)


def request(k_ptr, v_ptr, tokens, stride_layer, stride_head, stride_token, block_table_ptr=None,
            stride_block=0, block_tokens=0, num_phys_blocks=0):
    return Request(k_ptr, v_ptr, tokens, stride_layer, stride_head, stride_token, stride_block,
                   block_table_ptr, block_tokens, num_phys_blocks)


def contiguous_request(x, tokens=None):
    """x: torch tensor [layers, 2, heads, tokens, dim] (device), element strides taken from it."""
    assert x.dim() == 5 and x.shape[1] == 2 and x.stride(4) == 1
    tokens = x.shape[3] if tokens is None else tokens
    es = x.element_size()
    return request(x.data_ptr(), x.data_ptr() + x.stride(1) * es, tokens, x.stride(0), x.stride(2),
                   x.stride(3))


def paged_request(pool, table, tokens):
    """pool: [layers, 2, phys_blocks, block_tokens, heads, dim]; table: int32 device tensor."""
    assert pool.dim() == 6 and pool.shape[1] == 2 and pool.stride(5) == 1
    es = pool.element_size()
    return request(pool.data_ptr(), pool.data_ptr() + pool.stride(1) * es, tokens, pool.stride(0),
                   pool.stride(4), pool.stride(3), table.data_ptr(), pool.stride(2), pool.shape[3],
                   pool.shape[2])


def _offsets(offsets):
    arr = (C.c_uint64 * len(offsets))(*[int(o) for o in offsets])
    return arr


def compress(plan, requests, payload_ptr, offsets, out_bytes_ptr, status_ptr, workspace_ptr=None,
             stream=None):
    """kvc_compress. requests: list of Request; offsets: n+1 host ints; *_ptr: device addresses."""
    n = len(requests)
    reqs = (Request * n)(*requests)
    rc = load().kvc_compress(plan._h, reqs, n, payload_ptr, _offsets(offsets), out_bytes_ptr,
                             status_ptr, workspace_ptr, stream)
    if rc != OK:
        raise KvcError("kvc_compress", rc)


def compress_static(plan, requests, payload_ptr, offsets, out_bytes_ptr, status_ptr, stream=None):
    """kvc_compress_static: kvc_compress on the library's own static workspace (allocates nothing)."""
    n = len(requests)
    reqs = (Request * n)(*requests)
    rc = load().kvc_compress_static(plan._h, reqs, n, payload_ptr, _offsets(offsets), out_bytes_ptr,
                                    status_ptr, stream)
    if rc != OK:
        raise KvcError("kvc_compress_static", rc)


def decompress(plan, payload_ptr, offsets, requests, status_ptr, workspace_ptr=None, stream=None):
    """kvc_decompress into the tensors named by `requests`."""
    n = len(requests)
    reqs = (Request * n)(*requests)
    rc = load().kvc_decompress(plan._h, payload_ptr, _offsets(offsets), reqs, n, status_ptr,
                               workspace_ptr, stream)
    if rc != OK:
        raise KvcError("kvc_decompress", rc)


def payload_inspect(header_bytes):
    """kvc_payload_inspect on 128 host bytes -> (status, model, strategy, tokens, total, sections)."""
    buf = (C.c_uint8 * 128).from_buffer_copy(bytes(header_bytes[:128]).ljust(128, b"\0"))
    m, s = Model(), Strategy()
    t, total = C.c_int64(), C.c_uint64()
    sec = (C.c_uint64 * 10)()
    rc = load().kvc_payload_inspect(buf, C.byref(m), C.byref(s), C.byref(t), C.byref(total), sec)
    return rc, m, s, t.value, total.value, list(sec)


def trace(plan, events, capacity):
    """kvc_trace: install (or, with None, remove) an array of hipEvent_t handles in a plan."""
    return load().kvc_trace(plan._h, events, capacity)


def workspace_init(plan, workspace_ptr, stream=None):
    """kvc_workspace_init: the device image of a plan's width tables at the start of a workspace."""
    rc = load().kvc_workspace_init(plan._h, workspace_ptr, stream)
    if rc != OK:
        raise KvcError("kvc_workspace_init", rc)


def profile_throughput(cr, s_enc, s_dec):
    return load().kvc_profile_throughput(C.byref(Profile(cr, s_enc, s_dec)))


def benefit_threshold(cr, s_enc, s_dec):
    return load().kvc_benefit_threshold(C.byref(Profile(cr, s_enc, s_dec)))


def policy_build(profiles):
    """kvc_policy_build on a list of (cr, s_enc, s_dec); returns (rc, [(x_from, profile)])."""
    n = len(profiles)
    arr = (Profile * max(n, 1))(*[Profile(*p) for p in profiles])
    table = (PolicySegment * (n + 1))()
    count = C.c_int32(0)
    rc = load().kvc_policy_build(arr, n, table, n + 1, C.byref(count))
    return rc, [(table[i].x_from, table[i].profile) for i in range(count.value if rc == 0 else 0)]


def policy_lookup(table, bandwidth):
    """kvc_policy_lookup on a table returned by policy_build; returns (rc, profile, more_bw, less_bw)."""
    arr = (PolicySegment * len(table))(*[PolicySegment(x, p) for x, p in table])
    a, b, c = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    rc = load().kvc_policy_lookup(arr, len(table), bandwidth, C.byref(a), C.byref(b), C.byref(c))
    return rc, a.value, b.value, c.value


def stream_probe(mode, src_ptr, dst_ptr, rows, payload_row_bytes, stream=None):
    """kvc_stream_probe: bytes moved in the access shape of a tensor pass, without arithmetic."""
    rc = load().kvc_stream_probe(mode, src_ptr, dst_ptr, rows, payload_row_bytes, stream)
    if rc != OK:
        raise KvcError("kvc_stream_probe", rc)


SELFTEST_COUNTS = 8


def selftest(counts_dev_ptr, stream=0):
    """kvc_selftest: counts_dev_ptr is the device address of SELFTEST_COUNTS 64-bit words."""
    return load().kvc_selftest(counts_dev_ptr, stream)


def check_block_table(table_host, num_phys_blocks):
    arr = (C.c_int32 * len(table_host))(*[int(v) for v in table_host])
    return load().kvc_check_block_table(arr, len(table_host), num_phys_blocks)


# ---- device-buffer plumbing (torch owns the memory; nothing here computes) ------------------

class Buffers:
    """Payload, size, status and workspace buffers for a batch, allocated through torch."""

    def __init__(self, plan, token_counts, device="cuda"):
        import torch
        self.plan = plan
        self.tokens = list(token_counts)
        sizes = [plan.payload_size(t)[0] for t in self.tokens]
        self.offsets = [0]
        for s in sizes:
            self.offsets.append(self.offsets[-1] + (s + 255) // 256 * 256)
        self.payload = torch.empty(max(self.offsets[-1], 256), dtype=torch.uint8, device=device)
        self.out_bytes = torch.zeros(len(sizes), dtype=torch.int64, device=device)
        self.status = torch.zeros(len(sizes), dtype=torch.int32, device=device)
        ws = plan.workspace_size()
        self.workspace = torch.empty(max(ws, 256), dtype=torch.uint8, device=device)
        if load().kvc_table_bytes(plan._h):
            workspace_init(plan, self.workspace.data_ptr(), torch.cuda.current_stream().cuda_stream)

    def compress(self, requests, stream=None):
        compress(self.plan, requests, self.payload.data_ptr(), self.offsets, self.out_bytes.data_ptr(),
                 self.status.data_ptr(), self.workspace.data_ptr(), stream)

    def decompress(self, requests, stream=None):
        decompress(self.plan, self.payload.data_ptr(), self.offsets, requests, self.status.data_ptr(),
                   self.workspace.data_ptr(), stream)

    def payload_of(self, i):
        """Host copy (numpy uint8) of request i's payload, cut to its true size."""
        n = int(self.out_bytes[i].item())
        return self.payload[self.offsets[i]: self.offsets[i] + n].cpu().numpy()
