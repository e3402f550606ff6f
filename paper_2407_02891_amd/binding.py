"""ctypes binding of libbcq.so: same names as the C entry points, argument
marshalling only.  Tensors are torch CUDA(ROCm) tensors used as device memory;
the stream is torch's current stream unless one is given.  There is no CPU
fallback: if the library is missing, loading raises."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libbcq.so")

BCQ_OK, BCQ_ERR_INVALID_ARG, BCQ_ERR_UNSUPPORTED, BCQ_ERR_WORKSPACE, BCQ_ERR_HIP, BCQ_ERR_SCRATCH_LIMIT = range(6)
BCQ_NOALLOC_MAX_ROWS = 131072
BCQ_LAYOUT_VERSION = 2
BCQ_MAX_BATCH = 64

EXPORTS = ["bcq_packed_bytes", "bcq_workspace_bytes", "bcq_workspace_init", "bcq_pack",
           "bcq_pack_rows", "bcq_from_linear", "bcq_quant_workspace_bytes", "bcq_quant_hessian", "bcq_quant_factor_workspace_bytes", "bcq_quant_factor", "bcq_quant_search",
           "bcq_quant_gptq", "bcq_from_linear_rows", "bcq_unpack", "bcq_gemv", "bcq_gemv_noalloc", "bcq_gemm_skinny", "bcq_read_probe_sink_bytes",
           "bcq_read_probe", "bcq_set_option", "bcq_status_string"]


class Desc(ctypes.Structure):
    """struct bcq_desc"""
    _fields_ = [("M", ctypes.c_int32), ("N", ctypes.c_int32), ("q", ctypes.c_int32),
                ("group", ctypes.c_int32), ("has_offset", ctypes.c_int32),
                ("layout_version", ctypes.c_int32)]


class BcqError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {status_string(status)} (status {int(status)})")


_lib = None


def lib():
    """Load libbcq.so (built in-tree by build.py).  Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python __graft_entry__.py build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        dp = ctypes.POINTER(Desc)
        L.bcq_packed_bytes.restype, L.bcq_packed_bytes.argtypes = sz, [dp]
        L.bcq_workspace_bytes.restype, L.bcq_workspace_bytes.argtypes = sz, [dp, i32]
        L.bcq_workspace_init.restype, L.bcq_workspace_init.argtypes = i32, [vp, sz, vp]
        L.bcq_pack.restype, L.bcq_pack.argtypes = i32, [dp, vp, vp, vp, vp, vp]
        L.bcq_pack_rows.restype, L.bcq_pack_rows.argtypes = i32, [dp, i32, i32, vp, vp, vp, vp, vp]
        L.bcq_from_linear.restype = i32
        L.bcq_from_linear.argtypes = [i32, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_int32), vp, vp, vp, vp, vp, vp, vp]
        L.bcq_quant_workspace_bytes.restype, L.bcq_quant_workspace_bytes.argtypes = sz, [i32, i32]
        L.bcq_quant_hessian.restype, L.bcq_quant_hessian.argtypes = i32, [i32, i32, vp, vp, vp]
        L.bcq_quant_factor_workspace_bytes.restype, L.bcq_quant_factor_workspace_bytes.argtypes = sz, [i32]
        L.bcq_quant_factor.restype = i32
        L.bcq_quant_factor.argtypes = [i32, ctypes.c_float, vp, vp, vp, vp]
        L.bcq_quant_search.restype = i32
        L.bcq_quant_search.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.bcq_quant_gptq.restype = i32
        L.bcq_quant_gptq.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.bcq_from_linear_rows.restype = i32
        L.bcq_from_linear_rows.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.bcq_unpack.restype, L.bcq_unpack.argtypes = i32, [dp, vp, vp, vp, vp, vp]
        L.bcq_gemv.restype, L.bcq_gemv.argtypes = i32, [dp, vp, vp, vp, vp, vp]
        L.bcq_gemv_noalloc.restype, L.bcq_gemv_noalloc.argtypes = i32, [dp, vp, vp, vp, vp]
        L.bcq_gemm_skinny.restype = i32
        L.bcq_gemm_skinny.argtypes = [dp, vp, vp, i32, vp, i32, i32, vp, vp]
        L.bcq_read_probe_sink_bytes.restype, L.bcq_read_probe_sink_bytes.argtypes = sz, []
        L.bcq_read_probe.restype, L.bcq_read_probe.argtypes = i32, [vp, sz, vp, vp]
        L.bcq_set_option.restype, L.bcq_set_option.argtypes = i32, [ctypes.c_char_p, i32]
        L.bcq_status_string.restype, L.bcq_status_string.argtypes = ctypes.c_char_p, [i32]
        _lib = L
    return _lib


def status_string(status):
    return lib().bcq_status_string(int(status)).decode()


def _check(status, where):
    if status != BCQ_OK:
        raise BcqError(status, where)


def _ptr(t):
    """Device pointer of a tensor (or a raw int / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def packed_bytes(desc):
    return int(lib().bcq_packed_bytes(ctypes.byref(desc)))


def workspace_bytes(desc, batch=1):
    return int(lib().bcq_workspace_bytes(ctypes.byref(desc), int(batch)))


def workspace_init(workspace, nbytes=None, stream=None):
    if nbytes is None:
        nbytes = workspace.numel() * workspace.element_size()
    _check(lib().bcq_workspace_init(_ptr(workspace), nbytes, _stream(stream)), "bcq_workspace_init")


def pack(desc, codes, alpha, offset, packed, stream=None):
    _check(lib().bcq_pack(ctypes.byref(desc), _ptr(codes), _ptr(alpha), _ptr(offset), _ptr(packed),
                          _stream(stream)), "bcq_pack")


def pack_rows(desc, row_begin, rows, codes, alpha, offset, packed, stream=None):
    _check(lib().bcq_pack_rows(ctypes.byref(desc), int(row_begin), int(rows), _ptr(codes), _ptr(alpha),
                               _ptr(offset), _ptr(packed), _stream(stream)), "bcq_pack_rows")


def from_linear(M, N, group, n_bits, q, class_of_plane, w_int, S, qbias, codes, alpha, offset, stream=None):
    """class_of_plane: sequence of n_bits ints (host); the rest are device tensors."""
    labels = (ctypes.c_int32 * len(class_of_plane))(*[int(c) for c in class_of_plane])
    _check(lib().bcq_from_linear(int(M), int(N), int(group), int(n_bits), int(q), labels, _ptr(w_int), _ptr(S),
                                 _ptr(qbias), _ptr(codes), _ptr(alpha), _ptr(offset), _stream(stream)),
           "bcq_from_linear")


def quant_workspace_bytes(M, N):
    return int(lib().bcq_quant_workspace_bytes(int(M), int(N)))


def quant_hessian(N, T, X, H, stream=None):
    _check(lib().bcq_quant_hessian(int(N), int(T), _ptr(X), _ptr(H), _stream(stream)), "bcq_quant_hessian")


def quant_factor_workspace_bytes(N):
    return int(lib().bcq_quant_factor_workspace_bytes(int(N)))


def quant_factor(N, damp, H, U, workspace, stream=None):
    _check(lib().bcq_quant_factor(int(N), float(damp), _ptr(H), _ptr(U), _ptr(workspace), _stream(stream)),
           "bcq_quant_factor")


def quant_search(M, N, n_bits, q, grid, W, H, S, qbias, class_of_plane, err, workspace, stream=None):
    _check(lib().bcq_quant_search(int(M), int(N), int(n_bits), int(q), int(grid), _ptr(W), _ptr(H), _ptr(S),
                                  _ptr(qbias), _ptr(class_of_plane), _ptr(err), _ptr(workspace), _stream(stream)),
           "bcq_quant_search")


def quant_gptq(M, N, n_bits, q, W, U, S, qbias, class_of_plane, w_int, workspace, stream=None):
    _check(lib().bcq_quant_gptq(int(M), int(N), int(n_bits), int(q), _ptr(W), _ptr(U), _ptr(S), _ptr(qbias),
                                _ptr(class_of_plane), _ptr(w_int), _ptr(workspace), _stream(stream)), "bcq_quant_gptq")


def from_linear_rows(M, N, n_bits, q, class_of_plane, w_int, S, qbias, codes, alpha, offset, stream=None):
    _check(lib().bcq_from_linear_rows(int(M), int(N), int(n_bits), int(q), _ptr(class_of_plane), _ptr(w_int), _ptr(S),
                                      _ptr(qbias), _ptr(codes), _ptr(alpha), _ptr(offset), _stream(stream)),
           "bcq_from_linear_rows")


def unpack(desc, packed, codes, alpha, offset, stream=None):
    _check(lib().bcq_unpack(ctypes.byref(desc), _ptr(packed), _ptr(codes), _ptr(alpha), _ptr(offset),
                            _stream(stream)), "bcq_unpack")


def gemv(desc, packed, x, y, workspace, stream=None):
    _check(lib().bcq_gemv(ctypes.byref(desc), _ptr(packed), _ptr(x), _ptr(y), _ptr(workspace),
                          _stream(stream)), "bcq_gemv")


def gemv_noalloc(desc, packed, x, y, stream=None):
    _check(lib().bcq_gemv_noalloc(ctypes.byref(desc), _ptr(packed), _ptr(x), _ptr(y), _stream(stream)),
           "bcq_gemv_noalloc")


def gemm_skinny(desc, packed, X, ldx, Y, ldy, batch, workspace, stream=None):
    _check(lib().bcq_gemm_skinny(ctypes.byref(desc), _ptr(packed), _ptr(X), int(ldx), _ptr(Y), int(ldy),
                                 int(batch), _ptr(workspace), _stream(stream)), "bcq_gemm_skinny")


def read_probe(buf, nbytes, sink, stream=None):
    _check(lib().bcq_read_probe(_ptr(buf), int(nbytes), _ptr(sink), _stream(stream)), "bcq_read_probe")


def read_probe_sink_bytes():
    return int(lib().bcq_read_probe_sink_bytes())


def set_option(name, value):
    _check(lib().bcq_set_option(name.encode(), int(value)), "bcq_set_option")


class PackedLayer:
    """Device buffers of one packed layer: holds torch allocations and the
    descriptor, and forwards to the C entry points (no arithmetic here)."""

    def __init__(self, M, N, q, group=128, has_offset=False, max_batch=1, device="cuda"):
        import torch
        self.desc = Desc(M, N, q, group, 1 if has_offset else 0, 0)
        nbytes = packed_bytes(self.desc)
        if nbytes == 0:
            raise BcqError(BCQ_ERR_UNSUPPORTED, "bcq_packed_bytes")
        self.device = device
        self.packed = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.max_batch = max_batch
        ws = workspace_bytes(self.desc, max_batch)
        self.workspace = torch.empty(max(ws, 16), dtype=torch.uint8, device=device)
        self.workspace_bytes = ws
        workspace_init(self.workspace, self.workspace.numel())

    def pack_from(self, codes, alpha, offset):
        """codes uint8 [M][N], alpha fp16 [M][G][q], offset fp16 [M][G] or None (device tensors)."""
        pack(self.desc, codes, alpha, offset, self.packed)
        return self

    def pack_rows_from(self, row_begin, codes, alpha, offset):
        """Rows [row_begin, row_begin + codes.shape[0]) from tensors that hold only those rows."""
        pack_rows(self.desc, row_begin, codes.shape[0], codes, alpha, offset, self.packed)
        return self

    def gemv(self, x, y=None):
        import torch
        if y is None:
            y = torch.empty(self.desc.M, dtype=torch.float16, device=self.device)
        gemv(self.desc, self.packed, x, y, self.workspace if self.workspace_bytes else None)
        return y

    def gemm_skinny(self, X, Y=None):
        import torch
        batch = X.shape[0]
        if not 1 <= batch <= BCQ_MAX_BATCH:
            raise BcqError(BCQ_ERR_INVALID_ARG, "PackedLayer.gemm_skinny (batch outside 1..%d)" % BCQ_MAX_BATCH)
        if batch > self.max_batch:   # the workspace holds max_batch accumulators per row
            raise BcqError(BCQ_ERR_WORKSPACE, "PackedLayer.gemm_skinny (batch %d > max_batch %d)" % (batch, self.max_batch))
        if Y is None:
            Y = torch.empty((batch, self.desc.M), dtype=torch.float16, device=self.device)
        gemm_skinny(self.desc, self.packed, X, X.stride(0), Y, Y.stride(0), batch,
                    self.workspace if self.workspace_bytes else None)
        return Y
