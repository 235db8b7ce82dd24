"""Thin ctypes binding of libtreeattn (argument marshalling only; every step runs in the HIP kernels).

Function names and argument order follow include/treeattn.h.  Tensors are torch tensors on the GPU
(torch is used for device memory and streams only) or `Desc` objects (raw pointer + shape + strides,
used to exercise the host-side validation without a GPU).  There is no CPU fallback: if the shared
library is missing, importing the entry points fails loudly.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# TREEATTN_LIB names another build of the same library (the sanitizer build of the host code, which has no kernels
# behind it, is loaded that way by the host tests)
LIB_PATH = os.environ.get("TREEATTN_LIB") or os.path.join(_HERE, "libtreeattn.so")

TA_F32, TA_BF16, TA_I32, TA_U64 = 0, 1, 2, 3
TA_KERNEL_AUTO, TA_KERNEL_GENERIC, TA_KERNEL_MFMA, TA_KERNEL_MFMA_BASIC = 0, 1, 2, 3
TA_STATUS_BAD_PARENT, TA_STATUS_BAD_SEQLEN, TA_STATUS_BAD_PATH, TA_STATUS_BAD_PAGE = 1, 2, 4, 8
TA_MERGE_GENERAL, TA_MERGE_D128, TA_MERGE_D128_WIDE = 0, 1, 2

TA_OK = 0
TA_ERR_NULL, TA_ERR_DTYPE, TA_ERR_RANK, TA_ERR_SHAPE, TA_ERR_STRIDE, TA_ERR_HEADS = -1, -2, -3, -4, -5, -6
TA_ERR_HEAD_DIM, TA_ERR_TREE_SIZE, TA_ERR_PAGE_TABLE, TA_ERR_WORKSPACE, TA_ERR_HIP = -7, -8, -9, -10, -11
TA_ERR_BATCH, TA_ERR_OPTS = -12, -13

EXPORTS = (
    "tree_attn_fwd", "tree_attn_fwd_ex", "tree_attn_workspace_bytes", "tree_attn_reserve", "tree_attn_release",
    "tree_attn_encode", "tree_attn_append", "tree_attn_compact", "tree_attn_last_status", "tree_attn_plan",
    "tree_attn_dispatch_row", "tree_attn_stream_read", "tree_attn_mfma_probe", "tree_attn_fwd_static", "tree_attn_strerror", "tree_attn_version",
)


class ta_tensor(ctypes.Structure):
    _fields_ = [
        ("data", ctypes.c_void_p),
        ("dtype", ctypes.c_int32),
        ("ndim", ctypes.c_int32),
        ("shape", ctypes.c_int64 * 5),
        ("stride", ctypes.c_int64 * 5),
    ]


class ta_opts(ctypes.Structure):
    _fields_ = [
        ("scale", ctypes.c_float),
        ("num_splits", ctypes.c_int32),
        ("kernel", ctypes.c_int32),
        ("item_cost", ctypes.c_int32),
        ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_size_t),
        ("events", ctypes.c_void_p * 3),
        ("tree_masks", ctypes.c_void_p),
        ("tree_masks_stride", ctypes.c_int64),
        ("q_node_offset", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
        ("kv_start", ctypes.c_void_p),
        ("k_new", ctypes.POINTER(ta_tensor)),
        ("v_new", ctypes.POINTER(ta_tensor)),
        ("status", ctypes.c_void_p),
    ]


class Desc:
    """A tensor descriptor without storage behind it (host-side validation tests)."""

    def __init__(self, shape, dtype, stride=None, ptr=0x1000):
        self.shape = tuple(shape)
        self.dtype = dtype
        if stride is None:
            stride, acc = [], 1
            for s in reversed(self.shape):
                stride.append(acc)
                acc *= max(int(s), 1)
            stride = tuple(reversed(stride))
        self.stride = tuple(stride)
        self.ptr = ptr


class TreeAttnError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, tree_attn_strerror(status), status))


_lib = None


def load_library():
    """Load libtreeattn.so (built in-tree by paper_2508_08192_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "libtreeattn.so is not built: run `python -m paper_2508_08192_amd.build` "
                "(there is no CPU fallback for the tree-attention kernels)")
        # The callers' device memory and streams come from PyTorch, which ships a HIP runtime of its own: it has to be
        # in the process before this library is, so that both bind to the same one (loaded the other way round, the
        # library would sit on the system's runtime, PyTorch on its own, and every call here would fail).
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = ctypes.CDLL(LIB_PATH)
        T = ctypes.POINTER(ta_tensor)
        lib.tree_attn_fwd.restype = ctypes.c_int
        lib.tree_attn_fwd.argtypes = [T, T, T, T, T, T, T, T, ctypes.c_void_p]
        lib.tree_attn_fwd_ex.restype = ctypes.c_int
        lib.tree_attn_fwd_ex.argtypes = [T, T, T, T, T, T, T, T, ctypes.c_void_p, ctypes.POINTER(ta_opts)]
        lib.tree_attn_mfma_probe.restype = ctypes.c_int
        lib.tree_attn_mfma_probe.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64), ctypes.c_void_p]
        lib.tree_attn_fwd_static.restype = ctypes.c_int
        lib.tree_attn_fwd_static.argtypes = [T, T, T, T, T, T, T, T, ctypes.c_void_p, ctypes.POINTER(ta_opts)]
        lib.tree_attn_workspace_bytes.restype = ctypes.c_size_t
        lib.tree_attn_workspace_bytes.argtypes = [ctypes.c_int32] * 7
        lib.tree_attn_reserve.restype = ctypes.c_int
        lib.tree_attn_reserve.argtypes = [ctypes.c_size_t]
        lib.tree_attn_release.restype = ctypes.c_int
        lib.tree_attn_release.argtypes = []
        lib.tree_attn_dispatch_row.restype = ctypes.c_int
        lib.tree_attn_dispatch_row.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_int64)]
        lib.tree_attn_stream_read.restype = ctypes.c_int
        lib.tree_attn_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        lib.tree_attn_encode.restype = ctypes.c_int
        lib.tree_attn_encode.argtypes = [T, T, ctypes.c_void_p]
        lib.tree_attn_append.restype = ctypes.c_int
        lib.tree_attn_append.argtypes = [T, T, T, T, T, T, ctypes.c_void_p]
        lib.tree_attn_compact.restype = ctypes.c_int
        lib.tree_attn_compact.argtypes = [T, T, T, T, T, T, ctypes.c_int32, T, ctypes.c_void_p]
        lib.tree_attn_last_status.restype = ctypes.c_int
        lib.tree_attn_last_status.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p]
        lib.tree_attn_plan.restype = ctypes.c_int
        lib.tree_attn_plan.argtypes = [T, T, T, T, T, T, T, T, ctypes.POINTER(ta_opts), ctypes.c_int32,
                                       ctypes.POINTER(ctypes.c_int64)]
        lib.tree_attn_strerror.restype = ctypes.c_char_p
        lib.tree_attn_strerror.argtypes = [ctypes.c_int]
        lib.tree_attn_version.restype = ctypes.c_int
        lib.tree_attn_version.argtypes = []
        _lib = lib
    return _lib


def _torch_dtype_code(t):
    import torch
    table = {torch.float32: TA_F32, torch.bfloat16: TA_BF16, torch.int32: TA_I32, torch.int64: TA_U64,
             torch.uint64: TA_U64}
    if t.dtype not in table:
        return -1
    return table[t.dtype]


def _desc(t):
    """torch tensor | Desc | None -> (ta_tensor or None)."""
    if t is None:
        return None
    d = ta_tensor()
    if isinstance(t, Desc):
        shape, stride, d.data, d.dtype = t.shape, t.stride, t.ptr, t.dtype
    else:
        shape, stride, d.data, d.dtype = tuple(t.shape), tuple(t.stride()), t.data_ptr(), _torch_dtype_code(t)
    if len(shape) > 5:
        raise ValueError("at most 5 dimensions")
    d.ndim = len(shape)
    for i, (s, st) in enumerate(zip(shape, stride)):
        d.shape[i] = s
        d.stride[i] = st
    return d


def _ref(d):
    return ctypes.byref(d) if d is not None else None


def _stream_ptr(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _opts(scale=None, num_splits=0, kernel=TA_KERNEL_AUTO, workspace=None, events=None, item_cost=0, tree_masks=None,
          kv_start=None, q_node_offset=0, k_new=None, v_new=None, status=None):
    o = ta_opts()
    o._keep = [_desc(k_new), _desc(v_new)]             # the descriptors must outlive the call
    if o._keep[0] is not None:
        o.k_new = ctypes.pointer(o._keep[0])
    if o._keep[1] is not None:
        o.v_new = ctypes.pointer(o._keep[1])
    o.scale = 0.0 if scale is None else float(scale)
    o.num_splits = int(num_splits)
    o.kernel = int(kernel)
    o.item_cost = int(item_cost)
    if workspace is not None:
        o.workspace = workspace.data_ptr()
        o.workspace_bytes = workspace.numel() * workspace.element_size()
    if events is not None:
        for i, ev in enumerate(events):
            o.events[i] = ev
    if tree_masks is not None:                         # int64/uint64 words [B, T] or [T] from tree_attn_encode
        o.tree_masks = tree_masks.data_ptr()
        o.tree_masks_stride = int(tree_masks.stride(0)) if tree_masks.dim() == 2 else 0
    if kv_start is not None:                           # int32 [B], contiguous
        o.kv_start = kv_start.data_ptr()
    o.q_node_offset = int(q_node_offset)
    if status is not None:                             # int32 [1] on the device: the call's own status word
        o.status = status.ptr if isinstance(status, Desc) else status.data_ptr()
    return o


def tree_attn_version():
    return int(load_library().tree_attn_version())


def tree_attn_strerror(status):
    return load_library().tree_attn_strerror(int(status)).decode()


def tree_attn_fwd(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse=None, stream=None, check=True):
    """include/treeattn.h: tree_attn_fwd.  Returns the status code (raises TreeAttnError if check)."""
    ds = [_desc(x) for x in (q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse)]
    rc = load_library().tree_attn_fwd(*[_ref(d) for d in ds], _stream_ptr(stream) if stream != 0 else None)
    if check and rc != TA_OK:
        raise TreeAttnError(rc, "tree_attn_fwd")
    return rc


def tree_attn_fwd_ex(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse=None, stream=None,
                     scale=None, num_splits=0, kernel=TA_KERNEL_AUTO, workspace=None, events=None, check=True,
                     item_cost=0, tree_masks=None, kv_start=None, q_node_offset=0, k_new=None, v_new=None, status=None):
    """include/treeattn.h: tree_attn_fwd_ex.  `events`: up to three hipEvent_t handles (ctypes.c_void_p)."""
    ds = [_desc(x) for x in (q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse)]
    o = _opts(scale, num_splits, kernel, workspace, events, item_cost, tree_masks, kv_start, q_node_offset, k_new, v_new,
              status)
    rc = load_library().tree_attn_fwd_ex(*[_ref(d) for d in ds], _stream_ptr(stream) if stream != 0 else None,
                                         ctypes.byref(o))
    if check and rc != TA_OK:
        raise TreeAttnError(rc, "tree_attn_fwd_ex")
    return rc


TA_STATIC_SCRATCH_BYTES = 48 << 20


def tree_attn_fwd_static(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse=None, stream=None,
                         scale=None, num_splits=0, kernel=TA_KERNEL_AUTO, workspace=None, events=None, check=True,
                         item_cost=0, tree_masks=None, kv_start=None, q_node_offset=0, k_new=None, v_new=None,
                         status=None):
    """include/treeattn.h: tree_attn_fwd_static (the call that allocates nothing)."""
    ds = [_desc(x) for x in (q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse)]
    o = _opts(scale, num_splits, kernel, workspace, events, item_cost, tree_masks, kv_start, q_node_offset, k_new, v_new,
              status)
    rc = load_library().tree_attn_fwd_static(*[_ref(d) for d in ds], _stream_ptr(stream) if stream != 0 else None,
                                             ctypes.byref(o))
    if check and rc != TA_OK:
        raise TreeAttnError(rc, "tree_attn_fwd_static")
    return rc


def tree_attn_workspace_bytes(B, T, Hq, Hkv, D, dtype, num_cus=0):
    return int(load_library().tree_attn_workspace_bytes(B, T, Hq, Hkv, D, dtype, num_cus))


def tree_attn_reserve(nbytes, check=True):
    rc = load_library().tree_attn_reserve(int(nbytes))
    if check and rc != TA_OK:
        raise TreeAttnError(rc, "tree_attn_reserve")
    return rc


def tree_attn_release(check=True):
    """Frees the library-owned workspace buffers of the current device (synchronises it)."""
    rc = load_library().tree_attn_release()
    if check and rc != TA_OK:
        raise TreeAttnError(rc, "tree_attn_release")
    return rc


def tree_attn_dispatch_table():
    """The library's dispatch table as a list of dicts (host-only)."""
    keys = ("family", "rows_group_max", "lists_max", "wg_per_cu_x4", "min_share", "item_cost", "wide_from_parts",
            "wide_max_rows")
    rows, i = [], 0
    while True:
        row = (ctypes.c_int64 * 8)()
        if load_library().tree_attn_dispatch_row(i, row) != TA_OK:
            return rows
        rows.append(dict(zip(keys, [int(x) for x in row])))
        i += 1


def tree_attn_stream_read(buf, sink, stream=None, check=True):
    """include/treeattn.h: tree_attn_stream_read (measurement aid: one plain streaming read of `buf`)."""
    rc = load_library().tree_attn_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(),
                                              _stream_ptr(stream) if stream != 0 else None)
    if check and rc != TA_OK:
        raise TreeAttnError(rc, "tree_attn_stream_read")
    return rc


def tree_attn_mfma_probe(iters, sink, stream=None, check=True):
    """include/treeattn.h: tree_attn_mfma_probe (measurement aid); returns the flop of the launch."""
    flop = ctypes.c_int64(0)
    rc = load_library().tree_attn_mfma_probe(int(iters), sink.data_ptr(), ctypes.byref(flop),
                                             _stream_ptr(stream) if stream != 0 else None)
    if check and rc != TA_OK:
        raise TreeAttnError(rc, "tree_attn_mfma_probe")
    return int(flop.value)


def tree_attn_encode(tree_parent, masks, stream=None, check=True):
    a, b = _desc(tree_parent), _desc(masks)
    rc = load_library().tree_attn_encode(_ref(a), _ref(b), _stream_ptr(stream) if stream != 0 else None)
    if check and rc != TA_OK:
        raise TreeAttnError(rc, "tree_attn_encode")
    return rc


def tree_attn_append(k_new, v_new, k_cache, v_cache, page_table, seq_lens, stream=None, check=True):
    """include/treeattn.h: tree_attn_append (write-back of the tree tokens' keys and values)."""
    ds = [_desc(x) for x in (k_new, v_new, k_cache, v_cache, page_table, seq_lens)]
    rc = load_library().tree_attn_append(*[_ref(d) for d in ds], _stream_ptr(stream) if stream != 0 else None)
    if check and rc != TA_OK:
        raise TreeAttnError(rc, "tree_attn_append")
    return rc


def tree_attn_compact(k_cache, v_cache, page_table, seq_lens, accepted, n_accepted, tree_size, seq_lens_out=None,
                      stream=None, check=True):
    """include/treeattn.h: tree_attn_compact (bookkeeping after acceptance: the accepted path moves behind the prefix)."""
    ds = [_desc(x) for x in (k_cache, v_cache, page_table, seq_lens, accepted, n_accepted)]
    so = _desc(seq_lens_out)
    rc = load_library().tree_attn_compact(*[_ref(d) for d in ds], int(tree_size), _ref(so),
                                          _stream_ptr(stream) if stream != 0 else None)
    if check and rc != TA_OK:
        raise TreeAttnError(rc, "tree_attn_compact")
    return rc


def tree_attn_last_status(stream=None):
    """Reads and clears the device status word (synchronises the stream)."""
    val = ctypes.c_int32(0)
    rc = load_library().tree_attn_last_status(ctypes.byref(val), _stream_ptr(stream) if stream != 0 else None)
    if rc != TA_OK:
        raise TreeAttnError(rc, "tree_attn_last_status")
    return int(val.value)


def tree_attn_plan(q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse=None, num_cus=256,
                   scale=None, num_splits=0, kernel=TA_KERNEL_AUTO, check=True, item_cost=0, status=None):
    """Host-only launch plan; returns a dict (or the negative status if check is False and it failed)."""
    ds = [_desc(x) for x in (q, k_cache, v_cache, page_table, seq_lens, tree_parent, out, lse)]
    o = _opts(scale, num_splits, kernel, None, None, item_cost, status=status)
    plan = (ctypes.c_int64 * 16)()
    rc = load_library().tree_attn_plan(*[_ref(d) for d in ds], ctypes.byref(o), num_cus, plan)
    if rc != TA_OK:
        if check:
            raise TreeAttnError(rc, "tree_attn_plan")
        return rc
    keys = ("kernel", "kv_workgroups", "threads", "tile", "row_groups", "rows_per_group", "partial_slots",
            "merge_workgroups", "min_share", "item_cost", "merge_kernel", "table_row", "workspace_bytes",
            "partials_q15")
    return dict(zip(keys, [int(x) for x in plan]))
