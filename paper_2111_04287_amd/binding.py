"""ctypes binding of libbf: argument marshalling only.

Every function here has the name of the C entry point it forwards to (see
``include/bf.h``) and does nothing but turn torch tensors into device pointers,
sizes and the current HIP stream.  All arithmetic happens in the library's
kernels.  If ``libbf.so`` has not been built the import fails; there is no
fallback path.
"""

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbf.so")

BF_OK = 0
(BF_ERR_NULL, BF_ERR_SIZE, BF_ERR_ALIGN, BF_ERR_ALIAS, BF_ERR_KIND, BF_ERR_ROUND,
 BF_ERR_NOT_STOCHASTIC, BF_ERR_NOT_CONNECTED, BF_ERR_CSR, BF_ERR_TOPO_MISMATCH,
 BF_ERR_UNSUPPORTED, BF_ERR_HIP, BF_ERR_NOMEM) = range(-1, -14, -1)

BF_RING, BF_EXP_STATIC, BF_EXP2_ONE_PEER, BF_RANDOM_DIRECTED, BF_CSR_USER, BF_DENSE_USER = range(6)
BF_F32, BF_BF16 = 0, 1
BF_ATC, BF_AWC = 0, 1
BF_W_ANY, BF_W_PULL, BF_W_PUSH, BF_W_STANDARD = 0, 1, 2, 3

EXPORTS = [
    "bf_topology_create", "bf_topology_create_push_pull", "bf_topology_destroy", "bf_topology_n",
    "bf_topology_rounds", "bf_topology_nnz", "bf_topology_max_degree", "bf_topology_class",
    "bf_topology_export_csr", "bf_topology_chain_plan", "bf_topology_window_slots", "bf_topology_export_window",
    "bf_win_put", "bf_win_get", "bf_win_accumulate", "bf_win_put_weighted", "bf_win_get_weighted", "bf_win_accumulate_weighted", "bf_win_update_weighted", "bf_dgd_least_squares_run", "bf_dgd_least_squares_run_static", "bf_exact_diffusion_least_squares_run", "bf_dgd_status", "bf_stream_probe", "bf_win_update", "bf_win_update_then_collect", "bf_neighbor_allreduce", "bf_neighbor_allreduce_multi", "bf_hierarchical_neighbor_allreduce", "bf_dense_mix", "bf_pushsum_step", "bf_pushsum_atc_step", "bf_tracking_step",
    "bf_atc_step", "bf_atc_step_layouts", "bf_exact_diffusion_step", "bf_exact_diffusion_step_layouts", "bf_grad_least_squares", "bf_grad_quadratic", "bf_consensus_stats",
    "bf_strerror", "bf_last_hip_error", "bf_set_tuning", "bf_recommended_ld",
    "bf_blocked_elems", "bf_recommended_block", "bf_blocked_pack", "bf_blocked_unpack",
]


class bf_topo_params_t(C.Structure):
    _fields_ = [
        ("out_degree", C.c_int32),
        ("require_strongly_connected", C.c_int32),
        ("seed", C.c_uint64),
        ("rounds", C.c_int32),
        ("require_class", C.c_int32),
        ("rowptr", C.POINTER(C.c_int64)),
        ("col", C.POINTER(C.c_int32)),
        ("wgt", C.POINTER(C.c_float)),
        ("dense_w", C.POINTER(C.c_float)),
    ]


class BfError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = lib.bf_strerror(code).decode()
        if code == BF_ERR_HIP:
            msg += " (hipError %d)" % lib.bf_last_hip_error()
        super().__init__("%s: %s [%d]" % (where, msg, code))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libbf.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
            "from the repository root (needs hipcc). There is no CPU fallback.")
    # One HIP runtime per process: PyTorch ships its own libamdhip64 (same SONAME as the system
    # one).  Loading torch first makes libbf's dependency resolve to that already-loaded copy, so
    # device pointers and streams created by torch are valid inside libbf.
    import torch
    hip = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    if os.path.exists(hip):
        C.CDLL(hip, mode=C.RTLD_GLOBAL)
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    L.bf_topology_create.argtypes = [C.POINTER(vp), C.c_int, i32, C.POINTER(bf_topo_params_t)]
    L.bf_topology_create_push_pull.argtypes = [C.POINTER(vp), i32, vp, vp, vp, vp, vp, vp, vp]
    L.bf_topology_destroy.argtypes = [vp]
    L.bf_topology_n.argtypes = [vp]
    L.bf_topology_rounds.argtypes = [vp]
    L.bf_topology_nnz.argtypes = [vp, i32]
    L.bf_topology_nnz.restype = i64
    L.bf_topology_max_degree.argtypes = [vp, i32]
    L.bf_topology_class.argtypes = [vp, i32]
    L.bf_topology_export_csr.argtypes = [vp, i32, vp, vp, vp, C.POINTER(C.c_uint64)]
    L.bf_topology_chain_plan.argtypes = [vp, i32, vp]
    L.bf_neighbor_allreduce.argtypes = [vp, i32, vp, vp, i64, i64, C.c_int, vp]
    L.bf_topology_window_slots.argtypes = [vp, i32]
    L.bf_topology_window_slots.restype = i64
    L.bf_topology_export_window.argtypes = [vp, i32, C.POINTER(C.c_int64), C.POINTER(C.c_int32),
                                            C.POINTER(C.c_float), C.POINTER(C.c_float)]
    L.bf_win_put.argtypes = [vp, i32, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_dgd_least_squares_run.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, C.c_float, i64, i64, vp]
    L.bf_dgd_status.argtypes = [vp, C.POINTER(C.c_int32), vp]
    L.bf_dgd_least_squares_run_static.argtypes = [vp, i32, i32, i32, vp, vp, vp, C.c_float, i64, i64, vp]
    L.bf_exact_diffusion_least_squares_run.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, C.c_float, i64, i64, vp]
    L.bf_stream_probe.argtypes = [i32, vp, vp, i64, i32, vp]
    L.bf_win_get.argtypes = [vp, i32, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_win_put_weighted.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_win_get_weighted.argtypes = [vp, i32, vp, vp, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_win_accumulate_weighted.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_win_update_weighted.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_win_update.argtypes = [vp, i32, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_win_accumulate.argtypes = [vp, i32, vp, vp, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_win_update_then_collect.argtypes = [vp, i32, vp, vp, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_neighbor_allreduce_multi.argtypes = [vp, i32, i32, vp, vp, i64, i64, C.c_int, vp]
    L.bf_hierarchical_neighbor_allreduce.argtypes = [vp, i32, i32, vp, vp, i64, i64, C.c_int, vp]
    L.bf_dense_mix.argtypes = [vp, i32, vp, vp, i64, i64, C.c_int, vp]
    L.bf_pushsum_step.argtypes = [vp, i32, vp, vp, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_pushsum_atc_step.argtypes = [vp, i32, vp, vp, vp, f32, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_tracking_step.argtypes = [vp, i32, vp, vp, vp, vp, i64, i64, C.c_int, vp]
    L.bf_atc_step.argtypes = [vp, i32, vp, vp, vp, vp, f32, f32, C.c_int, i64, i64, C.c_int, vp]
    L.bf_atc_step_layouts.argtypes = [vp, i32, vp, vp, vp, vp, f32, f32, C.c_int, i64, i64, i64, i64, C.c_int, vp]
    L.bf_exact_diffusion_step.argtypes = [vp, i32, vp, vp, vp, vp, f32, i64, i64, C.c_int, vp]
    L.bf_exact_diffusion_step_layouts.argtypes = [vp, i32, vp, vp, vp, vp, f32, i64, i64, i64, i64, C.c_int, vp]
    L.bf_grad_least_squares.argtypes = [i32, i32, i64, vp, vp, vp, i64, vp, i64, vp]
    L.bf_grad_quadratic.argtypes = [i32, i64, i64, vp, vp, vp, f32, f32, vp, C.c_int, vp]
    L.bf_consensus_stats.argtypes = [i32, i64, i64, vp, vp, C.c_int, vp, vp, vp]
    L.bf_strerror.argtypes = [C.c_int]
    L.bf_strerror.restype = C.c_char_p
    L.bf_last_hip_error.argtypes = []
    L.bf_set_tuning.argtypes = [i32, i32]
    L.bf_recommended_ld.argtypes = [i64, C.c_int]
    L.bf_recommended_ld.restype = i64
    L.bf_blocked_elems.argtypes = [i32, i64, i64]
    L.bf_blocked_elems.restype = i64
    L.bf_recommended_block.argtypes = [vp, i64, C.c_int]
    L.bf_recommended_block.restype = i64
    L.bf_blocked_pack.argtypes = [i32, i64, i64, vp, i64, vp, C.c_int, vp]
    L.bf_blocked_unpack.argtypes = [i32, i64, i64, vp, i64, vp, C.c_int, vp]
    for name in EXPORTS:
        getattr(L, name)          # raises AttributeError if a declared symbol is missing
    return L


lib = _load()


def _check(code, where):
    if code != BF_OK:
        raise BfError(code, where)


def _np_ptr(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


class Topology:
    """Owner of a ``bf_topology_t*``."""

    def __init__(self, handle):
        self.handle = handle
        self._n = None                      # a topology never changes after creation: ask once
        self._rounds = None

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h:
            lib.bf_topology_destroy(h)

    @property
    def n(self):
        if self._n is None:
            self._n = lib.bf_topology_n(self.handle)
        return self._n

    @property
    def rounds(self):
        if self._rounds is None:
            self._rounds = lib.bf_topology_rounds(self.handle)
        return self._rounds


def bf_topology_create(kind, n, out_degree=0, seed=0, require_strongly_connected=True,
                       rounds=1, require_class=BF_W_ANY, rowptr=None, col=None, wgt=None, dense_w=None):
    p = bf_topo_params_t()
    p.out_degree = out_degree
    p.seed = seed
    p.require_strongly_connected = int(bool(require_strongly_connected))
    p.rounds = rounds
    p.require_class = require_class
    keep = []
    if rowptr is not None:
        a = np.ascontiguousarray(rowptr, dtype=np.int64); keep.append(a); p.rowptr = _np_ptr(a, C.c_int64)
    if col is not None:
        a = np.ascontiguousarray(col, dtype=np.int32); keep.append(a); p.col = _np_ptr(a, C.c_int32)
    if wgt is not None:
        a = np.ascontiguousarray(wgt, dtype=np.float32); keep.append(a); p.wgt = _np_ptr(a, C.c_float)
    if dense_w is not None:
        a = np.ascontiguousarray(dense_w, dtype=np.float32); keep.append(a); p.dense_w = _np_ptr(a, C.c_float)
    h = C.c_void_p()
    _check(lib.bf_topology_create(C.byref(h), kind, n, C.byref(p)), "bf_topology_create")
    return Topology(h)


def bf_topology_create_push_pull(n, self_weight, src_rowptr, src_rank, src_weight, dst_rowptr, dst_rank, dst_weight):
    def arr(a, dt):
        return None if a is None else np.ascontiguousarray(a, dtype=dt)
    sw = arr(self_weight, np.float32)
    srp, srk, swt = arr(src_rowptr, np.int64), arr(src_rank, np.int32), arr(src_weight, np.float32)
    drp, drk, dwt = arr(dst_rowptr, np.int64), arr(dst_rank, np.int32), arr(dst_weight, np.float32)
    ptr = lambda a: None if a is None else a.ctypes.data
    h = C.c_void_p()
    _check(lib.bf_topology_create_push_pull(C.byref(h), n, ptr(sw), ptr(srp), ptr(srk), ptr(swt),
                                            ptr(drp), ptr(drk), ptr(dwt)), "bf_topology_create_push_pull")
    return Topology(h)


def bf_topology_rounds(t):
    return lib.bf_topology_rounds(t.handle)


def bf_topology_nnz(t, rnd=0):
    return lib.bf_topology_nnz(t.handle, rnd)


def bf_topology_max_degree(t, rnd=0):
    return lib.bf_topology_max_degree(t.handle, rnd)


def bf_topology_class(t, rnd=0):
    return lib.bf_topology_class(t.handle, rnd)


def bf_topology_export_csr(t, rnd=0):
    """Returns (rowptr int64[n+1], col int32[nnz], wgt float32[nnz], accepted_seed)."""
    n = lib.bf_topology_n(t.handle)
    nnz = lib.bf_topology_nnz(t.handle, rnd)
    if nnz < 0:
        raise BfError(int(nnz), "bf_topology_nnz")
    rowptr = np.empty(n + 1, dtype=np.int64)
    col = np.empty(nnz, dtype=np.int32)
    wgt = np.empty(nnz, dtype=np.float32)
    seed = C.c_uint64(0)
    _check(lib.bf_topology_export_csr(t.handle, rnd, rowptr.ctypes.data, col.ctypes.data, wgt.ctypes.data,
                                      C.byref(seed)), "bf_topology_export_csr")
    return rowptr, col, wgt, seed.value


def bf_topology_chain_plan(t, rnd=0):
    """None if the round has no chain plan, else an (n, 8) int32 array of walk steps."""
    n = lib.bf_topology_chain_plan(t.handle, rnd, None)
    if n < 0:
        raise BfError(int(n), "bf_topology_chain_plan")
    if n == 0:
        return None
    steps = np.empty((n, 8), dtype=np.int32)
    lib.bf_topology_chain_plan(t.handle, rnd, steps.ctypes.data)
    return steps


# ---- tensor marshalling ----------------------------------------------------------------------
def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return BF_F32
    if t.dtype == torch.bfloat16:
        return BF_BF16
    raise TypeError("libbf handles float32 and bfloat16 matrices, got %s" % t.dtype)


class Blocked:
    """A matrix in the column-block layout (``BF_LD_BLOCKED`` in bf.h): ``data`` is a contiguous
    (ceil(d/B), n, B) tensor, ``d`` the number of columns that exist.  It stands where the calls
    that accept the layout take a 2-D tensor; nothing is computed here."""

    def __init__(self, data, d):
        if data.dim() != 3 or not data.is_contiguous():
            raise ValueError("a column-block matrix is a contiguous (blocks, n, B) tensor")
        nb, n, blk = data.shape
        if nb != (d + blk - 1) // blk:
            raise ValueError("%d columns in blocks of %d need %d blocks, the tensor has %d" % (d, blk, (d + blk - 1) // blk, nb))
        self.data, self.d = data, d
        self.shape = (n, d)
        self.dtype = data.dtype
        self.device = data.device

    def dim(self):
        return 2

    def stride(self, k):
        return -self.data.shape[2] if k == 0 else 1     # what the C calls take as ld

    def data_ptr(self):
        return self.data.data_ptr()

    def element_size(self):
        return self.data.element_size()


def _mat(t, name):
    """(ptr, n, d, ld) of an agent-major 2-D tensor with unit column stride, or of a Blocked."""
    if isinstance(t, Blocked):
        return t.data_ptr(), t.shape[0], t.d, t.stride(0)
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("%s must be 2-D with contiguous rows" % name)
    n, d = t.shape
    ld = t.stride(0) if n > 1 else max(d, 1)
    if n == 1:
        per16 = 16 // t.element_size()
        ld = (ld + per16 - 1) // per16 * per16 if ld % per16 else ld
    return t.data_ptr(), n, d, ld


_raw_stream = None


def _stream(stream):
    """HIP stream handle: the given torch stream (or raw handle), else torch's current stream.  The
    raw getter is several times cheaper than building a torch.cuda.Stream object, which matters for
    the latency-bound small configurations."""
    global _raw_stream
    if stream is None:
        import torch
        if _raw_stream is None:
            _raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", False)
        if _raw_stream:
            return _raw_stream(torch.cuda.current_device())
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _rows(t, n, per_agent=1):
    """The C entry points take the row count from the topology: a tensor with fewer rows would be
    read and written out of bounds, so the count is checked here, where the shapes are known."""
    if n != t.n * per_agent:
        raise ValueError("the matrix has %d rows, the topology %d agents" % (n, t.n * per_agent))


def _vec(w, n, name):
    import torch
    if w.dtype != torch.float32 or w.dim() != 1 or w.numel() != n or not w.is_contiguous():
        raise ValueError("%s must be a contiguous float32 vector with one entry per agent" % name)


def _same_layout(ref, other, name):
    if isinstance(ref, Blocked) != isinstance(other, Blocked):
        raise ValueError("%s must have the layout of X_in" % name)
    if other.shape != ref.shape or (ref.shape[0] > 1 and other.stride(0) != ref.stride(0)) or other.dtype != ref.dtype:
        raise ValueError("%s must match the shape, row stride and dtype of X_in" % name)


def bf_neighbor_allreduce(t, rnd, X_in, X_out, stream=None):
    ptr, n, d, ld = _mat(X_in, "X_in")
    _rows(t, n)
    _same_layout(X_in, X_out, "X_out")
    _check(lib.bf_neighbor_allreduce(t.handle, rnd, ptr, X_out.data_ptr(), d, ld, _dtype_code(X_in),
                                     _stream(stream)), "bf_neighbor_allreduce")
    return X_out


def bf_neighbor_allreduce_multi(t, rnd0, count, X_in, X_out, stream=None):
    ptr, n, d, ld = _mat(X_in, "X_in")
    _rows(t, n)
    _same_layout(X_in, X_out, "X_out")
    _check(lib.bf_neighbor_allreduce_multi(t.handle, rnd0, count, ptr, X_out.data_ptr(), d, ld,
                                           _dtype_code(X_in), _stream(stream)), "bf_neighbor_allreduce_multi")
    return X_out


def bf_hierarchical_neighbor_allreduce(machine_topology, rnd, local_size, X_in, X_out, stream=None):
    ptr, n, d, ld = _mat(X_in, "X_in")
    _same_layout(X_in, X_out, "X_out")
    _rows(machine_topology, n, local_size)
    _check(lib.bf_hierarchical_neighbor_allreduce(machine_topology.handle, rnd, local_size, ptr, X_out.data_ptr(), d, ld,
                                                  _dtype_code(X_in), _stream(stream)),
           "bf_hierarchical_neighbor_allreduce")
    return X_out


def bf_topology_window_slots(t, rnd=0):
    e = lib.bf_topology_window_slots(t.handle, rnd)
    if e < 0:
        raise BfError(int(e), "bf_topology_window_slots")
    return int(e)


def bf_topology_export_window(t, rnd=0):
    """(slot_rowptr int64[n+1], slot_src int32[E], slot_weight float32[E], self_weight float32[n])."""
    n, E = t.n, bf_topology_window_slots(t, rnd)
    rp = np.zeros(n + 1, dtype=np.int64)
    src = np.zeros(max(E, 1), dtype=np.int32)
    sw = np.zeros(max(E, 1), dtype=np.float32)
    selfw = np.zeros(n, dtype=np.float32)
    _check(lib.bf_topology_export_window(t.handle, rnd, _np_ptr(rp, C.c_int64), _np_ptr(src, C.c_int32),
                                         _np_ptr(sw, C.c_float), _np_ptr(selfw, C.c_float)), "bf_topology_export_window")
    return rp, src[:E], sw[:E], selfw


def _win_args(t, rnd, active, X, Win, p, win_p):
    import torch
    ptr, n, d, ld = _mat(X, "X")
    _rows(t, n)
    E = bf_topology_window_slots(t, rnd)
    if isinstance(X, Blocked) != isinstance(Win, Blocked):
        raise ValueError("Win must have the layout of X")
    if Win.dim() != 2 or Win.shape != (E, d) or Win.dtype != torch.float32 or (E > 1 and Win.stride(0) != ld) or \
            (d > 1 and Win.stride(1) != 1):
        raise ValueError("Win must be a float32 (slots, d) matrix with the row stride (in elements) of X")
    if active is not None and (active.dtype != torch.int32 or active.numel() != n or not active.is_contiguous()):
        raise ValueError("active must be a contiguous int32 vector with one flag per agent")
    if (p is None) != (win_p is None):
        raise ValueError("p and win_p go together")
    if p is not None:
        _vec(p, n, "p")
        _vec(win_p, E, "win_p")
    return ptr, d, ld, None if active is None else active.data_ptr()


def bf_win_put(t, rnd, X, Win, active=None, stream=None):
    ptr, d, ld, act = _win_args(t, rnd, active, X, Win, None, None)
    _check(lib.bf_win_put(t.handle, rnd, act, ptr, Win.data_ptr(), d, ld, _dtype_code(X), _stream(stream)), "bf_win_put")
    return Win


def bf_win_get(t, rnd, X, Win, active=None, stream=None):
    ptr, d, ld, act = _win_args(t, rnd, active, X, Win, None, None)
    _check(lib.bf_win_get(t.handle, rnd, act, ptr, Win.data_ptr(), d, ld, _dtype_code(X), _stream(stream)), "bf_win_get")
    return Win


def bf_win_accumulate(t, rnd, X, p, Win, win_p, active=None, stream=None):
    ptr, d, ld, act = _win_args(t, rnd, active, X, Win, p, win_p)
    _check(lib.bf_win_accumulate(t.handle, rnd, act, ptr, None if p is None else p.data_ptr(), Win.data_ptr(),
                                 None if win_p is None else win_p.data_ptr(), d, ld, _dtype_code(X), _stream(stream)),
           "bf_win_accumulate")
    return X, p, Win, win_p


def bf_win_update(t, rnd, X, Win, active=None, stream=None):
    ptr, d, ld, act = _win_args(t, rnd, active, X, Win, None, None)
    _check(lib.bf_win_update(t.handle, rnd, act, ptr, Win.data_ptr(), d, ld, _dtype_code(X), _stream(stream)),
           "bf_win_update")
    return X


def bf_win_update_then_collect(t, rnd, X, p, Win, win_p, active=None, stream=None):
    ptr, d, ld, act = _win_args(t, rnd, active, X, Win, p, win_p)
    _check(lib.bf_win_update_then_collect(t.handle, rnd, act, ptr, None if p is None else p.data_ptr(), Win.data_ptr(),
                                          None if win_p is None else win_p.data_ptr(), d, ld, _dtype_code(X),
                                          _stream(stream)), "bf_win_update_then_collect")
    return X, p, Win, win_p


def _call_weights(t, rnd, n, self_weight, edge_weight, edge_on):
    import torch
    E = bf_topology_window_slots(t, rnd)
    if self_weight is not None:
        _vec(self_weight, n, "self_weight")
    if edge_weight is not None:
        _vec(edge_weight, E, "dst_weight / src_weight")
    if edge_on is not None and (edge_on.dtype != torch.int32 or edge_on.numel() != E or not edge_on.is_contiguous()):
        raise ValueError("dst_on / src_on must be a contiguous int32 vector with one flag per slot")
    return tuple(None if v is None else v.data_ptr() for v in (self_weight, edge_weight, edge_on))


def bf_win_put_weighted(t, rnd, X, Win, self_weight=None, dst_weight=None, dst_on=None, active=None, stream=None):
    ptr, d, ld, act = _win_args(t, rnd, active, X, Win, None, None)
    sw, ew, eo = _call_weights(t, rnd, X.shape[0], self_weight, dst_weight, dst_on)
    _check(lib.bf_win_put_weighted(t.handle, rnd, act, ptr, Win.data_ptr(), sw, ew, eo, d, ld, _dtype_code(X), _stream(stream)),
           "bf_win_put_weighted")
    return X, Win


def bf_win_get_weighted(t, rnd, X, Win, src_weight=None, src_on=None, active=None, stream=None):
    ptr, d, ld, act = _win_args(t, rnd, active, X, Win, None, None)
    _, ew, eo = _call_weights(t, rnd, X.shape[0], None, src_weight, src_on)
    _check(lib.bf_win_get_weighted(t.handle, rnd, act, ptr, Win.data_ptr(), ew, eo, d, ld, _dtype_code(X), _stream(stream)),
           "bf_win_get_weighted")
    return Win


def bf_win_accumulate_weighted(t, rnd, X, p, Win, win_p, self_weight=None, dst_weight=None, dst_on=None, active=None,
                               stream=None):
    ptr, d, ld, act = _win_args(t, rnd, active, X, Win, p, win_p)
    sw, ew, eo = _call_weights(t, rnd, X.shape[0], self_weight, dst_weight, dst_on)
    _check(lib.bf_win_accumulate_weighted(t.handle, rnd, act, ptr, None if p is None else p.data_ptr(), Win.data_ptr(),
                                          None if win_p is None else win_p.data_ptr(), sw, ew, eo, d, ld, _dtype_code(X),
                                          _stream(stream)), "bf_win_accumulate_weighted")
    return X, p, Win, win_p


def bf_win_update_weighted(t, rnd, X, Win, self_weight=None, src_weight=None, src_on=None, active=None, stream=None):
    ptr, d, ld, act = _win_args(t, rnd, active, X, Win, None, None)
    sw, ew, eo = _call_weights(t, rnd, X.shape[0], self_weight, src_weight, src_on)
    _check(lib.bf_win_update_weighted(t.handle, rnd, act, ptr, Win.data_ptr(), sw, ew, eo, d, ld, _dtype_code(X),
                                      _stream(stream)), "bf_win_update_weighted")
    return X


def bf_dense_mix(t, rnd, X_in, X_out, stream=None):
    ptr, n, d, ld = _mat(X_in, "X_in")
    _rows(t, n)
    _same_layout(X_in, X_out, "X_out")
    _check(lib.bf_dense_mix(t.handle, rnd, ptr, X_out.data_ptr(), d, ld, _dtype_code(X_in), _stream(stream)),
           "bf_dense_mix")
    return X_out


def bf_pushsum_step(t, rnd, X_in, X_out, w_in, w_out, Y=None, stream=None):
    ptr, n, d, ld = _mat(X_in, "X_in")
    _rows(t, n)
    _same_layout(X_in, X_out, "X_out")
    if Y is not None:
        _same_layout(X_in, Y, "Y")
    _vec(w_in, n, "w_in")
    _vec(w_out, n, "w_out")
    _check(lib.bf_pushsum_step(t.handle, rnd, ptr, X_out.data_ptr(), w_in.data_ptr(), w_out.data_ptr(),
                               None if Y is None else Y.data_ptr(), d, ld, _dtype_code(X_in), _stream(stream)),
           "bf_pushsum_step")
    return X_out, w_out, Y


def bf_pushsum_atc_step(t, rnd, X_in, X_out, G, alpha, w_in, w_out, Y=None, stream=None):
    ptr, n, d, ld = _mat(X_in, "X_in")
    _rows(t, n)
    _same_layout(X_in, X_out, "X_out")
    _same_layout(X_in, G, "G")
    if Y is not None:
        _same_layout(X_in, Y, "Y")
    _vec(w_in, n, "w_in")
    _vec(w_out, n, "w_out")
    _check(lib.bf_pushsum_atc_step(t.handle, rnd, ptr, X_out.data_ptr(), G.data_ptr(), alpha, w_in.data_ptr(),
                                   w_out.data_ptr(), None if Y is None else Y.data_ptr(), d, ld,
                                   _dtype_code(X_in), _stream(stream)), "bf_pushsum_atc_step")
    return X_out, w_out, Y


def bf_tracking_step(t, rnd, Y_in, Y_out, G_new, G_old, stream=None):
    ptr, n, d, ld = _mat(Y_in, "Y_in")
    _rows(t, n)
    for nm, o in (("Y_out", Y_out), ("G_new", G_new), ("G_old", G_old)):
        _same_layout(Y_in, o, nm)
    _check(lib.bf_tracking_step(t.handle, rnd, ptr, Y_out.data_ptr(), G_new.data_ptr(), G_old.data_ptr(), d, ld,
                                _dtype_code(Y_in), _stream(stream)), "bf_tracking_step")
    return Y_out


def bf_atc_step(t, rnd, X_in, X_out, G, M=None, alpha=0.0, beta=0.0, mode=BF_ATC, stream=None):
    ptr, n, d, ld = _mat(X_in, "X_in")
    _rows(t, n)
    _same_layout(X_in, X_out, "X_out")
    _same_layout(X_in, G, "G")
    if M is not None:
        import torch
        if M.dtype != torch.float32 or M.shape != X_in.shape or (n > 1 and M.stride(0) != ld):
            raise ValueError("M must be float32 with the shape and row stride of X_in")
    _check(lib.bf_atc_step(t.handle, rnd, ptr, X_out.data_ptr(), G.data_ptr(),
                           None if M is None else M.data_ptr(), alpha, beta, mode, d, ld,
                           _dtype_code(X_in), _stream(stream)), "bf_atc_step")
    return X_out


def bf_atc_step_layouts(t, rnd, X_in, X_out, G, M=None, alpha=0.0, beta=0.0, mode=BF_ATC, stream=None):
    """bf_atc_step with a layout per matrix: X_in/X_out, G and M may each be an agent-major tensor or a
    Blocked (e.g. parameters and gradients as per-agent vectors, the momentum in column blocks)."""
    import torch
    ptr, n, d, ld = _mat(X_in, "X_in")
    _rows(t, n)
    _same_layout(X_in, X_out, "X_out")
    gptr, gn, gd, ld_g = _mat(G, "G")
    if (gn, gd) != (n, d) or G.dtype != X_in.dtype:
        raise ValueError("G must have the shape and dtype of X_in")
    mptr, ld_m = None, ld
    if M is not None:
        mptr, mn, md, ld_m = _mat(M, "M")
        if (mn, md) != (n, d) or M.dtype != torch.float32:
            raise ValueError("M must be float32 with the shape of X_in")
    _check(lib.bf_atc_step_layouts(t.handle, rnd, ptr, X_out.data_ptr(), gptr, mptr, alpha, beta, mode, d, ld, ld_g,
                                   ld_m, _dtype_code(X_in), _stream(stream)), "bf_atc_step_layouts")
    return X_out


def bf_exact_diffusion_step(t, rnd, X_in, X_out, G, Psi_prev, alpha, stream=None):
    import torch
    ptr, n, d, ld = _mat(X_in, "X_in")
    _rows(t, n)
    _same_layout(X_in, X_out, "X_out")
    _same_layout(X_in, G, "G")
    if Psi_prev.dtype != torch.float32 or Psi_prev.shape != X_in.shape or (n > 1 and Psi_prev.stride(0) != ld):
        raise ValueError("Psi_prev must be float32 with the shape and row stride of X_in")
    _check(lib.bf_exact_diffusion_step(t.handle, rnd, ptr, X_out.data_ptr(), G.data_ptr(), Psi_prev.data_ptr(),
                                       alpha, d, ld, _dtype_code(X_in), _stream(stream)), "bf_exact_diffusion_step")
    return X_out


def bf_exact_diffusion_step_layouts(t, rnd, X_in, X_out, G, Psi_prev, alpha, stream=None):
    """bf_exact_diffusion_step with a layout per matrix (X_in/X_out, G, Psi_prev: tensor or Blocked each)."""
    import torch
    ptr, n, d, ld = _mat(X_in, "X_in")
    _rows(t, n)
    _same_layout(X_in, X_out, "X_out")
    gptr, gn, gd, ld_g = _mat(G, "G")
    pptr, pn, pd, ld_p = _mat(Psi_prev, "Psi_prev")
    if (gn, gd) != (n, d) or G.dtype != X_in.dtype or (pn, pd) != (n, d) or Psi_prev.dtype != torch.float32:
        raise ValueError("G must have the shape and dtype of X_in, Psi_prev its shape in float32")
    _check(lib.bf_exact_diffusion_step_layouts(t.handle, rnd, ptr, X_out.data_ptr(), gptr, pptr, alpha, d, ld, ld_g, ld_p,
                                               _dtype_code(X_in), _stream(stream)), "bf_exact_diffusion_step_layouts")
    return X_out


def bf_dgd_least_squares_run(t, rnd0, iterations, A, b, X, work, alpha, stream=None):
    import torch
    n, m, d = A.shape
    xp, xn, xd, ldx = _mat(X, "X")
    _rows(t, xn)
    if not A.is_contiguous() or not b.is_contiguous() or (xn, xd) != (n, d) or tuple(b.shape) != (n, m) or \
            A.dtype != torch.float32 or b.dtype != torch.float32 or X.dtype != torch.float32:
        raise ValueError("shapes: A (n,m,d) contiguous, b (n,m) contiguous, X (n,d), all float32")
    if work.dtype != torch.float32 or not work.is_contiguous() or work.numel() < 2 * n * ldx:
        raise ValueError("work must be a contiguous float32 tensor of at least 2 * n * ld elements")
    _check(lib.bf_dgd_least_squares_run(t.handle, rnd0, iterations, m, A.data_ptr(), b.data_ptr(), xp, work.data_ptr(),
                                        alpha, d, ldx, _stream(stream)), "bf_dgd_least_squares_run")
    return X


def bf_dgd_least_squares_run_static(t, rnd0, iterations, A, b, X, alpha, stream=None):
    import torch
    n, m, d = A.shape
    xp, xn, xd, ldx = _mat(X, "X")
    _rows(t, xn)
    if not A.is_contiguous() or not b.is_contiguous() or (xn, xd) != (n, d) or tuple(b.shape) != (n, m) or \
            A.dtype != torch.float32 or b.dtype != torch.float32 or X.dtype != torch.float32:
        raise ValueError("shapes: A (n,m,d) contiguous, b (n,m) contiguous, X (n,d), all float32")
    _check(lib.bf_dgd_least_squares_run_static(t.handle, rnd0, iterations, m, A.data_ptr(), b.data_ptr(), xp,
                                               alpha, d, ldx, _stream(stream)), "bf_dgd_least_squares_run_static")
    return X


def bf_exact_diffusion_least_squares_run(t, rnd0, iterations, A, b, X, Psi_prev, work, alpha, stream=None):
    import torch
    n, m, d = A.shape
    xp, xn, xd, ldx = _mat(X, "X")
    _rows(t, xn)
    if not A.is_contiguous() or not b.is_contiguous() or (xn, xd) != (n, d) or tuple(b.shape) != (n, m) or \
            A.dtype != torch.float32 or b.dtype != torch.float32 or X.dtype != torch.float32:
        raise ValueError("shapes: A (n,m,d) contiguous, b (n,m) contiguous, X (n,d), all float32")
    _same_layout(X, Psi_prev, "Psi_prev")
    if work.dtype != torch.float32 or not work.is_contiguous() or work.numel() < 2 * n * ldx:
        raise ValueError("work must be a contiguous float32 tensor of at least 2 * n * ld elements")
    _check(lib.bf_exact_diffusion_least_squares_run(t.handle, rnd0, iterations, m, A.data_ptr(), b.data_ptr(), xp,
                                                    Psi_prev.data_ptr(), work.data_ptr(), alpha, d, ldx, _stream(stream)),
           "bf_exact_diffusion_least_squares_run")
    return X


def bf_dgd_status(t, stream=None):
    out = C.c_int32(0)
    _check(lib.bf_dgd_status(t.handle, C.byref(out), _stream(stream)), "bf_dgd_status")
    return int(out.value)


def bf_stream_probe(mode, src, dst, workgroups_per_cu=1, stream=None):
    """mode 0 copy, 1 read only, 2 write only, over dst.numel() * element_size bytes."""
    nbytes = dst.numel() * dst.element_size()
    if not dst.is_contiguous() or (src is not None and (not src.is_contiguous() or src.numel() * src.element_size() < nbytes)):
        raise ValueError("contiguous tensors, src at least as large as dst")
    _check(lib.bf_stream_probe(mode, None if src is None else src.data_ptr(), dst.data_ptr(), nbytes, workgroups_per_cu,
                               _stream(stream)), "bf_stream_probe")
    return dst


def bf_grad_least_squares(A, b, X, G, stream=None):
    n, m, d = A.shape
    xp, xn, xd, ldx = _mat(X, "X")
    gp, gn, gd, ldg = _mat(G, "G")
    if not A.is_contiguous() or not b.is_contiguous() or (xn, xd) != (n, d) or (gn, gd) != (n, d) or tuple(b.shape) != (n, m):
        raise ValueError("shapes: A (n,m,d) contiguous, b (n,m) contiguous, X and G (n,d)")
    _check(lib.bf_grad_least_squares(n, m, d, A.data_ptr(), b.data_ptr(), xp, ldx, gp, ldg, _stream(stream)),
           "bf_grad_least_squares")
    return G


def bf_grad_quadratic(X, Cc, E, lam, sigma, G, stream=None):
    ptr, n, d, ld = _mat(X, "X")
    for nm, o in (("C", Cc), ("E", E), ("G", G)):
        _same_layout(X, o, nm)
    _check(lib.bf_grad_quadratic(n, d, ld, ptr, Cc.data_ptr(), E.data_ptr(), lam, sigma, G.data_ptr(),
                                 _dtype_code(X), _stream(stream)), "bf_grad_quadratic")
    return G


def bf_consensus_stats(X, p=None, stats=None, mean_out=None, stream=None):
    """stats: float64 device tensor of 3 (sum of squared deviations, max deviation, max |y|)."""
    import torch
    ptr, n, d, ld = _mat(X, "X")
    if stats is None:
        stats = torch.empty(3, dtype=torch.float64, device=X.device)
    _check(lib.bf_consensus_stats(n, d, ld, ptr, None if p is None else p.data_ptr(), _dtype_code(X),
                                  stats.data_ptr(), None if mean_out is None else mean_out.data_ptr(),
                                  _stream(stream)), "bf_consensus_stats")
    return stats


def bf_blocked_elems(n, d, block):
    e = lib.bf_blocked_elems(n, d, block)
    if e < 0:
        raise BfError(int(e), "bf_blocked_elems")
    return e


def bf_recommended_block(t, d, dt):
    b = lib.bf_recommended_block(t.handle, d, dt)
    if b < 0:
        raise BfError(int(b), "bf_recommended_block")
    return b


def bf_blocked_pack(X, Xb, stream=None):
    """X: agent-major 2-D tensor; Xb: Blocked of the same n, d and dtype (written)."""
    ptr, n, d, ld = _mat(X, "X")
    if not isinstance(Xb, Blocked) or Xb.shape != (n, d) or Xb.dtype != X.dtype:
        raise ValueError("Xb must be a Blocked matrix with the shape and dtype of X")
    _check(lib.bf_blocked_pack(n, d, ld, ptr, -Xb.stride(0), Xb.data_ptr(), _dtype_code(X), _stream(stream)),
           "bf_blocked_pack")
    return Xb


def bf_blocked_unpack(Xb, X, stream=None):
    """Xb: Blocked; X: agent-major 2-D tensor of the same n, d and dtype (written)."""
    ptr, n, d, ld = _mat(X, "X")
    if not isinstance(Xb, Blocked) or Xb.shape != (n, d) or Xb.dtype != X.dtype:
        raise ValueError("Xb must be a Blocked matrix with the shape and dtype of X")
    _check(lib.bf_blocked_unpack(n, d, -Xb.stride(0), Xb.data_ptr(), ld, ptr, _dtype_code(X), _stream(stream)),
           "bf_blocked_unpack")
    return X


def bf_recommended_ld(d, dt):
    ld = lib.bf_recommended_ld(d, dt)
    if ld < 0:
        raise BfError(int(ld), "bf_recommended_ld")
    return ld


def bf_set_tuning(knob, value):
    _check(lib.bf_set_tuning(knob, value), "bf_set_tuning")
