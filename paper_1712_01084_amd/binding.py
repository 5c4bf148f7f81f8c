"""ctypes binding of libpivotfc.so: the same entry points as include/pivot_fc.h,
argument marshalling only.  Every step of the path runs inside the library's
HIP kernels; there is no CPU fallback and a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpivotfc.so")

PIVOT_F32, PIVOT_F16 = 0, 1
PIVOT_BRC, PIVOT_BCR, PIVOT_CBR = 0, 1, 2
PIVOT_PLAN_GATHER_FROM_GLOBAL = 1
PIVOT_PLAN_LSTM_LAUNCH_PER_STEP = 2
PIVOT_PLAN_GATHER_FROM_LDS_COPY = 4
PIVOT_PLAN_LSTM_ONE_LAUNCH_ALWAYS = 8
PIVOT_ACT_NONE, PIVOT_ACT_RELU = 0, 1
PIVOT_W_NATURAL, PIVOT_W_PIVOTED = 0, 1
PIVOT_MLP_KEEP_FINAL_BLOCK_ORDER = 1
PIVOT_MLP_LAUNCH_PER_LAYER = 2

PIVOT_OK = 0
PIVOT_E_NULL, PIVOT_E_SHAPE, PIVOT_E_NOT_PERMUTATION, PIVOT_E_UNSUPPORTED = -1, -2, -3, -4
PIVOT_E_ALLOC, PIVOT_E_HIP, PIVOT_E_WORKSPACE, PIVOT_E_NO_DEVICE = -5, -6, -7, -8

EXPORTS = [
    "pivot_version", "pivot_last_error",
    "pivot_fc_plan", "pivot_fc_plan_host_view", "pivot_fc_plan_clone", "pivot_fc_plan_destroy",
    "pivot_fc_workspace_bytes", "pivot_workspace_init", "pivot_fc_run", "pivot_fc_run_static", "pivot_fc_kernel_name",
    "pivot_mlp_plan", "pivot_mlp_plan_host_view", "pivot_mlp_plan_destroy",
    "pivot_mlp_workspace_bytes", "pivot_mlp_run", "pivot_mlp_status", "pivot_mlp_status_word",
    "pivot_lstm_workspace_bytes", "pivot_lstm_run", "pivot_lstm_status", "pivot_lstm_status_word",
    "pivot_dense_run", "pivot_csr_run", "pivot_null_run", "pivot_stream_read_run", "pivot_exchange_probe_run", "pivot_feedback_search",
]


class PivotError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("pivot error %d: %s" % (code, text))
        self.code = code


class pivot_fc_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("M", "K", "bh", "bw", "wdtype", "layout", "act", "chunk_tiles", "device", "wg_waves", "row_slices", "flags")]


class pivot_plan_view(C.Structure):
    _fields_ = ([(n, C.c_int32) for n in
                 ("M", "K", "bh", "bw", "wdtype", "layout", "act", "nbr", "nbc", "M_pad", "K_pad",
                  "T", "chunk_tiles", "wg_waves", "row_slices", "nchunks")]
                + [("row_ptr", C.POINTER(C.c_int32)), ("col_idx", C.POINTER(C.c_int32)),
                   ("vals", C.c_void_p), ("bias_p", C.POINTER(C.c_float)),
                   ("invprow", C.POINTER(C.c_int32)), ("invpcol", C.POINTER(C.c_int32)),
                   ("prow_pad", C.POINTER(C.c_int32)), ("pcol_pad", C.POINTER(C.c_int32)),
                   ("chunks", C.POINTER(C.c_int32)), ("part_base", C.POINTER(C.c_int32)),
                   ("xidx", C.POINTER(C.c_int32)), ("xsort", C.POINTER(C.c_int32)),
                   ("xsort_blk", C.POINTER(C.c_int32))])


class pivot_mlp_view(C.Structure):
    _fields_ = [("L", C.c_int32), ("flags", C.c_int32),
                ("q", C.POINTER(C.POINTER(C.c_int32))), ("dst", C.POINTER(C.POINTER(C.c_int32))),
                ("identity", C.POINTER(C.c_int32)), ("one_launch", C.c_int32)]


_lib = None


def lib():
    """Loads libpivotfc.so (built in-tree by paper_1712_01084_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libpivotfc.so is not built: run `python -m paper_1712_01084_amd.build` "
                           "(there is no CPU fallback)")
    # Kernel arguments in device memory instead of host memory: the first
    # scalar load of every wavefront then stays on the device (about 1 us per
    # launch on MI355X).  Only effective if set before the HIP runtime starts.
    os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")
    try:
        import torch  # noqa: F401  -- so that the library binds to the HIP runtime torch already loaded
    except Exception:
        pass
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
    L.pivot_version.restype = C.c_int
    L.pivot_last_error.restype = C.c_char_p
    L.pivot_fc_plan.argtypes = [C.POINTER(pivot_fc_desc), vp, i32, vp, vp, vp, vp, C.POINTER(vp)]
    L.pivot_fc_plan_host_view.argtypes = [vp, C.POINTER(pivot_plan_view)]
    L.pivot_fc_plan_clone.argtypes = [vp, C.POINTER(vp)]
    L.pivot_fc_plan_destroy.argtypes = [vp]
    L.pivot_fc_plan_destroy.restype = None
    L.pivot_fc_workspace_bytes.argtypes = [vp, i32]
    L.pivot_fc_workspace_bytes.restype = sz
    L.pivot_workspace_init.argtypes = [vp, sz, vp]
    L.pivot_fc_run.argtypes = [vp, vp, i64, vp, i64, i32, vp, sz, vp]
    L.pivot_fc_kernel_name.argtypes = [vp, i32, C.c_char_p, sz]
    L.pivot_fc_run_static.argtypes = [vp, vp, i64, vp, i64, i32, vp]
    L.pivot_mlp_plan.argtypes = [C.POINTER(vp), i32, i32, C.POINTER(vp)]
    L.pivot_mlp_plan_host_view.argtypes = [vp, C.POINTER(pivot_mlp_view)]
    L.pivot_mlp_plan_destroy.argtypes = [vp]
    L.pivot_mlp_plan_destroy.restype = None
    L.pivot_mlp_workspace_bytes.argtypes = [vp, i32]
    L.pivot_mlp_workspace_bytes.restype = sz
    L.pivot_mlp_run.argtypes = [vp, vp, i64, vp, i64, i32, vp, sz, vp]
    L.pivot_mlp_status.argtypes = [vp, vp, C.POINTER(C.c_int)]
    L.pivot_mlp_status_word.argtypes = [vp, C.POINTER(vp)]
    L.pivot_lstm_status_word.argtypes = [vp, i32, i32, vp, C.POINTER(vp)]
    L.pivot_lstm_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    L.pivot_lstm_workspace_bytes.restype = sz
    L.pivot_lstm_run.argtypes = [vp, i32, i32, vp, vp, vp, vp, i32, i32, vp, sz, vp]
    L.pivot_lstm_status.argtypes = [vp, i32, i32, vp, vp, C.POINTER(C.c_int)]
    L.pivot_dense_run.argtypes = [vp, i32, i32, i32, vp, i64, vp, vp, i64, i32, i32, vp]
    L.pivot_null_run.argtypes = [vp]
    L.pivot_stream_read_run.argtypes = [vp, sz, vp, vp]
    L.pivot_exchange_probe_run.argtypes = [vp, sz, C.c_int, vp]
    L.pivot_feedback_search.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, C.POINTER(C.c_double)]
    L.pivot_csr_run.argtypes = [vp, vp, vp, i32, i32, i64, vp, vp, vp, i32, vp]
    _lib = L
    return L


def _check(rc):
    if rc != PIVOT_OK:
        raise PivotError(rc, (lib().pivot_last_error() or b"").decode())


def _np_ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def pivot_version():
    return lib().pivot_version()


def pivot_last_error():
    return (lib().pivot_last_error() or b"").decode()


def pivot_fc_plan(M, K, bh, bw, wdtype, W, w_space, tile_mask, prow, pcol, bias, *, layout=PIVOT_BRC,
                  act=PIVOT_ACT_NONE, chunk_tiles=0, device=-1, wg_waves=0, row_slices=0, flags=0):
    """Host numpy arrays in, opaque plan handle out."""
    d = pivot_fc_desc(M, K, bh, bw, wdtype, layout, act, chunk_tiles, device, wg_waves, row_slices, flags)
    W = None if W is None else np.ascontiguousarray(W, dtype=np.float32 if wdtype == PIVOT_F32 else np.float16)
    tile_mask = None if tile_mask is None else np.ascontiguousarray(tile_mask, dtype=np.uint8)
    prow = None if prow is None else np.ascontiguousarray(prow, dtype=np.int32)
    pcol = None if pcol is None else np.ascontiguousarray(pcol, dtype=np.int32)
    bias = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    out = C.c_void_p()
    _check(lib().pivot_fc_plan(C.byref(d), _np_ptr(W), w_space, _np_ptr(tile_mask), _np_ptr(prow), _np_ptr(pcol),
                               _np_ptr(bias), C.byref(out)))
    return out


def pivot_fc_plan_host_view(plan):
    """Copies of the plan's canonical host arrays as numpy arrays."""
    v = pivot_plan_view()
    _check(lib().pivot_fc_plan_host_view(plan, C.byref(v)))

    def arr(ptr, n, dtype):
        if n == 0:
            return np.zeros(0, dtype=dtype)
        return np.ctypeslib.as_array(C.cast(ptr, C.POINTER(C.c_uint8)), shape=(n * np.dtype(dtype).itemsize,)).view(dtype).copy()

    wd = np.float32 if v.wdtype == PIVOT_F32 else np.float16
    out = {k: getattr(v, k) for k in ("M", "K", "bh", "bw", "wdtype", "layout", "act", "nbr", "nbc", "M_pad",
                                      "K_pad", "T", "chunk_tiles", "wg_waves", "row_slices", "nchunks")}
    out["row_ptr"] = arr(v.row_ptr, v.nbr + 1, np.int32)
    out["col_idx"] = arr(v.col_idx, v.T, np.int32)
    out["vals"] = arr(v.vals, v.T * v.bh * v.bw, wd)
    out["bias_p"] = arr(v.bias_p, v.M_pad, np.float32)
    out["invprow"] = arr(v.invprow, v.M, np.int32)
    out["invpcol"] = arr(v.invpcol, v.K, np.int32)
    out["prow_pad"] = arr(v.prow_pad, v.M_pad, np.int32)
    out["pcol_pad"] = arr(v.pcol_pad, v.K_pad, np.int32)
    out["chunks"] = arr(v.chunks, v.nchunks * 4, np.int32).reshape(-1, 4)
    out["part_base"] = arr(v.part_base, v.nbr + 1, np.int32)
    out["xidx"] = arr(v.xidx, v.T * v.bw, np.int32)
    out["xsort"] = arr(v.xsort, v.T * v.bw, np.int32) if v.xsort else None
    out["xsort_blk"] = arr(v.xsort_blk, v.T * v.bw, np.int32) if v.xsort_blk else None
    return out


def pivot_fc_plan_clone(plan):
    out = C.c_void_p()
    _check(lib().pivot_fc_plan_clone(plan, C.byref(out)))
    return out


def pivot_fc_plan_destroy(plan):
    lib().pivot_fc_plan_destroy(plan)


def pivot_fc_workspace_bytes(plan, batch):
    return int(lib().pivot_fc_workspace_bytes(plan, batch))


def pivot_workspace_init(ws_ptr, ws_bytes, stream=None):
    _check(lib().pivot_workspace_init(ws_ptr, ws_bytes, stream))


def pivot_fc_run(plan, x_ptr, ldx, y_ptr, ldy, batch, ws_ptr, ws_bytes, stream=None):
    _check(lib().pivot_fc_run(plan, x_ptr, ldx, y_ptr, ldy, batch, ws_ptr, ws_bytes, stream))


def pivot_fc_kernel_name(plan, batch):
    """Name of the kernel instantiation pivot_fc_run launches for this plan and batch."""
    buf = C.create_string_buffer(256)
    _check(lib().pivot_fc_kernel_name(plan, batch, buf, 256))
    return buf.value.decode()


def pivot_fc_run_static(plan, x_ptr, ldx, y_ptr, ldy, batch, stream=None):
    _check(lib().pivot_fc_run_static(plan, x_ptr, ldx, y_ptr, ldy, batch, stream))


def pivot_mlp_plan(layer_plans, flags=0):
    n = len(layer_plans)
    arr = (C.c_void_p * max(n, 1))(*[p.value if isinstance(p, C.c_void_p) else p for p in layer_plans])
    out = C.c_void_p()
    _check(lib().pivot_mlp_plan(arr, n, flags, C.byref(out)))
    return out


def pivot_mlp_plan_host_view(mlp, layer_views):
    """layer_views: the host views of the layer plans (for array lengths)."""
    v = pivot_mlp_view()
    _check(lib().pivot_mlp_plan_host_view(mlp, C.byref(v)))
    qs, dsts, ident = [], [], []
    for l in range(v.L - 1):
        nq = layer_views[l + 1]["K"]
        nd = layer_views[l]["M_pad"]
        qs.append(np.ctypeslib.as_array(v.q[l], shape=(nq,)).copy())
        dsts.append(np.ctypeslib.as_array(v.dst[l], shape=(nd,)).copy())
        ident.append(int(v.identity[l]))
    return dict(L=v.L, flags=v.flags, q=qs, dst=dsts, identity=ident, one_launch=int(v.one_launch))


def pivot_mlp_plan_destroy(mlp):
    lib().pivot_mlp_plan_destroy(mlp)


def pivot_mlp_workspace_bytes(mlp, batch):
    return int(lib().pivot_mlp_workspace_bytes(mlp, batch))


def pivot_mlp_run(mlp, x_ptr, ldx, y_ptr, ldy, batch, ws_ptr, ws_bytes, stream=None):
    _check(lib().pivot_mlp_run(mlp, x_ptr, ldx, y_ptr, ldy, batch, ws_ptr, ws_bytes, stream))


def pivot_mlp_status(mlp, stream=None):
    """0 if every one-launch run of the chain since the last call completed (synchronises the stream)."""
    st = C.c_int(0)
    _check(lib().pivot_mlp_status(mlp, stream, C.byref(st)))
    return int(st.value)


def pivot_mlp_status_word(mlp):
    """Device address of the chain's status word (0 if the chain has no one-launch form)."""
    out = C.c_void_p()
    _check(lib().pivot_mlp_status_word(mlp, C.byref(out)))
    return out.value or 0


def pivot_lstm_status_word(plan, steps, batch, ws_ptr):
    """Device address of the recurrent run's status word inside its workspace."""
    out = C.c_void_p()
    _check(lib().pivot_lstm_status_word(plan, steps, batch, ws_ptr, C.byref(out)))
    return out.value or 0


def pivot_lstm_workspace_bytes(plan, H, I, steps, batch):
    return int(lib().pivot_lstm_workspace_bytes(plan, H, I, steps, batch))


def pivot_lstm_run(plan, H, I, xs_ptr, h_ptr, c_ptr, z_dbg_ptr, steps, batch, ws_ptr, ws_bytes, stream=None):
    _check(lib().pivot_lstm_run(plan, H, I, xs_ptr, h_ptr, c_ptr, z_dbg_ptr, steps, batch, ws_ptr, ws_bytes, stream))


def pivot_lstm_status(plan, steps, batch, ws_ptr, stream=None):
    """Synchronises the stream; 0 = the last pivot_lstm_run on this workspace completed."""
    st = C.c_int(-1)
    _check(lib().pivot_lstm_status(plan, steps, batch, ws_ptr, stream, C.byref(st)))
    return st.value


def pivot_dense_run(W_ptr, wdtype, M, K, x_ptr, ldx, bias_ptr, y_ptr, ldy, batch, act, stream=None):
    _check(lib().pivot_dense_run(W_ptr, wdtype, M, K, x_ptr, ldx, bias_ptr, y_ptr, ldy, batch, act, stream))


def pivot_null_run(stream=None):
    _check(lib().pivot_null_run(stream))


PIVOT_PROBE_SCRATCH_BYTES = 32768


def pivot_exchange_probe_run(scratch_ptr, scratch_bytes, rounds, stream=None):
    _check(lib().pivot_exchange_probe_run(scratch_ptr, scratch_bytes, rounds, stream))


def pivot_stream_read_run(buf_ptr, nbytes, out_ptr, stream=None):
    _check(lib().pivot_stream_read_run(buf_ptr, nbytes, out_ptr, stream))


def pivot_csr_run(row_ptr_ptr, col_ptr, val_ptr, wdtype, M, nnz, x_ptr, bias_ptr, y_ptr, act, stream=None):
    _check(lib().pivot_csr_run(row_ptr_ptr, col_ptr, val_ptr, wdtype, M, nnz, x_ptr, bias_ptr, y_ptr, act, stream))


def pivot_feedback_search(absW, levels, prow0, pcol0, max_iter=50):
    """Host numpy in, (prow, pcol, captured_mass) out."""
    absW = np.ascontiguousarray(absW, dtype=np.float32)
    M, K = absW.shape
    prow0 = np.ascontiguousarray(prow0, dtype=np.int32)
    pcol0 = np.ascontiguousarray(pcol0, dtype=np.int32)
    prow = np.empty(M, dtype=np.int32)
    pcol = np.empty(K, dtype=np.int32)
    mass = C.c_double(0.0)
    _check(lib().pivot_feedback_search(_np_ptr(absW), M, K, levels, max_iter, _np_ptr(prow0), _np_ptr(pcol0),
                                       _np_ptr(prow), _np_ptr(pcol), C.byref(mass)))
    return prow, pcol, mass.value
