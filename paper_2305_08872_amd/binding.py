"""ctypes binding over the C ABI of libamulet.so (argument marshalling only).

Each function has the name of the C entry point it calls.  Tensor arguments
are torch tensors already resident on the GPU; the binding takes their data
pointers, row strides and the current torch stream and passes them through.
There is no fallback: if the shared library has not been built, every call
raises.
"""
from __future__ import annotations

import ctypes
import os

AMULET_IDENTITY, AMULET_DISCOUNT, AMULET_BOOST, AMULET_COUNT_GT = 0, 1, 2, 3
AMULET_TASK_COUNT_I8 = 100
AMULET_THRES_COL, AMULET_THRES_ROW, AMULET_THRES_CONST, AMULET_THRES_ELEM = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libamulet.so")
_lib = None


class AmuletError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = ""
        if code == -5 and _lib is not None:
            detail = ": " + _lib.amulet_last_launch_error().decode()
        super().__init__("%s failed: %s (status %d)%s" % (where, amulet_strerror(code), code, detail))


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libamulet.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            "libamulet.so is missing at %s: build it with "
            "`python -m paper_2305_08872_amd.build` (needs hipcc); there is no fallback path"
            % _LIB_PATH)
    # torch ships its own HIP runtime (same soname as the system one): import it
    # first so that libamulet.so binds to the runtime torch's allocations and
    # streams live in, instead of bringing a second runtime into the process.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
    lib.amulet_mmlike_f32.restype = i32
    lib.amulet_mmlike_f32.argtypes = [i32, i64, i64, i64, vp, i64, vp, i64, vp, vp, i64, vp]
    lib.amulet_mmlike_f32_shape.restype = i32
    lib.amulet_mmlike_f32_shape.argtypes = [i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, vp, i64, vp]
    lib.amulet_mmlike_f64.restype = i32
    lib.amulet_mmlike_f64.argtypes = [i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, vp, i64, vp]
    lib.amulet_mmlike_f64_general.restype = i32
    lib.amulet_mmlike_f64_general.argtypes = [i32, i32, i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, vp,
                                              i64, vp]
    lib.amulet_mmlike_f32_general.restype = i32
    lib.amulet_mmlike_f32_general.argtypes = [i32, i32, i32, i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64,
                                              vp, vp, i64, vp]
    lib.amulet_mmlike_f32_adaptive.restype = i32
    lib.amulet_mmlike_f32_adaptive.argtypes = [i32, i64, i64, i64, vp, i64, vp, i64, vp, vp, i64, vp,
                                               ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.amulet_mmlike_f32_adaptive_general.restype = i32
    lib.amulet_mmlike_f32_adaptive_general.argtypes = [i32, i32, i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64,
                                                       vp, vp, i64, vp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.amulet_count_i8.restype = i32
    lib.amulet_count_i8.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp]
    lib.amulet_count_i8_adaptive.restype = i32
    lib.amulet_count_i8_adaptive.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, ctypes.POINTER(ctypes.c_int),
                                             ctypes.POINTER(ctypes.c_int)]
    lib.amulet_pitch_collides.restype = i32
    lib.amulet_pitch_collides.argtypes = [i64, i32]
    lib.amulet_packed_ld.restype = i64
    lib.amulet_packed_ld.argtypes = [i64, i32]
    lib.amulet_pack.restype = i32
    lib.amulet_pack.argtypes = [i32, i64, i64, vp, i64, vp, i64, vp]
    lib.amulet_autopack_workspace_bytes.restype = ctypes.c_size_t
    lib.amulet_autopack_workspace_bytes.argtypes = [i32, i64, i64]
    lib.amulet_mmlike_f32_autopack.restype = i32
    lib.amulet_mmlike_f32_autopack.argtypes = [i32, i32, i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, vp,
                                               i64, vp, ctypes.c_size_t, vp]
    lib.amulet_mmlike_f64_shape.restype = i32
    lib.amulet_mmlike_f64_shape.argtypes = [i32, i32, i32, i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, vp,
                                            i64, vp]
    lib.amulet_mmlike_f64_adaptive.restype = i32
    lib.amulet_mmlike_f64_adaptive.argtypes = [i32, i32, i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, vp,
                                               i64, vp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    lib.amulet_f64_shape_count.restype = i32
    lib.amulet_f64_shape_count.argtypes = []
    lib.amulet_f64_shape_name.restype = ctypes.c_char_p
    lib.amulet_f64_shape_name.argtypes = [i32]
    lib.amulet_selected_shape_f64.restype = i32
    lib.amulet_selected_shape_f64.argtypes = [i32, i64, i64, i64]
    lib.amulet_mmlike_f64_autopack.restype = i32
    lib.amulet_mmlike_f64_autopack.argtypes = lib.amulet_mmlike_f32_autopack.argtypes
    lib.amulet_count_i8_workspace_bytes.restype = ctypes.c_size_t
    lib.amulet_count_i8_workspace_bytes.argtypes = [i32, i32, i64, i64, i64]
    lib.amulet_count_i8_repack_workspace_bytes.restype = ctypes.c_size_t
    lib.amulet_count_i8_repack_workspace_bytes.argtypes = [i64, i64, i64]
    lib.amulet_count_i8_general.restype = i32
    lib.amulet_count_i8_general.argtypes = [i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, ctypes.c_size_t, vp]
    lib.amulet_count_i8_static.restype = i32
    lib.amulet_count_i8_static.argtypes = [i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp]
    lib.amulet_count_i8_shape.restype = i32
    lib.amulet_count_i8_shape.argtypes = [i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp]
    lib.amulet_count_i8_assign.restype = i32
    lib.amulet_count_i8_assign.argtypes = [i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp]
    lib.amulet_tune.restype = i32
    lib.amulet_tune.argtypes = [i32, i64, i64, i64, vp]
    lib.amulet_shape_count.restype = i32
    lib.amulet_shape_count.argtypes = [i32]
    lib.amulet_shape_name.restype = ctypes.c_char_p
    lib.amulet_shape_name.argtypes = [i32, i32]
    lib.amulet_selected_shape.restype = i32
    lib.amulet_selected_shape.argtypes = [i32, i64, i64, i64]
    lib.amulet_clear_selections.restype = None
    lib.amulet_clear_selections.argtypes = []
    lib.amulet_greedy_search.restype = i32
    lib.amulet_greedy_search.argtypes = [i32, i32, _SCORE_FN, vp, ctypes.POINTER(i32),
                                         ctypes.POINTER(i32)]
    lib.amulet_register_demand.restype = i32
    lib.amulet_register_demand.argtypes = [i32] * 8
    lib.amulet_choose_kernel_height.restype = i32
    lib.amulet_choose_kernel_height.argtypes = [i32] * 9
    lib.amulet_probe_valu.restype = i32
    lib.amulet_probe_valu.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_double), vp]
    lib.amulet_tile_grid.restype = i64
    lib.amulet_tile_grid.argtypes = [i64, i64]
    lib.amulet_tile_of_workgroup.restype = i32
    lib.amulet_tile_of_workgroup.argtypes = [i64, i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.amulet_probe_mfma_i8.restype = i32
    lib.amulet_probe_mfma_i8.argtypes = [i32, ctypes.POINTER(ctypes.c_double), vp]
    lib.amulet_strerror.restype = ctypes.c_char_p
    lib.amulet_strerror.argtypes = [i32]
    lib.amulet_last_launch_error.restype = ctypes.c_char_p
    lib.amulet_last_launch_error.argtypes = []
    lib.amulet_set_deterministic.restype = None
    lib.amulet_set_deterministic.argtypes = [i32]
    lib.amulet_get_deterministic.restype = i32
    lib.amulet_get_deterministic.argtypes = []
    lib.amulet_debug_fail_launches.restype = None
    lib.amulet_debug_fail_launches.argtypes = [i32]
    lib.amulet_version.restype = ctypes.c_char_p
    lib.amulet_version.argtypes = []
    _lib = lib
    return lib


_SCORE_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_void_p)


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _mat(t, dtype_name: str, what: str):
    """(data_ptr, rows, cols, leading dimension in elements) of a 2-D device tensor."""
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % what)
    if t.dim() != 2 or str(t.dtype) != dtype_name:
        raise ValueError("%s must be a 2-D %s tensor" % (what, dtype_name))
    rows, cols = t.shape
    if cols > 1 and t.stride(1) != 1:
        raise ValueError("%s must have unit column stride" % what)
    ld = t.stride(0) if rows > 1 else max(cols, 1)
    return t.data_ptr(), rows, cols, max(ld, 1)


def _params_ptr(task: int, params, N: int):
    n_rows = {AMULET_IDENTITY: 0, AMULET_DISCOUNT: 2, AMULET_BOOST: 1, AMULET_COUNT_GT: 1}.get(task, 0)
    if n_rows == 0 or params is None:
        return None
    if not params.is_cuda or str(params.dtype) != "torch.float32" or not params.is_contiguous() \
            or params.numel() != n_rows * N:
        raise ValueError("params must be a contiguous fp32 device tensor of %d x %d" % (n_rows, N))
    return params.data_ptr()


def _check(rc: int, where: str):
    if rc < 0:
        raise AmuletError(rc, where)
    return rc


def amulet_mmlike_f32(task: int, A, B, params, R, stream=None):
    """R += sum_k g(A[i,k]*B[k,j], params[:, j]) on the GPU, in place; enqueues and returns."""
    lib = load_library()
    pa, M, K, lda = _mat(A, "torch.float32", "A")
    pb, K2, N, ldb = _mat(B, "torch.float32", "B")
    pr, M2, N2, ldr = _mat(R, "torch.float32", "R")
    if K2 != K or M2 != M or N2 != N:
        raise ValueError("shape mismatch: A %dx%d, B %dx%d, R %dx%d" % (M, K, K2, N, M2, N2))
    _check(lib.amulet_mmlike_f32(task, M, N, K, pa, lda, pb, ldb, _params_ptr(task, params, N), pr, ldr,
                                 _stream_ptr(stream)), "amulet_mmlike_f32")


def amulet_mmlike_f32_adaptive(task: int, A, B, params, R, stream=None):
    """R += task(A, B, params) with the paper's in-flight adaptive execution: trial tile shapes
    run on row slabs of this very task.  Returns (chosen shape id, number of trial slabs)."""
    lib = load_library()
    pa, M, K, lda = _mat(A, "torch.float32", "A")
    pb, K2, N, ldb = _mat(B, "torch.float32", "B")
    pr, M2, N2, ldr = _mat(R, "torch.float32", "R")
    if K2 != K or M2 != M or N2 != N:
        raise ValueError("shape mismatch: A %dx%d, B %dx%d, R %dx%d" % (M, K, K2, N, M2, N2))
    chosen, trials = ctypes.c_int(-1), ctypes.c_int(0)
    _check(lib.amulet_mmlike_f32_adaptive(task, M, N, K, pa, lda, pb, ldb, _params_ptr(task, params, N), pr,
                                          ldr, _stream_ptr(stream), ctypes.byref(chosen), ctypes.byref(trials)),
           "amulet_mmlike_f32_adaptive")
    return chosen.value, trials.value


def amulet_mmlike_f32_shape(task: int, shape: int, A, B, params, R, stream=None):
    lib = load_library()
    pa, M, K, lda = _mat(A, "torch.float32", "A")
    pb, K2, N, ldb = _mat(B, "torch.float32", "B")
    pr, M2, N2, ldr = _mat(R, "torch.float32", "R")
    if K2 != K or M2 != M or N2 != N:
        raise ValueError("shape mismatch: A %dx%d, B %dx%d, R %dx%d" % (M, K, K2, N, M2, N2))
    _check(lib.amulet_mmlike_f32_shape(task, shape, M, N, K, pa, lda, pb, ldb,
                                       _params_ptr(task, params, N), pr, ldr, _stream_ptr(stream)),
           "amulet_mmlike_f32_shape")


def _general_args(dtype_name: str, task: int, A, B, thres, dis, R, thres_form: int, trans_a: bool,
                  trans_b: bool):
    """Pointers, sizes and pitches of a general-form call, in the order the C entry points take
    them from M on: (M, N, K, A, lda, B, ldb, thres, ldt, dis, R, ldr)."""
    pa, ra, ca, lda = _mat(A, dtype_name, "A")
    pb, rb, cb, ldb = _mat(B, dtype_name, "B")
    pr, M, N, ldr = _mat(R, dtype_name, "R")
    Ma, K = (ca, ra) if trans_a else (ra, ca)
    K2, Nb = (cb, rb) if trans_b else (rb, cb)
    if K2 != K or Ma != M or Nb != N:
        raise ValueError("shape mismatch between A, B and R")
    pt, ldt = None, 0
    if task != AMULET_IDENTITY:
        if thres is None or not thres.is_cuda or str(thres.dtype) != dtype_name:
            raise ValueError("thres must be a device tensor of the operands' type")
        if thres_form == AMULET_THRES_ELEM:
            pt, tm, tn, ldt = _mat(thres, dtype_name, "thres")
            if (tm, tn) != (M, N):
                raise ValueError("thres[i][j] must be M x N")
        else:
            want = {AMULET_THRES_COL: N, AMULET_THRES_ROW: M, AMULET_THRES_CONST: 1}[thres_form]
            if not thres.is_contiguous() or thres.numel() != want:
                raise ValueError("thres must hold %d contiguous values" % want)
            pt = thres.data_ptr()
    pd = None
    if task == AMULET_DISCOUNT:
        if dis is None or not dis.is_cuda or str(dis.dtype) != dtype_name or not dis.is_contiguous() \
                or dis.numel() != N:
            raise ValueError("dis must hold N contiguous values of the operands' type on the device")
        pd = dis.data_ptr()
    return M, N, K, pa, lda, pb, ldb, pt, ldt, pd, pr, ldr


def amulet_mmlike_f32_general(task: int, A, B, thres, dis, R, *, thres_form: int = AMULET_THRES_COL,
                              trans_a: bool = False, trans_b: bool = False, shape: int = -1, stream=None):
    """General test-query form: A may be stored K x M (trans_a), B N x K (trans_b); `thres` is a
    device tensor of N, M, 1 or M x N values according to `thres_form`; `dis` has N values."""
    lib = load_library()
    args = _general_args("torch.float32", task, A, B, thres, dis, R, thres_form, trans_a, trans_b)
    _check(lib.amulet_mmlike_f32_general(task, thres_form, int(trans_a), int(trans_b), shape, *args,
                                         _stream_ptr(stream)), "amulet_mmlike_f32_general")


def amulet_mmlike_f32_adaptive_general(task: int, A, B, thres, dis, R, *, thres_form: int = AMULET_THRES_COL,
                                       trans_a: bool = False, trans_b: bool = False, stream=None):
    """The general test-query form with the paper's in-flight adaptive execution.  Returns
    (chosen shape id, number of trial slabs)."""
    lib = load_library()
    args = _general_args("torch.float32", task, A, B, thres, dis, R, thres_form, trans_a, trans_b)
    chosen, trials = ctypes.c_int(-1), ctypes.c_int(0)
    _check(lib.amulet_mmlike_f32_adaptive_general(task, thres_form, int(trans_a), int(trans_b), *args,
                                                  _stream_ptr(stream), ctypes.byref(chosen), ctypes.byref(trials)),
           "amulet_mmlike_f32_adaptive_general")
    return chosen.value, trials.value


def amulet_mmlike_f64(task: int, A, B, thres, dis, R, *, thres_form: int = AMULET_THRES_COL,
                      trans_a: bool = False, trans_b: bool = False, shape: int = -1, stream=None):
    """The tasks in the paper's own element type: fp64 device tensors; A may be stored K x M
    (trans_a), B N x K (trans_b); `thres` holds N, M, 1 or M x N values according to
    `thres_form`; `dis` has N values; `shape` -1 is the selected (else the built-in) fp64 shape."""
    lib = load_library()
    args = _general_args("torch.float64", task, A, B, thres, dis, R, thres_form, trans_a, trans_b)
    _check(lib.amulet_mmlike_f64_shape(task, shape, thres_form, int(trans_a), int(trans_b), *args,
                                       _stream_ptr(stream)), "amulet_mmlike_f64_shape")


def amulet_mmlike_f64_adaptive(task: int, A, B, thres, dis, R, *, thres_form: int = AMULET_THRES_COL,
                               trans_a: bool = False, trans_b: bool = False, stream=None):
    """The fp64 tasks with the paper's in-flight adaptive execution.  Returns (chosen fp64 shape
    id, number of trial slabs)."""
    lib = load_library()
    args = _general_args("torch.float64", task, A, B, thres, dis, R, thres_form, trans_a, trans_b)
    chosen, trials = ctypes.c_int(-1), ctypes.c_int(0)
    _check(lib.amulet_mmlike_f64_adaptive(task, thres_form, int(trans_a), int(trans_b), *args, _stream_ptr(stream),
                                          ctypes.byref(chosen), ctypes.byref(trials)), "amulet_mmlike_f64_adaptive")
    return chosen.value, trials.value


def amulet_f64_shape_count() -> int:
    return int(load_library().amulet_f64_shape_count())


def amulet_f64_shape_name(shape: int) -> str:
    return load_library().amulet_f64_shape_name(shape).decode()


def amulet_selected_shape_f64(task: int, M: int, N: int, K: int) -> int:
    """The fp64 shape a plain call would use for this size (cached selection, else built-in)."""
    return _check(load_library().amulet_selected_shape_f64(task, M, N, K), "amulet_selected_shape_f64")


def amulet_pitch_collides(ld: int, elem_bytes: int) -> bool:
    """True if rows `ld` elements apart fall into the same cache sets and memory channel."""
    return bool(load_library().amulet_pitch_collides(ld, elem_bytes))


def amulet_packed_ld(cols: int, elem_bytes: int) -> int:
    """Row pitch, in elements, of a packed copy of rows of `cols` elements."""
    return int(load_library().amulet_packed_ld(cols, elem_bytes))


def amulet_autopack_workspace_bytes(elem_bytes: int, M: int, K: int) -> int:
    """Bytes of workspace an auto-packing call on an M x K operand A may need."""
    return int(load_library().amulet_autopack_workspace_bytes(elem_bytes, M, K))


def amulet_pack(src, dst, stream=None):
    """Copy the 2-D device tensor `src` into `dst` (same shape and element size, any row
    pitches); enqueues and returns."""
    lib = load_library()
    if not (src.is_cuda and dst.is_cuda) or src.dim() != 2 or dst.shape != src.shape or \
            src.element_size() != dst.element_size():
        raise ValueError("src and dst must be 2-D device tensors of one shape and element size")
    if (src.shape[1] > 1 and src.stride(1) != 1) or (dst.shape[1] > 1 and dst.stride(1) != 1):
        raise ValueError("rows must be contiguous")
    rows, cols = int(src.shape[0]), int(src.shape[1])
    _check(lib.amulet_pack(src.element_size(), rows, cols, src.data_ptr(), int(src.stride(0)) if rows > 1 else cols,
                           dst.data_ptr(), int(dst.stride(0)) if rows > 1 else cols, _stream_ptr(stream)),
           "amulet_pack")


def _autopack(fn_name: str, dtype_name: str, task, A, B, thres, dis, R, workspace, thres_form, trans_a, trans_b,
              stream):
    lib = load_library()
    args = _general_args(dtype_name, task, A, B, thres, dis, R, thres_form, trans_a, trans_b)
    pw, nw = None, 0
    if workspace is not None:
        if not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous device tensor")
        pw, nw = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    _check(getattr(lib, fn_name)(task, thres_form, int(trans_a), int(trans_b), *args, pw, nw,
                                 _stream_ptr(stream)), fn_name)


def amulet_mmlike_f32_autopack(task: int, A, B, thres, dis, R, workspace, *, thres_form: int = AMULET_THRES_COL,
                               trans_a: bool = False, trans_b: bool = False, stream=None):
    """amulet_mmlike_f32_general with packing allowed: `workspace` (any contiguous device tensor
    of at least amulet_autopack_workspace_bytes(4, M, K) bytes, or None) may receive a packed
    copy of A that the task then reads."""
    _autopack("amulet_mmlike_f32_autopack", "torch.float32", task, A, B, thres, dis, R, workspace, thres_form,
              trans_a, trans_b, stream)


def amulet_mmlike_f64_autopack(task: int, A, B, thres, dis, R, workspace, *, thres_form: int = AMULET_THRES_COL,
                               trans_a: bool = False, trans_b: bool = False, stream=None):
    """amulet_mmlike_f64 with packing allowed (see amulet_mmlike_f32_autopack; 8-byte elements)."""
    _autopack("amulet_mmlike_f64_autopack", "torch.float64", task, A, B, thres, dis, R, workspace, thres_form,
              trans_a, trans_b, stream)


def amulet_count_i8(A, B, R, stream=None):
    """R += A @ B for int8 A, B and int32 R on the GPU, exact; enqueues and returns."""
    lib = load_library()
    pa, M, K, lda = _mat(A, "torch.int8", "A")
    pb, K2, N, ldb = _mat(B, "torch.int8", "B")
    pr, M2, N2, ldr = _mat(R, "torch.int32", "R")
    if K2 != K or M2 != M or N2 != N:
        raise ValueError("shape mismatch: A %dx%d, B %dx%d, R %dx%d" % (M, K, K2, N, M2, N2))
    _check(lib.amulet_count_i8(M, N, K, pa, lda, pb, ldb, pr, ldr, _stream_ptr(stream)),
           "amulet_count_i8")


def amulet_count_i8_adaptive(A, B, R, stream=None):
    """amulet_count_i8 with the paper's in-flight adaptive execution: the matrix-core kernels are
    tried on slabs of rows of R, the rest runs with the fastest.  Returns (chosen shape id, number
    of trial slabs)."""
    lib = load_library()
    pa, M, K, lda = _mat(A, "torch.int8", "A")
    pb, K2, N, ldb = _mat(B, "torch.int8", "B")
    pr, M2, N2, ldr = _mat(R, "torch.int32", "R")
    if K2 != K or M2 != M or N2 != N:
        raise ValueError("shape mismatch: A %dx%d, B %dx%d, R %dx%d" % (M, K, K2, N, M2, N2))
    chosen, trials = ctypes.c_int(-1), ctypes.c_int(0)
    _check(lib.amulet_count_i8_adaptive(M, N, K, pa, lda, pb, ldb, pr, ldr, _stream_ptr(stream), ctypes.byref(chosen),
                                        ctypes.byref(trials)), "amulet_count_i8_adaptive")
    return chosen.value, trials.value


def amulet_count_i8_workspace_bytes(trans_a: bool, trans_b: bool, M: int, N: int, K: int) -> int:
    """Bytes of workspace amulet_count_i8_general needs for these layouts (0 for row-major)."""
    return int(load_library().amulet_count_i8_workspace_bytes(int(trans_a), int(trans_b), M, N, K))


def amulet_count_i8_repack_workspace_bytes(M: int, N: int, K: int) -> int:
    """Bytes of workspace with which amulet_count_i8_general also gives unaligned operands, or
    operands whose K is not a multiple of 64, an aligned, zero-padded home."""
    return int(load_library().amulet_count_i8_repack_workspace_bytes(M, N, K))


def amulet_count_i8_general(A, B, R, workspace=None, *, trans_a: bool = False, trans_b: bool = False, stream=None):
    """The join count with A stored K x M (trans_a) and / or B stored N x K (trans_b); `workspace`
    is a contiguous device tensor of at least amulet_count_i8_workspace_bytes(...) bytes, or of
    amulet_count_i8_repack_workspace_bytes(...) to have unaligned operands re-pitched as well."""
    lib = load_library()
    pa, ra, ca, lda = _mat(A, "torch.int8", "A")
    pb, rb, cb, ldb = _mat(B, "torch.int8", "B")
    pr, M, N, ldr = _mat(R, "torch.int32", "R")
    Ma, K = (ca, ra) if trans_a else (ra, ca)
    K2, Nb = (cb, rb) if trans_b else (rb, cb)
    if K2 != K or Ma != M or Nb != N:
        raise ValueError("shape mismatch between A, B and R")
    pw, nw = None, 0
    if workspace is not None:
        if not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous device tensor")
        pw, nw = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    _check(lib.amulet_count_i8_general(int(trans_a), int(trans_b), M, N, K, pa, lda, pb, ldb, pr, ldr, pw, nw,
                                       _stream_ptr(stream)), "amulet_count_i8_general")


AMULET_STATIC_SCRATCH_BYTES = 32 << 20


def amulet_count_i8_static(A, B, R, *, trans_a: bool = False, trans_b: bool = False, stream=None):
    """amulet_count_i8_general without a workspace argument: the copies go into the library's own
    static device array (AMULET_STATIC_SCRATCH_BYTES); the call allocates nothing."""
    lib = load_library()
    pa, ra, ca, lda = _mat(A, "torch.int8", "A")
    pb, rb, cb, ldb = _mat(B, "torch.int8", "B")
    pr, M, N, ldr = _mat(R, "torch.int32", "R")
    Ma, K = (ca, ra) if trans_a else (ra, ca)
    K2, Nb = (cb, rb) if trans_b else (rb, cb)
    if K2 != K or Ma != M or Nb != N:
        raise ValueError("shape mismatch between A, B and R")
    _check(lib.amulet_count_i8_static(int(trans_a), int(trans_b), M, N, K, pa, lda, pb, ldb, pr, ldr,
                                      _stream_ptr(stream)), "amulet_count_i8_static")


def amulet_count_i8_shape(shape: int, A, B, R, stream=None):
    lib = load_library()
    pa, M, K, lda = _mat(A, "torch.int8", "A")
    pb, K2, N, ldb = _mat(B, "torch.int8", "B")
    pr, M2, N2, ldr = _mat(R, "torch.int32", "R")
    if K2 != K or M2 != M or N2 != N:
        raise ValueError("shape mismatch: A %dx%d, B %dx%d, R %dx%d" % (M, K, K2, N, M2, N2))
    _check(lib.amulet_count_i8_shape(shape, M, N, K, pa, lda, pb, ldb, pr, ldr, _stream_ptr(stream)),
           "amulet_count_i8_shape")


def amulet_count_i8_assign(A, B, R, shape: int = -1, stream=None):
    """R = A @ B for int8 A, B and int32 R on the GPU, exact: the counts are written, whatever R
    held before; `shape` -1 is the selected shape.  Enqueues and returns."""
    lib = load_library()
    pa, M, K, lda = _mat(A, "torch.int8", "A")
    pb, K2, N, ldb = _mat(B, "torch.int8", "B")
    pr, M2, N2, ldr = _mat(R, "torch.int32", "R")
    if K2 != K or M2 != M or N2 != N:
        raise ValueError("shape mismatch: A %dx%d, B %dx%d, R %dx%d" % (M, K, K2, N, M2, N2))
    _check(lib.amulet_count_i8_assign(shape, M, N, K, pa, lda, pb, ldb, pr, ldr, _stream_ptr(stream)),
           "amulet_count_i8_assign")


def amulet_tune(task: int, M: int, N: int, K: int, stream=None) -> int:
    """Time the task's tile shapes at this size, cache and return the winner's id."""
    return _check(load_library().amulet_tune(task, M, N, K, _stream_ptr(stream)), "amulet_tune")


def amulet_shape_count(task: int) -> int:
    return load_library().amulet_shape_count(task)


def amulet_shape_name(task: int, shape: int) -> str:
    return load_library().amulet_shape_name(task, shape).decode()


def amulet_selected_shape(task: int, M: int, N: int, K: int) -> int:
    return _check(load_library().amulet_selected_shape(task, M, N, K), "amulet_selected_shape")


def amulet_clear_selections() -> None:
    load_library().amulet_clear_selections()


def amulet_greedy_search(n0: int, n1: int, score):
    """Run the library's two-stage greedy search with a Python score(i0, i1) callback.
    Returns (best0, best1, number of score calls)."""
    lib = load_library()
    cb = _SCORE_FN(lambda i0, i1, _ctx: float(score(i0, i1)))
    b0, b1 = ctypes.c_int(-1), ctypes.c_int(-1)
    calls = _check(lib.amulet_greedy_search(n0, n1, cb, None, ctypes.byref(b0), ctypes.byref(b1)),
                   "amulet_greedy_search")
    return b0.value, b1.value, calls


def amulet_register_demand(I_h, I_w, S_w, n_const, n_i, n_j, n_ij, n_temp) -> int:
    return _check(load_library().amulet_register_demand(I_h, I_w, S_w, n_const, n_i, n_j, n_ij, n_temp),
                  "amulet_register_demand")


def amulet_choose_kernel_height(I_h_max, I_w, S_w, n_const, n_i, n_j, n_ij, n_temp, budget) -> int:
    return _check(load_library().amulet_choose_kernel_height(I_h_max, I_w, S_w, n_const, n_i, n_j, n_ij,
                                                             n_temp, budget),
                  "amulet_choose_kernel_height")


def amulet_probe_valu(mix: int, waves_per_simd: int, stream=None) -> float:
    """Sustained products/s of a register-only loop of a task's instruction mix."""
    out = ctypes.c_double(0.0)
    _check(load_library().amulet_probe_valu(mix, waves_per_simd, ctypes.byref(out), _stream_ptr(stream)),
           "amulet_probe_valu")
    return out.value


def amulet_tile_grid(tiles_m: int, tiles_n: int) -> int:
    """Workgroups launched for a tiles_m x tiles_n grid of R tiles (padding included)."""
    return load_library().amulet_tile_grid(tiles_m, tiles_n)


def amulet_tile_of_workgroup(block: int, tiles_m: int, tiles_n: int):
    """(tm, tn) of workgroup `block`, or None when that workgroup is padding."""
    tm, tn = ctypes.c_int64(0), ctypes.c_int64(0)
    rc = _check(load_library().amulet_tile_of_workgroup(block, tiles_m, tiles_n, ctypes.byref(tm), ctypes.byref(tn)),
                "amulet_tile_of_workgroup")
    return (tm.value, tn.value) if rc == 1 else None


def amulet_probe_mfma_i8(waves_per_simd: int, stream=None) -> float:
    """Sustained int8 multiply-adds/s of a register-only loop of the join count's matrix-core instruction."""
    out = ctypes.c_double(0.0)
    _check(load_library().amulet_probe_mfma_i8(waves_per_simd, ctypes.byref(out), _stream_ptr(stream)),
           "amulet_probe_mfma_i8")
    return out.value


def amulet_strerror(code: int) -> str:
    if _lib is None and not os.path.exists(_LIB_PATH):
        return "status %d" % code
    return load_library().amulet_strerror(code).decode()


def amulet_last_launch_error() -> str:
    return load_library().amulet_last_launch_error().decode()


def amulet_set_deterministic(on: bool) -> None:
    """No launch splits K while on: floating-point results are reproducible bit for bit."""
    load_library().amulet_set_deterministic(int(bool(on)))


def amulet_get_deterministic() -> bool:
    return bool(load_library().amulet_get_deterministic())


def amulet_debug_fail_launches(n: int) -> None:
    """Test seam: the next n kernel launches are refused on the host and reported as failed."""
    load_library().amulet_debug_fail_launches(int(n))


def amulet_version() -> str:
    return load_library().amulet_version().decode()
