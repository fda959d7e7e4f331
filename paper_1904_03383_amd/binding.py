"""ctypes binding of the tgemm C-ABI (include/tgemm.h).  Argument marshalling only.

Functions mirror the C entry points: ``sgemm`` -> tg_sgemm, ``sgemm_batched`` ->
tg_sgemm_batched, ``tune`` -> tg_tune, and so on.  torch is used for device memory and
the current stream; it performs no arithmetic here.
"""
from __future__ import annotations

import ctypes
import pathlib

_LIB_PATH = pathlib.Path(__file__).resolve().parent / "libtgemm.so"
_lib = None
_workspace = None  # keeps the workspace tensor alive while the library points at it

TG_OK = 0
STATUS_NAMES = {0: "TG_OK", 1: "TG_ERR_INVALID_ARG", 2: "TG_ERR_UNSUPPORTED", 3: "TG_ERR_WORKSPACE",
                4: "TG_ERR_HIP", 5: "TG_ERR_INTERNAL"}

# Every symbol declared in include/tgemm.h: name -> (restype, argtypes)
_i64, _p, _sz, _int, _cstr = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_char_p
SIGNATURES = {
    "tg_sgemm": (_int, [_i64, _i64, _i64, _p, _i64, _p, _i64, _p, _i64, _p]),
    "tg_sgemm_splitk_static": (_int, [_i64, _i64, _i64, _p, _i64, _p, _i64, _p, _i64, _p]),
    "tg_sgemm_batched": (_int, [_i64, _i64, _i64, _i64, _p, _i64, _i64, _p, _i64, _i64, _p, _i64, _i64, _p]),
    "tg_sgemm_strided": (_int, [_i64, _i64, _i64, _p, _i64, _i64, _p, _i64, _i64, _p, _i64, _p]),
    "tg_saxpy": (_int, [_i64, ctypes.c_float, _p, _p, _p, _p]),
    "tg_tune": (_int, [_i64, _i64, _i64, _i64, _p, _i64, _i64, _p, _i64, _i64, _p, _i64, _i64, _p, _int]),
    "tg_set_workspace": (_int, [_p, _sz]),
    "tg_workspace_bytes": (_sz, [_i64, _i64, _i64, _i64]),
    "tg_strided_workspace_bytes": (_sz, [_i64, _i64, _i64, _i64, _i64]),
    "tg_force_config": (_int, [_cstr]),
    "tg_set_math": (_int, [_int]),
    "tg_get_math": (_int, []),
    "tg_get_config": (_int, [_i64, _i64, _i64, _i64, _p, _sz]),
    "tg_num_candidates": (_int, [_i64, _i64, _i64, _i64]),
    "tg_candidate": (_int, [_i64, _i64, _i64, _i64, _int, _p, _sz, _p, _p]),
    "tg_tune_is_launch_bound": (_int, [_i64, _i64, _i64, _i64]),
    "tg_last_config": (_cstr, []),
    "tg_num_kernels": (_int, []),
    "tg_kernel_name": (_int, [_int, _p, _sz]),
    "tg_load_tune_cache": (_int, [_cstr]),
    "tg_save_tune_cache": (_int, [_cstr]),
    "tg_clear_tune_cache": (None, []),
    "tg_status_string": (_cstr, [_int]),
    "tg_last_error": (_cstr, []),
    "tg_version": (_int, []),
}


class TgemmError(RuntimeError):
    def __init__(self, status: int, detail: str):
        self.status = status
        self.status_name = STATUS_NAMES.get(status, f"status {status}")
        super().__init__(f"{self.status_name}: {detail}")


def library_path() -> pathlib.Path:
    return _LIB_PATH


def load_library():
    """Open libtgemm.so (built by ``python -m paper_1904_03383_amd.build``); fail loudly if absent."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_1904_03383_amd.build` "
                "(there is no fallback implementation)")
        # torch is imported first so that libtgemm.so binds to the HIP runtime torch has
        # already loaded (same soname); a second runtime in the process would not see the GPU.
        import torch  # noqa: F401
        lib = ctypes.CDLL(str(_LIB_PATH))
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def poison_library_path() -> pathlib.Path:
    return _LIB_PATH.with_name("libtgemm_poison.so")


def open_library(path):
    """A second, independent instance of the library (e.g. the debug flavour at poison_library_path()), with the
    argument types set; the functions of this module keep using the one load_library() returns."""
    path = pathlib.Path(path)
    if not path.exists():
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_1904_03383_amd.build --poison`")
    import torch  # noqa: F401  (see load_library)
    lib = ctypes.CDLL(str(path))
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


def _check(status: int):
    if status != TG_OK:
        raise TgemmError(status, load_library().tg_last_error().decode())


# torch and the few attributes the per-call path needs, looked up once (a call through this binding is
# launch-bound for small products: every attribute chain dropped from it shows in the per-call time)
_torch = None
_Tensor = None
_f32 = None
_raw_stream = None
_cur_dev = None


def _torch_mod():
    global _torch, _Tensor, _f32, _raw_stream, _cur_dev
    if _torch is None:
        import torch
        _Tensor, _f32 = torch.Tensor, torch.float32
        _raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)   # avoids building a Stream object per call
        _cur_dev = torch.cuda.current_device
        _torch = torch
    return _torch


def _stream_handle(stream=None) -> int:
    """hipStream_t of `stream` (a torch.cuda.Stream) or of torch's current stream, as an integer."""
    if stream is not None:
        return int(stream.cuda_stream)
    torch = _torch or _torch_mod()
    if _raw_stream is not None:
        return int(_raw_stream(_cur_dev()))
    return int(torch.cuda.current_stream().cuda_stream)


def _require_f32_cuda(name, t):
    if _torch is None:
        _torch_mod()
    if not isinstance(t, _Tensor) or t.dtype is not _f32 or not t.is_cuda:
        raise ValueError(f"{name} must be a float32 tensor in device memory")


def _ld(t, rows_dim, cols) -> int:
    """Leading dimension of a row-major matrix view; unit stride along columns required."""
    if t.shape[rows_dim + 1] > 1 and t.stride(rows_dim + 1) != 1:
        raise ValueError("matrices must have unit stride along their rows (row-major)")
    ld = t.stride(rows_dim) if t.shape[rows_dim] > 1 else max(cols, 1)
    return max(int(ld), 1)


def _row_major_ld(t, rows, cols, strides) -> int:
    """Leading dimension of a 2-D row-major view given its (row, column) strides."""
    if cols > 1 and strides[1] != 1:
        raise ValueError("matrices must have unit stride along their rows (row-major)")
    if rows > 1 and strides[0] < cols:
        raise ValueError("rows of a matrix overlap (row stride smaller than the row length)")
    ld = strides[0] if rows > 1 else cols
    return ld if ld > 1 else 1


def sgemm(a, b, out=None, stream=None):
    """C = A.B for 2-D float32 device tensors a (m,k), b (k,n); returns out (m,n).  -> tg_sgemm"""
    torch = _torch or _torch_mod()
    _require_f32_cuda("a", a)
    _require_f32_cuda("b", b)
    sa, sb = a.shape, b.shape
    if len(sa) != 2 or len(sb) != 2 or sa[1] != sb[0]:
        raise ValueError(f"shape mismatch: {tuple(sa)} x {tuple(sb)}")
    m, k = sa
    n = sb[1]
    if out is None:
        out = torch.empty((m, n), dtype=torch.float32, device=a.device)
    else:
        _require_f32_cuda("out", out)
        so = out.shape
        if len(so) != 2 or so[0] != m or so[1] != n:
            raise ValueError("out has the wrong shape")
    st = (_lib or load_library()).tg_sgemm(m, n, k, a.data_ptr(), _row_major_ld(a, m, k, a.stride()),
                                 b.data_ptr(), _row_major_ld(b, k, n, b.stride()),
                                 out.data_ptr(), _row_major_ld(out, m, n, out.stride()), _stream_handle(stream))
    if st != TG_OK:
        _check(st)
    return out


def _elem_strides(t):
    """(row stride, column stride) in elements of a 2-D view, for tg_sgemm_strided.

    A dimension of extent > 1 must have a positive stride: an expanded (stride 0) view has no element-stride
    form, and passing 1 in its place would make the library read past the tensor's storage."""
    for d in (0, 1):
        if t.shape[d] > 1 and t.stride(d) < 1:
            raise ValueError("operands must have positive strides along every dimension of extent > 1 "
                             "(expanded or broadcast views are not supported: materialise them first)")
    rs = int(t.stride(0)) if t.shape[0] > 1 else 1
    cs = int(t.stride(1)) if t.shape[1] > 1 else 1
    return rs, cs


STATIC_SCRATCH_BYTES = 32 << 20   # TG_STATIC_SCRATCH_BYTES


def sgemm_splitk_static(a, b, out=None, stream=None):
    """C = A.B as a split-K product whose partials live in the library's own fixed device array: the entry
    point for callers that cannot allocate (the binding itself allocates `out` only when none is given).
    -> tg_sgemm_splitk_static"""
    torch = _torch or _torch_mod()
    _require_f32_cuda("a", a)
    _require_f32_cuda("b", b)
    sa, sb = a.shape, b.shape
    if len(sa) != 2 or len(sb) != 2 or sa[1] != sb[0]:
        raise ValueError(f"shape mismatch: {tuple(sa)} x {tuple(sb)}")
    m, k = sa
    n = sb[1]
    if out is None:
        out = torch.empty((m, n), dtype=torch.float32, device=a.device)
    else:
        _require_f32_cuda("out", out)
        if tuple(out.shape) != (m, n):
            raise ValueError("out has the wrong shape")
    _check((_lib or load_library()).tg_sgemm_splitk_static(
        m, n, k, a.data_ptr(), _row_major_ld(a, m, k, a.stride()), b.data_ptr(), _row_major_ld(b, k, n, b.stride()),
        out.data_ptr(), _row_major_ld(out, m, n, out.stride()), _stream_handle(stream)))
    return out


def sgemm_strided(a, b, out=None, stream=None):
    """C = A.B for 2-D float32 device tensors with any positive strides (views such as a[:, ::32] or a.T).

    out, if given, must be row-major (unit stride along its rows).  -> tg_sgemm_strided
    """
    import torch
    _require_f32_cuda("a", a)
    _require_f32_cuda("b", b)
    if a.dim() != 2 or b.dim() != 2 or a.shape[1] != b.shape[0]:
        raise ValueError(f"shape mismatch: {tuple(a.shape)} x {tuple(b.shape)}")
    m, k = a.shape
    n = b.shape[1]
    if out is None:
        out = torch.empty((m, n), dtype=torch.float32, device=a.device)
    _require_f32_cuda("out", out)
    if tuple(out.shape) != (m, n):
        raise ValueError("out has the wrong shape")

    rsa, csa = _elem_strides(a)
    rsb, csb = _elem_strides(b)
    if csa == 1:
        rsa = max(rsa, k, 1)
    if csb == 1:
        rsb = max(rsb, n, 1)
    _check(load_library().tg_sgemm_strided(m, n, k, a.data_ptr(), rsa, csa, b.data_ptr(), rsb, csb,
                                           out.data_ptr(), _ld(out, 0, n), _stream_handle(stream)))
    return out


def saxpy(alpha: float, x, y, out=None, stream=None):
    """out = alpha * x + y for 1-D contiguous float32 device tensors; out may be y or x.  -> tg_saxpy"""
    import torch
    _require_f32_cuda("x", x)
    _require_f32_cuda("y", y)
    if x.dim() != 1 or y.dim() != 1 or x.numel() != y.numel() or not x.is_contiguous() or not y.is_contiguous():
        raise ValueError("x and y must be contiguous 1-D tensors of equal length")
    if out is None:
        out = torch.empty_like(y)
    _require_f32_cuda("out", out)
    if out.dim() != 1 or out.numel() != x.numel() or not out.is_contiguous():
        raise ValueError("out has the wrong shape")
    _check(load_library().tg_saxpy(x.numel(), float(alpha), x.data_ptr(), y.data_ptr(), out.data_ptr(),
                                   _stream_handle(stream)))
    return out


def _batched_args(a, b, out):
    import torch
    _require_f32_cuda("a", a)
    _require_f32_cuda("b", b)
    sa, sb = a.shape, b.shape
    if len(sa) != 3 or len(sb) != 3 or sa[0] != sb[0] or sa[2] != sb[1]:
        raise ValueError(f"shape mismatch: {tuple(sa)} x {tuple(sb)}")
    batch, m, k = sa
    n = sb[2]
    if out is None:
        out = torch.empty((batch, m, n), dtype=torch.float32, device=a.device)
    else:
        _require_f32_cuda("out", out)
        if tuple(out.shape) != (batch, m, n):
            raise ValueError("out has the wrong shape")
    ta, tb, to = a.stride(), b.stride(), out.stride()
    multi = batch > 1
    args = (batch, m, n, k,
            a.data_ptr(), _row_major_ld(a, m, k, ta[1:]), ta[0] if multi else m * k,
            b.data_ptr(), _row_major_ld(b, k, n, tb[1:]), tb[0] if multi else k * n,
            out.data_ptr(), _row_major_ld(out, m, n, to[1:]), to[0] if multi else m * n)
    return args, out


def sgemm_batched(a, b, out=None, stream=None):
    """out[i] = a[i].b[i] for 3-D float32 device tensors (batch,m,k), (batch,k,n).  -> tg_sgemm_batched"""
    args, out = _batched_args(a, b, out)
    st = load_library().tg_sgemm_batched(*args, _stream_handle(stream))
    if st != TG_OK:
        _check(st)
    return out


def tune(a, b, out=None, reps: int = 5, stream=None):
    """Time the candidate configurations on these operands and cache the winner.  -> tg_tune

    Accepts 2-D or 3-D operands; returns out holding the product.  Blocking.
    """
    squeeze = a.dim() == 2
    if squeeze:
        a, b = a.unsqueeze(0), b.unsqueeze(0)
        out = out.unsqueeze(0) if out is not None else None
    args, out = _batched_args(a, b, out)
    _check(load_library().tg_tune(*args, _stream_handle(stream), int(reps)))
    return out[0] if squeeze else out


def set_workspace(tensor):
    """Give the library a device buffer for split-K partial sums (None removes it).  -> tg_set_workspace"""
    global _workspace
    lib = load_library()
    if tensor is None:
        _check(lib.tg_set_workspace(None, 0))
        _workspace = None
        return
    if not tensor.is_cuda or not tensor.is_contiguous():
        raise ValueError("workspace must be a contiguous device tensor")
    _check(lib.tg_set_workspace(tensor.data_ptr(), tensor.numel() * tensor.element_size()))
    _workspace = tensor


def workspace_bytes(batch: int, m: int, n: int, k: int) -> int:
    return int(load_library().tg_workspace_bytes(batch, m, n, k))


def strided_workspace_bytes(m: int, n: int, k: int, csa: int, csb: int) -> int:
    return int(load_library().tg_strided_workspace_bytes(m, n, k, csa, csb))


def force_config(spec):
    _check(load_library().tg_force_config(spec.encode() if spec else None))


MATH_FP32_MFMA, MATH_BF16_PIECES = 0, 1


def set_math(mode: int):
    """Which arithmetic the automatic choice may use: MATH_FP32_MFMA (default) or MATH_BF16_PIECES."""
    _check(load_library().tg_set_math(mode))


def get_math() -> int:
    return int(load_library().tg_get_math())


def get_config(batch: int, m: int, n: int, k: int) -> str:
    buf = ctypes.create_string_buffer(256)
    _check(load_library().tg_get_config(batch, m, n, k, ctypes.cast(buf, ctypes.c_void_p), 256))
    return buf.value.decode()


def candidates(batch: int, m: int, n: int, k: int):
    """The configurations ``tune`` would consider, in timing order: (spec, lower_bound_us, model_us) each."""
    lib = load_library()
    count = lib.tg_num_candidates(batch, m, n, k)
    if count < 0:
        raise TgemmError(1, lib.tg_last_error().decode())
    buf = ctypes.create_string_buffer(256)
    bound, model = ctypes.c_double(), ctypes.c_double()
    out = []
    for i in range(count):
        _check(lib.tg_candidate(batch, m, n, k, i, ctypes.cast(buf, ctypes.c_void_p), 256,
                                ctypes.cast(ctypes.byref(bound), ctypes.c_void_p),
                                ctypes.cast(ctypes.byref(model), ctypes.c_void_p)))
        out.append((buf.value.decode(), bound.value, model.value))
    return out


def tune_is_launch_bound(batch: int, m: int, n: int, k: int) -> bool:
    """Whether ``tune`` would time this problem's leaders as graph replays (decided by the cost model).  -> tg_tune_is_launch_bound"""
    lib = load_library()
    r = lib.tg_tune_is_launch_bound(batch, m, n, k)
    if r < 0:
        raise TgemmError(1, lib.tg_last_error().decode())
    return bool(r)


def last_config() -> str:
    return load_library().tg_last_config().decode()


def kernel_names():
    lib = load_library()
    out = []
    buf = ctypes.create_string_buffer(128)
    for i in range(lib.tg_num_kernels()):
        _check(lib.tg_kernel_name(i, ctypes.cast(buf, ctypes.c_void_p), 128))
        out.append(buf.value.decode())
    return out


def load_tune_cache(path):
    _check(load_library().tg_load_tune_cache(str(path).encode()))


def save_tune_cache(path):
    _check(load_library().tg_save_tune_cache(str(path).encode()))


def clear_tune_cache():
    load_library().tg_clear_tune_cache()


def version() -> int:
    return int(load_library().tg_version())
