"""ctypes binding for libswz: same names as the C entry points, argument marshalling only.

torch is used for device memory (``tensor.data_ptr()``) and streams only.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libswz.so")

MODE_RR, MODE_XCD, MODE_XCD_GROUPM, MODE_GROUPM = 0, 1, 2, 3
MODE_SKEW = 4                          # flag: add to any of the four for the skewed raster (modes 4..7)
MODES = {"rr": MODE_RR, "xcd": MODE_XCD, "xcd_groupm": MODE_XCD_GROUPM, "groupm": MODE_GROUPM}
MODES.update({name + "_skew": m + MODE_SKEW for name, m in list(MODES.items())})
DTYPE_BF16 = 0

EXPORTS = ("swz_status_string", "swz_device_info", "swz_pid_map", "swz_pid_map_device", "swz_gemm", "swz_gemm_ex",
           "swz_gemm_plan", "swz_copy_bytes", "swz_pid_map_persistent", "swz_pid_map_persistent_device", "swz_transpose",
           "swz_softmax", "swz_layernorm", "swz_mfma_peak", "swz_gemm_probe")


class SwzParams(ctypes.Structure):
    _fields_ = [("bm", ctypes.c_int32), ("bn", ctypes.c_int32), ("bk", ctypes.c_int32),
                ("group_m", ctypes.c_int32), ("num_xcd", ctypes.c_int32), ("persistent", ctypes.c_int32),
                ("num_wg", ctypes.c_int32)]


class SwzError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def _ensure_hip_runtime() -> None:
    """libswz.so leaves its hip* symbols to the process: make one HIP runtime globally visible.

    torch's streams and allocations belong to the runtime torch ships, so that is the one the
    library must bind to; re-opening it with RTLD_GLOBAL exposes its symbols to libswz.so.
    """
    try:
        import torch
        path = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
        if not os.path.exists(path):
            path = "libamdhip64.so"
    except ImportError:  # no torch: a plain ROCm install
        path = "libamdhip64.so"
    ctypes.CDLL(path, mode=ctypes.RTLD_GLOBAL)


def _load() -> ctypes.CDLL:
    _ensure_hip_runtime()
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python paper_2508_20258_amd/build.py` "
            "(hipcc, gfx950). There is no fallback path.")
    L = ctypes.CDLL(LIB_PATH)
    i, i64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
    ip = ctypes.POINTER(ctypes.c_int)
    pp = ctypes.POINTER(SwzParams)
    L.swz_status_string.argtypes = [i]
    L.swz_status_string.restype = ctypes.c_char_p
    L.swz_device_info.argtypes = [ip, ip, ip, ip]
    L.swz_pid_map.argtypes = [i, i, i, i, i, vp]
    L.swz_pid_map_device.argtypes = [i, i, i, i, i, vp, vp, vp]
    L.swz_gemm.argtypes = [vp, vp, vp, i64, i64, i64, i, i, vp]
    L.swz_gemm_ex.argtypes = [vp, vp, vp, i64, i64, i64, i, i, pp, vp]
    L.swz_gemm_plan.argtypes = [i64, i64, i64, pp, pp, ip, ip]
    L.swz_gemm_probe.argtypes = [vp, vp, vp, i64, i64, i64, i, i, pp, vp, i64, vp]
    L.swz_copy_bytes.argtypes = [vp, vp, i64, vp]
    L.swz_transpose.argtypes = [vp, vp, i64, i64, i, i, i, pp, vp]
    L.swz_softmax.argtypes = [vp, vp, i64, i64, i, i, pp, vp]
    L.swz_layernorm.argtypes = [vp, vp, vp, vp, i64, i64, ctypes.c_float, i, i, pp, vp]
    L.swz_mfma_peak.argtypes = [vp, i64, i, i, ip, vp]
    L.swz_pid_map_persistent.argtypes = [i, i, i, i, i, i, vp]
    L.swz_pid_map_persistent_device.argtypes = [i, i, i, i, i, i, vp, vp, vp]
    for name in EXPORTS:
        if name != "swz_status_string":
            getattr(L, name).restype = i
    return L


lib = _load()


def status_string(status: int) -> str:
    return lib.swz_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise SwzError(status, where)


def _stream_handle(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _same_current_device(stream, *tensors) -> None:
    """The library launches on the calling thread's current device: every tensor must live there (and the stream too)."""
    import torch
    cur = torch.cuda.current_device()
    for t in tensors:
        if t.device.index != cur:
            raise ValueError(f"tensor on cuda:{t.device.index} but the current device is cuda:{cur}")
    if stream is not None and getattr(stream, "device", None) is not None and stream.device.index != cur:
        raise ValueError(f"stream of cuda:{stream.device.index} but the current device is cuda:{cur}")


def _params(bm=0, bn=0, bk=0, group_m=0, num_xcd=0, persistent=0, num_wg=0) -> SwzParams:
    return SwzParams(int(bm), int(bn), int(bk), int(group_m), int(num_xcd), int(persistent), int(num_wg))


def device_info() -> dict:
    v = [ctypes.c_int(0) for _ in range(4)]
    _check(lib.swz_device_info(*[ctypes.byref(x) for x in v]), "swz_device_info")
    return dict(num_xcd=v[0].value, compute_units=v[1].value, l2_bytes=v[2].value, lds_bytes=v[3].value)


def pid_map(grid_m: int, grid_n: int, num_xcd: int, group_m: int, mode: int) -> np.ndarray:
    """Host PID map: out[w] = pm*grid_n + pn (int32 numpy array)."""
    n = int(grid_m) * int(grid_n)
    out = np.full(max(n, 1) if 0 < n < (1 << 31) else 1, -1, dtype=np.int32)
    _check(lib.swz_pid_map(int(grid_m), int(grid_n), int(num_xcd), int(group_m), int(mode), out.ctypes.data),
           "swz_pid_map")
    return out


def pid_map_device(grid_m: int, grid_n: int, num_xcd: int, group_m: int, mode: int, stream=None):
    """Device PID map: (tile, xcc) int32 CUDA tensors filled by the kernel's own decode."""
    import torch
    n = int(grid_m) * int(grid_n)
    if not 0 < n < (1 << 31):
        n = 1  # let the library report the error; keep the buffers valid
    tile = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    xcc = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    _check(lib.swz_pid_map_device(int(grid_m), int(grid_n), int(num_xcd), int(group_m), int(mode), tile.data_ptr(),
                                  xcc.data_ptr(), _stream_handle(stream)), "swz_pid_map_device")
    return tile, xcc


def gemm_plan(M: int, N: int, K: int, **params) -> dict:
    r = SwzParams()
    gm, gn = ctypes.c_int(0), ctypes.c_int(0)
    p = _params(**params)
    _check(lib.swz_gemm_plan(int(M), int(N), int(K), ctypes.byref(p), ctypes.byref(r), ctypes.byref(gm),
                             ctypes.byref(gn)), "swz_gemm_plan")
    return dict(bm=r.bm, bn=r.bn, bk=r.bk, group_m=r.group_m, num_xcd=r.num_xcd, persistent=r.persistent,
                num_wg=r.num_wg, grid_m=gm.value, grid_n=gn.value)


def gemm(a, b, c=None, mode: int = MODE_XCD_GROUPM, stream=None, **params):
    """C = A @ B on the GPU through swz_gemm / swz_gemm_ex.

    a (M x K), b (K x N): contiguous torch.bfloat16 CUDA tensors; c (M x N) is allocated if not given.
    Keyword params (bm, bn, bk, group_m, num_xcd, persistent, num_wg) select swz_gemm_ex.
    """
    import torch
    assert a.is_cuda and b.is_cuda and a.dtype == torch.bfloat16 and b.dtype == torch.bfloat16
    assert a.is_contiguous() and b.is_contiguous() and a.dim() == 2 and b.dim() == 2 and a.shape[1] == b.shape[0]
    M, K = a.shape
    N = b.shape[1]
    if c is None:
        c = torch.empty((M, N), dtype=torch.bfloat16, device=a.device)
    assert c.is_cuda and c.dtype == torch.bfloat16 and c.is_contiguous() and tuple(c.shape) == (M, N)
    _same_current_device(stream, a, b, c)
    h = _stream_handle(stream)
    if params:
        p = _params(**params)
        st = lib.swz_gemm_ex(a.data_ptr(), b.data_ptr(), c.data_ptr(), M, N, K, DTYPE_BF16, int(mode), ctypes.byref(p), h)
        _check(st, "swz_gemm_ex")
    else:
        _check(lib.swz_gemm(a.data_ptr(), b.data_ptr(), c.data_ptr(), M, N, K, DTYPE_BF16, int(mode), h), "swz_gemm")
    return c


PROBE_WORDS = 16


def gemm_probe(a, b, c=None, mode: int = MODE_XCD_GROUPM, stream=None, probe=None, **params):
    """swz_gemm_probe: C = A @ B by the time-stamping instantiation of the kernel.

    Returns (c, probe): probe is an int64 CUDA tensor of shape (workgroups, 16), row w written by hardware
    workgroup w (layout in include/swz.h)."""
    import torch
    assert a.is_cuda and b.is_cuda and a.dtype == torch.bfloat16 and b.dtype == torch.bfloat16
    assert a.is_contiguous() and b.is_contiguous() and a.dim() == 2 and b.dim() == 2 and a.shape[1] == b.shape[0]
    M, K = a.shape
    N = b.shape[1]
    if c is None:
        c = torch.empty((M, N), dtype=torch.bfloat16, device=a.device)
    assert c.is_cuda and c.dtype == torch.bfloat16 and c.is_contiguous() and tuple(c.shape) == (M, N)
    _same_current_device(stream, a, b, c)
    plan = gemm_plan(M, N, K, **params)
    if probe is None:
        probe = torch.full((plan["grid_m"] * plan["grid_n"], PROBE_WORDS), -1, dtype=torch.int64, device=a.device)
    assert probe.is_cuda and probe.is_contiguous() and probe.dtype == torch.int64
    p = _params(**params)
    _check(lib.swz_gemm_probe(a.data_ptr(), b.data_ptr(), c.data_ptr(), M, N, K, DTYPE_BF16, int(mode), ctypes.byref(p),
                              probe.data_ptr(), probe.numel(), _stream_handle(stream)), "swz_gemm_probe")
    return c, probe


def copy_bytes(src, dst, stream=None) -> None:
    """Plain device copy of src into dst (same byte size), the calibration kernel of known traffic."""
    nbytes = src.numel() * src.element_size()
    assert src.is_cuda and dst.is_cuda and dst.numel() * dst.element_size() == nbytes
    _same_current_device(stream, src, dst)
    _check(lib.swz_copy_bytes(src.data_ptr(), dst.data_ptr(), nbytes, _stream_handle(stream)), "swz_copy_bytes")


def _rounds(grid_m: int, grid_n: int, num_wg: int) -> int:
    n = int(grid_m) * int(grid_n)
    return -(-n // int(num_wg)) if 0 < n < (1 << 31) and num_wg > 0 else 1


def pid_map_persistent(grid_m: int, grid_n: int, num_xcd: int, group_m: int, mode: int, num_wg: int) -> np.ndarray:
    """Host PID map of the persistent launch: out[round, w] = tile or -1 (int32, shape rounds x num_wg)."""
    rounds = _rounds(grid_m, grid_n, num_wg)
    out = np.full((rounds, max(int(num_wg), 1)), -2, dtype=np.int32)
    _check(lib.swz_pid_map_persistent(int(grid_m), int(grid_n), int(num_xcd), int(group_m), int(mode), int(num_wg),
                                      out.ctypes.data), "swz_pid_map_persistent")
    return out


def pid_map_persistent_device(grid_m: int, grid_n: int, num_xcd: int, group_m: int, mode: int, num_wg: int, stream=None):
    """Device PID map of the persistent launch: (tile [rounds x num_wg], xcc [num_wg]) int32 CUDA tensors."""
    import torch
    rounds = _rounds(grid_m, grid_n, num_wg)
    tile = torch.full((rounds, max(int(num_wg), 1)), -2, dtype=torch.int32, device="cuda")
    xcc = torch.full((max(int(num_wg), 1),), -1, dtype=torch.int32, device="cuda")
    _check(lib.swz_pid_map_persistent_device(int(grid_m), int(grid_n), int(num_xcd), int(group_m), int(mode), int(num_wg),
                                             tile.data_ptr(), xcc.data_ptr(), _stream_handle(stream)),
           "swz_pid_map_persistent_device")
    return tile, xcc


def transpose(x, out=None, tile: int = 64, mode: int = MODE_XCD_GROUPM + MODE_SKEW, stream=None, **params):
    """out (N x M) = x (M x N) transposed on the GPU through swz_transpose; tensors of 2-byte or 4-byte elements.
    The defaults (64-wide tiles, XCD renumbering + grouped raster + skew) are the fastest combination measured."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.dim() == 2 and x.element_size() in (2, 4)
    M, N = x.shape
    if out is None:
        out = torch.empty((N, M), dtype=x.dtype, device=x.device)
    assert out.is_cuda and out.is_contiguous() and tuple(out.shape) == (N, M) and out.dtype == x.dtype
    _same_current_device(stream, x, out)
    p = _params(**params)
    _check(lib.swz_transpose(x.data_ptr(), out.data_ptr(), M, N, x.element_size(), int(tile), int(mode), ctypes.byref(p),
                             _stream_handle(stream)), "swz_transpose")
    return out


def _row_args(x, out):
    import torch
    assert x.is_cuda and x.is_contiguous() and x.dim() == 2 and x.dtype == torch.bfloat16
    if out is None:
        out = torch.empty_like(x)
    assert out.is_cuda and out.is_contiguous() and out.shape == x.shape and out.dtype == x.dtype
    return out


def softmax(x, out=None, chunks: int = 1, mode: int = MODE_XCD, stream=None, **params):
    """Row softmax of a bf16 matrix on the GPU through swz_softmax; `chunks` workgroups per row."""
    out = _row_args(x, out)
    _same_current_device(stream, x, out)
    p = _params(**params)
    _check(lib.swz_softmax(x.data_ptr(), out.data_ptr(), x.shape[0], x.shape[1], int(chunks), int(mode), ctypes.byref(p),
                           _stream_handle(stream)), "swz_softmax")
    return out


def layernorm(x, gamma, beta, out=None, eps: float = 1e-5, chunks: int = 1, mode: int = MODE_XCD, stream=None, **params):
    """Layer normalisation of every row of a bf16 matrix on the GPU through swz_layernorm."""
    out = _row_args(x, out)
    for t in (gamma, beta):
        assert t.is_cuda and t.is_contiguous() and t.dtype == x.dtype and t.numel() == x.shape[1]
    _same_current_device(stream, x, out, gamma, beta)
    p = _params(**params)
    _check(lib.swz_layernorm(x.data_ptr(), gamma.data_ptr(), beta.data_ptr(), out.data_ptr(), x.shape[0], x.shape[1],
                             float(eps), int(chunks), int(mode), ctypes.byref(p), _stream_handle(stream)), "swz_layernorm")
    return out


def mfma_peak(out, iters: int, random_operands: bool = True, stream=None) -> int:
    """Launch the MFMA-rate measurement kernel (swz_mfma_peak); returns the flop count of the launch."""
    import torch
    assert out.is_cuda and out.is_contiguous() and out.dtype == torch.float32
    _same_current_device(stream, out)
    wgs = ctypes.c_int(0)
    _check(lib.swz_mfma_peak(out.data_ptr(), out.numel(), int(iters), int(bool(random_operands)), ctypes.byref(wgs),
                             _stream_handle(stream)), "swz_mfma_peak")
    return wgs.value * 8 * int(iters) * 64 * 16384
