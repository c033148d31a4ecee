"""ctypes binding of liblords.so.  Same names as include/lords.h; argument
marshalling only (tensor -> device pointer, current stream -> void*)."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblords.so")
_lib = None

LORDS_BF16, LORDS_F32 = 0, 1
LORDS_PATH_AUTO, LORDS_PATH_DECODE, LORDS_PATH_PREFILL, LORDS_PATH_GEMV, LORDS_PATH_SMALLM = 0, 1, 2, 3, 4
LORDS_PATH_MFMA = LORDS_PATH_PREFILL
STATUS_NAMES = {0: "LORDS_OK", 1: "LORDS_ERR_NULL", 2: "LORDS_ERR_BITS", 3: "LORDS_ERR_SHAPE",
                4: "LORDS_ERR_ALIGN", 5: "LORDS_ERR_DTYPE", 6: "LORDS_ERR_LAUNCH", 7: "LORDS_ERR_UNSUPPORTED",
                8: "LORDS_ERR_WORKSPACE"}

EXPORTS = ["lords_version", "lords_status_string", "lords_row_bytes", "lords_equivalent_rank", "lords_mixed_schedule",
           "lords_unpack", "lords_dequant", "lords_quantize", "lords_block_init", "lords_matmul", "lords_matmul_ex",
           "lords_workspace_bytes", "lords_workspace_zero_bytes", "lords_matmul_ws", "lords_noalloc_limit", "lords_matmul_noalloc", "lords_probe_stream_read", "lords_probe_mfma_bf16",
           "lords_repack_bytes", "lords_repack", "lords_matmul_repacked",
           "lords_matmul_batched", "lords_gate_up", "lords_transpose_codes", "lords_backward_input", "lords_backward_factors"]


class LordsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({lords_status_string(status)})")


def library_path() -> str:
    return _LIB_PATH


def library():
    """Load liblords.so (built in-tree by paper_2601_22716_amd.build). Fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2601_22716_amd.build` "
                "(there is no fallback implementation)")
        # PyTorch-ROCm ships its own HIP runtime; load it first so that the library, torch's
        # allocator and torch's streams all live in ONE runtime instance.
        import torch  # noqa: F401
        lib = ctypes.CDLL(_LIB_PATH)
        vp, ci, cl = ctypes.c_void_p, ctypes.c_int, ctypes.c_long
        lib.lords_version.restype = ci
        lib.lords_version.argtypes = []
        lib.lords_status_string.restype = ctypes.c_char_p
        lib.lords_status_string.argtypes = [ci]
        lib.lords_row_bytes.restype = ctypes.c_size_t
        lib.lords_row_bytes.argtypes = [ci, ci]
        lib.lords_equivalent_rank.restype = cl
        lib.lords_equivalent_rank.argtypes = [cl, cl, cl]
        lib.lords_mixed_schedule.restype = ci
        lib.lords_mixed_schedule.argtypes = [ci, ctypes.c_double, ci, ci, ctypes.POINTER(ci), ctypes.POINTER(ctypes.c_double)]
        lib.lords_unpack.restype = ci
        lib.lords_unpack.argtypes = [vp, vp, ci, ci, ci, vp]
        lib.lords_dequant.restype = ci
        lib.lords_dequant.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp]
        lib.lords_matmul.restype = ci
        lib.lords_matmul.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
        lib.lords_matmul_ex.restype = ci
        lib.lords_matmul_ex.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp, ci]
        lib.lords_matmul_ws.restype = ci
        lib.lords_matmul_ws.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp, ci, vp, ctypes.c_size_t]
        lib.lords_matmul_noalloc.restype = ci
        lib.lords_matmul_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
        lib.lords_workspace_bytes.restype = ctypes.c_size_t
        lib.lords_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci, ci]
        lib.lords_workspace_zero_bytes.restype = ctypes.c_size_t
        lib.lords_workspace_zero_bytes.argtypes = []
        lib.lords_probe_stream_read.restype = ci
        lib.lords_probe_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        lib.lords_probe_mfma_bf16.restype = ci
        lib.lords_probe_mfma_bf16.argtypes = [ci, ci, vp, ctypes.POINTER(ctypes.c_double), vp]
        lib.lords_noalloc_limit.restype = ctypes.c_size_t
        lib.lords_noalloc_limit.argtypes = []
        lib.lords_repack_bytes.restype = ctypes.c_size_t
        lib.lords_repack_bytes.argtypes = [ci, ci, ci]
        lib.lords_repack.restype = ci
        lib.lords_repack.argtypes = [vp, vp, ci, ci, ci, vp]
        lib.lords_matmul_repacked.restype = ci
        lib.lords_matmul_repacked.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp, ci]
        lib.lords_quantize.restype = ci
        lib.lords_quantize.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp]
        lib.lords_block_init.restype = ci
        lib.lords_block_init.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp]
        lib.lords_matmul_batched.restype = ci
        lib.lords_matmul_batched.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
        lib.lords_gate_up.restype = ci
        lib.lords_gate_up.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
        lib.lords_transpose_codes.restype = ci
        lib.lords_transpose_codes.argtypes = [vp, vp, ci, ci, ci, vp]
        lib.lords_backward_input.restype = ci
        lib.lords_backward_input.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
        lib.lords_backward_factors.restype = ci
        lib.lords_backward_factors.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp]
        _lib = lib
    return _lib


def bf16_from_bits(bits_u16, device="cuda"):
    """numpy uint16 bf16 bit patterns -> torch.bfloat16 tensor on `device` (a reinterpretation, no arithmetic)."""
    import numpy as np
    import torch
    a = np.ascontiguousarray(bits_u16, dtype=np.uint16)
    return torch.from_numpy(a.view(np.int16).copy()).to(device).view(torch.bfloat16)


def _ptr(t):
    """Device pointer of a torch tensor (or a raw int / None passed through)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensors handed to the library must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return LORDS_BF16
    if t.dtype == torch.float32:
        return LORDS_F32
    raise TypeError(f"unsupported dtype {t.dtype}: the library takes bfloat16 or float32")


def _check(status: int, where: str):
    if status != 0:
        raise LordsError(status, where)


def lords_version() -> int:
    return int(library().lords_version())


def lords_status_string(status: int) -> str:
    return library().lords_status_string(int(status)).decode()


def lords_row_bytes(K: int, bits: int) -> int:
    return int(library().lords_row_bytes(K, bits))


def lords_equivalent_rank(N: int, K: int, group: int) -> int:
    return int(library().lords_equivalent_rank(N, K, group))


def lords_mixed_schedule(n_layers: int, fraction_first: float, bits_first: int = 4, bits_rest: int = 2):
    """Returns (list of per-layer code widths, their mean)."""
    out = (ctypes.c_int * max(int(n_layers), 1))()
    avg = ctypes.c_double(0.0)
    _check(library().lords_mixed_schedule(n_layers, fraction_first, bits_first, bits_rest, out, ctypes.byref(avg)),
           "lords_mixed_schedule")
    return [int(v) for v in out[:n_layers]], float(avg.value)


def lords_unpack(codes, idx, N: int, K: int, bits: int, stream=None) -> None:
    _check(library().lords_unpack(_ptr(codes), _ptr(idx), N, K, bits, _stream(stream)), "lords_unpack")


def lords_dequant(codes, codebook, B, A, W, N: int, K: int, r: int, bits: int, stream=None) -> None:
    _check(library().lords_dequant(_ptr(codes), _ptr(codebook), _ptr(B), _ptr(A), _ptr(W), N, K, r, bits,
                                   _dtype_code(B), _dtype_code(W), _stream(stream)), "lords_dequant")


def lords_quantize(W, codebook, B, A, codes, N: int, K: int, r: int, bits: int, stream=None) -> None:
    _check(library().lords_quantize(_ptr(W), _ptr(codebook), _ptr(B), _ptr(A), _ptr(codes), N, K, r, bits,
                                    _dtype_code(W), _dtype_code(B), _stream(stream)), "lords_quantize")


def lords_block_init(W, codebook, B, A, N: int, K: int, r: int, bits: int, stream=None) -> None:
    _check(library().lords_block_init(_ptr(W), _ptr(codebook), _ptr(B), _ptr(A), N, K, r, bits,
                                      _dtype_code(W), _dtype_code(B), _stream(stream)), "lords_block_init")


def lords_matmul(X, codes, codebook, B, A, Y, M: int, N: int, K: int, r: int, bits: int, stream=None) -> None:
    _check(library().lords_matmul(_ptr(X), _ptr(codes), _ptr(codebook), _ptr(B), _ptr(A), _ptr(Y), M, N, K, r, bits,
                                  _dtype_code(B), _dtype_code(Y), _stream(stream)), "lords_matmul")


def lords_matmul_ex(X, codes, codebook, B, A, Y, M: int, N: int, K: int, r: int, bits: int,
                    path: int = LORDS_PATH_AUTO, stream=None) -> None:
    _check(library().lords_matmul_ex(_ptr(X), _ptr(codes), _ptr(codebook), _ptr(B), _ptr(A), _ptr(Y), M, N, K, r, bits,
                                     _dtype_code(B), _dtype_code(Y), _stream(stream), path), "lords_matmul_ex")


def lords_workspace_bytes(M: int, N: int, K: int, r: int, bits: int, factor_dtype: int = LORDS_BF16,
                          path: int = LORDS_PATH_AUTO) -> int:
    return int(library().lords_workspace_bytes(M, N, K, r, bits, factor_dtype, path))


def lords_workspace_zero_bytes() -> int:
    return int(library().lords_workspace_zero_bytes())


def lords_noalloc_limit() -> int:
    return int(library().lords_noalloc_limit())


def lords_matmul_ws(X, codes, codebook, B, A, Y, M: int, N: int, K: int, r: int, bits: int, workspace,
                    path: int = LORDS_PATH_AUTO, stream=None) -> None:
    """`workspace`: a device byte tensor, at least lords_workspace_bytes(...) long, its first
    lords_workspace_zero_bytes() bytes zero when first handed over."""
    _check(library().lords_matmul_ws(_ptr(X), _ptr(codes), _ptr(codebook), _ptr(B), _ptr(A), _ptr(Y), M, N, K, r, bits,
                                     _dtype_code(B), _dtype_code(Y), _stream(stream), path, _ptr(workspace),
                                     workspace.numel() * workspace.element_size()), "lords_matmul_ws")


def lords_matmul_noalloc(X, codes, codebook, B, A, Y, M: int, N: int, K: int, r: int, bits: int, stream=None) -> None:
    _check(library().lords_matmul_noalloc(_ptr(X), _ptr(codes), _ptr(codebook), _ptr(B), _ptr(A), _ptr(Y), M, N, K, r, bits,
                                          _dtype_code(B), _dtype_code(Y), _stream(stream)), "lords_matmul_noalloc")


def lords_repack_bytes(N: int, K: int, bits: int) -> int:
    return int(library().lords_repack_bytes(N, K, bits))


def lords_repack(codes, codes_tiled, N: int, K: int, bits: int, stream=None) -> None:
    _check(library().lords_repack(_ptr(codes), _ptr(codes_tiled), N, K, bits, _stream(stream)), "lords_repack")


def lords_matmul_repacked(X, codes_tiled, codebook, B, A, Y, M: int, N: int, K: int, r: int, bits: int,
                          path: int = LORDS_PATH_AUTO, stream=None) -> None:
    _check(library().lords_matmul_repacked(_ptr(X), _ptr(codes_tiled), _ptr(codebook), _ptr(B), _ptr(A), _ptr(Y), M, N, K, r, bits,
                                           _dtype_code(B), _dtype_code(Y), _stream(stream), path), "lords_matmul_repacked")


def lords_probe_stream_read(buffer, sink, stream=None) -> None:
    _check(library().lords_probe_stream_read(_ptr(buffer), buffer.numel() * buffer.element_size(), _ptr(sink), _stream(stream)),
           "lords_probe_stream_read")


def lords_probe_mfma_bf16(iterations: int, sink, pattern: int = 1, stream=None) -> float:
    """Returns the floating-point operations of the launch."""
    flop = ctypes.c_double(0.0)
    _check(library().lords_probe_mfma_bf16(iterations, pattern, _ptr(sink), ctypes.byref(flop), _stream(stream)),
           "lords_probe_mfma_bf16")
    return flop.value


def _ptr_array(tensors):
    """Host array of device pointers (void *[L]) from a sequence of tensors / raw ints / None."""
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = _ptr(t)
    return arr


def lords_matmul_batched(X, codes, codebook, B, A, Y, N, M: int, K: int, r: int, bits: int, stream=None) -> None:
    """codes, B, A, Y: sequences of L tensors; N: sequence of L row counts."""
    L = len(N)
    if not (len(codes) == len(B) == len(A) == len(Y) == L):
        raise ValueError("codes, B, A, Y and N must have the same length")
    n_arr = (ctypes.c_int * L)(*[int(n) for n in N])
    _check(library().lords_matmul_batched(_ptr(X), _ptr_array(codes), _ptr(codebook), _ptr_array(B), _ptr_array(A),
                                          _ptr_array(Y), n_arr, L, M, K, r, bits, _dtype_code(B[0]), _dtype_code(Y[0]),
                                          _stream(stream)), "lords_matmul_batched")


def lords_gate_up(X, codes_gate, B_gate, A_gate, codes_up, B_up, A_up, codebook, H, M: int, N: int, K: int, r: int,
                  bits: int, stream=None) -> None:
    _check(library().lords_gate_up(_ptr(X), _ptr(codes_gate), _ptr(B_gate), _ptr(A_gate), _ptr(codes_up), _ptr(B_up),
                                   _ptr(A_up), _ptr(codebook), _ptr(H), M, N, K, r, bits, _dtype_code(B_gate),
                                   _dtype_code(H), _stream(stream)), "lords_gate_up")


def lords_transpose_codes(codes, codes_t, N: int, K: int, bits: int, stream=None) -> None:
    _check(library().lords_transpose_codes(_ptr(codes), _ptr(codes_t), N, K, bits, _stream(stream)), "lords_transpose_codes")


def lords_backward_input(dY, codes_t, codebook, B, A, dX, M: int, N: int, K: int, r: int, bits: int, stream=None) -> None:
    _check(library().lords_backward_input(_ptr(dY), _ptr(codes_t), _ptr(codebook), _ptr(B), _ptr(A), _ptr(dX), M, N, K, r,
                                          bits, _dtype_code(B), _dtype_code(dX), _stream(stream)), "lords_backward_input")


def lords_backward_factors(dY, X, codes, codebook, B, A, dB, dA, M: int, N: int, K: int, r: int, bits: int,
                           stream=None) -> None:
    _check(library().lords_backward_factors(_ptr(dY), _ptr(X), _ptr(codes), _ptr(codebook), _ptr(B), _ptr(A), _ptr(dB),
                                            _ptr(dA), M, N, K, r, bits, _dtype_code(B), _stream(stream)),
           "lords_backward_factors")
