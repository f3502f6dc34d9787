"""Thin ctypes binding of ``libattnw.so`` -- argument marshalling only.

Every step of the path (contraction, scaling, row max, exponentials, row sum,
normalisation, stores) runs inside the HIP kernels behind the C ABI declared
in ``include/attnw.h``.  The functions here have the same names as the C entry
points, accept either raw device addresses (ints) or objects with a
``data_ptr()`` method (PyTorch tensors), and raise :class:`AttnwError` on a
non-zero status.  There is no CPU fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

ATTNW_F32 = 0
ATTNW_BF16 = 1

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
_CSRC = os.path.join(_PKG, "csrc")
_LIB = os.path.join(_PKG, "libattnw.so")

EXPORTS = ("attnw_fused", "attnw_softmax", "attnw_softmax_cast", "attnw_gemm_scores", "attnw_scale", "attnw_attention",
           "attnw_status_string", "attnw_version")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]

_lib = None


class AttnwError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libattnw status {status}: {message}")
        self.status = status


def library_path() -> str:
    return _LIB


def sources() -> list:
    return sorted(os.path.join(_CSRC, f) for f in os.listdir(_CSRC) if f.endswith(".hip"))


def build(verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 into ``libattnw.so`` (always recompiles): one hipcc process per
    source, side by side, objects in a temporary directory, then one link step."""
    import concurrent.futures
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    include = ["-I", os.path.join(_ROOT, "include"), "-I", _CSRC]

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        proc = subprocess.run(cmd, capture_output=True, text=True)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + proc.stdout + proc.stderr)

    with tempfile.TemporaryDirectory(prefix="attnw_build_") as tmp:
        jobs = [(src, os.path.join(tmp, os.path.basename(src) + ".o")) for src in sources()]
        workers = max(1, min(len(jobs), os.cpu_count() or 1, 8))
        with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(lambda j: run([hipcc, *compile_flags, *include, "-c", j[0], "-o", j[1]]), jobs))
        run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[o for _, o in jobs], "-o", _LIB])
    global _lib
    _lib = None
    return _LIB


def load_library():
    """Load ``libattnw.so``; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            raise FileNotFoundError(
                f"{_LIB} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        lib = ctypes.CDLL(_LIB)
        i64, vp, ci, cf = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        lib.attnw_fused.argtypes = [vp, vp, vp, i64, i64, i64, i64, cf, ci, vp]
        lib.attnw_fused.restype = ci
        lib.attnw_gemm_scores.argtypes = [vp, vp, vp, i64, i64, i64, i64, cf, ci, vp]
        lib.attnw_gemm_scores.restype = ci
        lib.attnw_attention.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, cf, ci, vp]
        lib.attnw_attention.restype = ci
        lib.attnw_softmax.argtypes = [vp, vp, i64, i64, ci, vp]
        lib.attnw_softmax.restype = ci
        lib.attnw_softmax_cast.argtypes = [vp, vp, i64, i64, ci, ci, vp]
        lib.attnw_softmax_cast.restype = ci
        lib.attnw_scale.argtypes = [vp, vp, i64, ctypes.c_float, ci, vp]
        lib.attnw_scale.restype = ci
        lib.attnw_status_string.argtypes = [ci]
        lib.attnw_status_string.restype = ctypes.c_char_p
        lib.attnw_version.argtypes = []
        lib.attnw_version.restype = ci
        _lib = lib
    return _lib


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if hasattr(stream, "cuda_stream"):      # torch.cuda.Stream exposes the hipStream_t here
        return int(stream.cuda_stream)
    return int(stream)


def _check(status: int) -> None:
    if status != 0:
        raise AttnwError(status, attnw_status_string(status))


def attnw_status_string(status: int) -> str:
    return load_library().attnw_status_string(int(status)).decode()


def attnw_version() -> int:
    return int(load_library().attnw_version())


def attnw_fused(Q, K, P, B: int, H: int, N: int, d: int, scale: float, dtype: int, stream=None) -> None:
    """P = softmax(scale * Q K^T) over keys; see ``attnw_fused`` in include/attnw.h."""
    _check(load_library().attnw_fused(_ptr(Q), _ptr(K), _ptr(P), B, H, N, d, float(scale), int(dtype),
                                      _stream(stream)))


def attnw_softmax(S, P, rows: int, cols: int, dtype: int, stream=None) -> None:
    """Row softmax of S into P; see ``attnw_softmax`` in include/attnw.h."""
    _check(load_library().attnw_softmax(_ptr(S), _ptr(P), rows, cols, int(dtype), _stream(stream)))


def attnw_softmax_cast(S, P, rows: int, cols: int, in_dtype: int, out_dtype: int, stream=None) -> None:
    """Row softmax with separate input and output types; see ``attnw_softmax_cast`` in include/attnw.h."""
    _check(load_library().attnw_softmax_cast(_ptr(S), _ptr(P), rows, cols, int(in_dtype), int(out_dtype),
                                             _stream(stream)))


def attnw_scale(X, Y, count: int, scale: float, dtype: int, stream=None) -> None:
    """Y = scale * X elementwise; see ``attnw_scale`` in include/attnw.h."""
    _check(load_library().attnw_scale(_ptr(X), _ptr(Y), count, float(scale), int(dtype), _stream(stream)))


def attnw_gemm_scores(Q, K, S, B: int, H: int, N: int, d: int, scale: float, dtype: int, stream=None) -> None:
    """S = scale * Q K^T written to device memory; see ``attnw_gemm_scores`` in include/attnw.h."""
    _check(load_library().attnw_gemm_scores(_ptr(Q), _ptr(K), _ptr(S), B, H, N, d, float(scale), int(dtype),
                                            _stream(stream)))


def attnw_attention(Q, K, V, O, B: int, H: int, N: int, d: int, scale: float, dtype: int, stream=None) -> None:
    """O = softmax(scale * Q K^T) V, weights kept on chip; see ``attnw_attention`` in include/attnw.h."""
    _check(load_library().attnw_attention(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), B, H, N, d, float(scale), int(dtype),
                                          _stream(stream)))
