"""ctypes front end of the CPU oracle (``scalecom_oracle.cpp``).

TEST INFRASTRUCTURE ONLY.  The oracle states, in plain single-threaded code, what one
iteration of the paper's Algorithm 1 (lines 6, 7, 10; Eq. 2, 3, 5) computes.  Only the
tests, the smoke check and the ``cpu_baseline`` leg of the benchmark may import this
package; the GPU library and its Python binding never do.

All functions take and return NumPy arrays in host memory.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "scalecom_oracle.cpp")
_LIB = os.path.join(_HERE, "libscalecom_oracle.so")

GRAD_F32 = 0
GRAD_BF16 = 1


def build(force: bool = True) -> str:
    """Compile the oracle with the host compiler (no fused contractions beyond the
    explicit fmaf calls, default IEEE environment)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        i64, i32, f32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_void_p
        lib.oracle_accumulate.argtypes = [vp, vp, i32, i64, f32, vp]
        lib.oracle_topk_sort.argtypes = [vp, i64, i64, vp]
        lib.oracle_topk_select.argtypes = [vp, i64, i64, vp]
        lib.oracle_chunk_select.argtypes = [vp, i64, i64, vp]
        lib.oracle_step_chunked.argtypes = [vp, vp, i32, i32, i64, i64, f32, f32, i64, vp, vp]
        lib.oracle_apply_update.argtypes = [vp, i64, vp, vp, i64, f32]
        lib.oracle_apply_update.restype = ctypes.c_int
        lib.oracle_layer_rate.argtypes = [ctypes.c_double]
        lib.oracle_layer_rate.restype = ctypes.c_int64
        lib.oracle_hamming_distance.argtypes = [vp, vp, i32, i32, i64, i64, f32, i64]
        lib.oracle_hamming_distance.restype = ctypes.c_int64
        lib.oracle_cosine_distance.argtypes = [vp, vp, i64]
        lib.oracle_cosine_distance.restype = ctypes.c_double
        lib.oracle_gather.argtypes = [vp, vp, i64, vp]
        lib.oracle_reduce.argtypes = [vp, i32, i64, vp]
        lib.oracle_memory_update.argtypes = [vp, vp, vp, i64, i64, f32]
        lib.oracle_step.argtypes = [vp, vp, i32, i32, i64, i64, f32, f32, i64, vp, vp]
        lib.oracle_step_layers.argtypes = [vp, vp, i32, i32, i32, vp, vp, f32, f32, i64, vp, vp]
        lib.oracle_step_layers_chunked.argtypes = [vp, vp, i32, i32, i32, vp, vp, f32, f32, i64, vp, vp]
        for name in ("oracle_accumulate", "oracle_topk_sort", "oracle_topk_select", "oracle_gather",
                     "oracle_chunk_select", "oracle_step_chunked", "oracle_step_layers_chunked",
                     "oracle_reduce", "oracle_memory_update", "oracle_step", "oracle_step_layers"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a: np.ndarray) -> int:
    return a.ctypes.data


def _check_f32(a, name):
    if not (isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags.c_contiguous and a.ndim == 1):
        raise TypeError(f"{name}: need a contiguous 1-d float32 array")


def _grad_dtype(g: np.ndarray) -> int:
    """float32 gradients are passed as they are; bfloat16 gradients are passed as their
    16-bit patterns in a uint16 array."""
    if g.dtype == np.float32:
        return GRAD_F32
    if g.dtype == np.uint16:
        return GRAD_BF16
    raise TypeError("gradient must be float32, or uint16 holding bfloat16 patterns")


def _ptr_array(arrays):
    return (ctypes.c_void_p * len(arrays))(*[_p(a) for a in arrays])


def accumulate(mem: np.ndarray, grad: np.ndarray, lr: float) -> np.ndarray:
    _check_f32(mem, "mem")
    acc = np.empty_like(mem)
    rc = _load().oracle_accumulate(_p(mem), _p(grad), _grad_dtype(grad), mem.size, lr, _p(acc))
    if rc:
        raise ValueError("oracle_accumulate: bad arguments")
    return acc


def topk_sort(x: np.ndarray, k: int) -> np.ndarray:
    _check_f32(x, "x")
    idx = np.empty(k, dtype=np.int32)
    if _load().oracle_topk_sort(_p(x), x.size, k, _p(idx)):
        raise ValueError("oracle_topk_sort: bad arguments")
    return idx


def topk_select(x: np.ndarray, k: int) -> np.ndarray:
    _check_f32(x, "x")
    idx = np.empty(k, dtype=np.int32)
    if _load().oracle_topk_select(_p(x), x.size, k, _p(idx)):
        raise ValueError("oracle_topk_select: bad arguments")
    return idx


def chunk_select(x: np.ndarray, chunk: int) -> np.ndarray:
    """One position per chunk of ``chunk`` consecutive elements: its largest magnitude."""
    _check_f32(x, "x")
    if chunk < 1:
        raise ValueError("chunk must be >= 1")
    idx = np.empty(-(-x.size // chunk), dtype=np.int32)
    if _load().oracle_chunk_select(_p(x), x.size, chunk, _p(idx)):
        raise ValueError("oracle_chunk_select: bad arguments")
    return idx


def step_chunked(mem, grad, chunk: int, beta: float, lr: float, step: int):
    """One iteration with the chunk-wise selector.  Returns (idx, reduced); ``mem`` updated in place."""
    n = len(mem)
    for m in mem:
        _check_f32(m, "mem[i]")
    numel = mem[0].size
    if chunk < 1:
        raise ValueError("chunk must be >= 1")
    k = -(-numel // chunk)
    idx = np.empty(k, dtype=np.int32)
    red = np.empty(k, dtype=np.float32)
    rc = _load().oracle_step_chunked(_ptr_array(mem), _ptr_array(grad), _grad_dtype(grad[0]), n, numel, chunk, beta,
                                     lr, step, _p(idx), _p(red))
    if rc:
        raise ValueError("oracle_step_chunked: bad arguments")
    return idx, red


def apply_update(theta: np.ndarray, idx: np.ndarray, reduced: np.ndarray, scale: float) -> None:
    """theta[idx] -= scale * reduced, in place (Alg. 1 lines 10 and 12 on the index set)."""
    _check_f32(theta, "theta")
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    reduced = np.ascontiguousarray(reduced, dtype=np.float32)
    if _load().oracle_apply_update(_p(theta), theta.size, _p(idx), _p(reduced), idx.size, scale):
        raise ValueError("oracle_apply_update: index out of range")


def layer_rate(flops_per_gradient: float) -> int:
    """Compression rate of a layer from its FLOPs/gradient ratio (Sec. 4)."""
    return int(_load().oracle_layer_rate(float(flops_per_gradient)))


def hamming_distance(mem, grad, k: int, lr: float, step: int) -> int:
    """d of Eq. 6 between the leader's top-k and the top-k of the summed error-feedback gradients."""
    for m in mem:
        _check_f32(m, "mem[i]")
    d = _load().oracle_hamming_distance(_ptr_array(mem), _ptr_array(grad), _grad_dtype(grad[0]), len(mem),
                                        mem[0].size, k, lr, step)
    if d < 0:
        raise ValueError("oracle_hamming_distance: bad arguments")
    return int(d)


def cosine_distance(a: np.ndarray, b: np.ndarray) -> float:
    _check_f32(a, "a")
    _check_f32(b, "b")
    return float(_load().oracle_cosine_distance(_p(a), _p(b), a.size))


def gather(acc: np.ndarray, idx: np.ndarray) -> np.ndarray:
    _check_f32(acc, "acc")
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    vals = np.empty(idx.size, dtype=np.float32)
    _load().oracle_gather(_p(acc), _p(idx), idx.size, _p(vals))
    return vals


def reduce(vals) -> np.ndarray:
    vals = [np.ascontiguousarray(v, dtype=np.float32) for v in vals]
    k = vals[0].size
    out = np.empty(k, dtype=np.float32)
    if _load().oracle_reduce(_ptr_array(vals), len(vals), k, _p(out)):
        raise ValueError("oracle_reduce: bad arguments")
    return out


def memory_update(mem: np.ndarray, acc: np.ndarray, idx: np.ndarray, beta: float) -> None:
    """In place on ``mem``."""
    _check_f32(mem, "mem")
    _check_f32(acc, "acc")
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if _load().oracle_memory_update(_p(mem), _p(acc), _p(idx), idx.size, mem.size, beta):
        raise ValueError("oracle_memory_update: index out of range")


def step(mem, grad, k: int, beta: float, lr: float, step: int):
    """One iteration on whole vectors.  ``mem``: list of n float32 arrays, updated in place;
    ``grad``: list of n arrays (float32, or uint16 bfloat16 patterns).  Returns (idx, reduced)."""
    n = len(mem)
    for m in mem:
        _check_f32(m, "mem[i]")
    numel = mem[0].size
    gd = _grad_dtype(grad[0])
    idx = np.empty(k, dtype=np.int32)
    red = np.empty(k, dtype=np.float32)
    rc = _load().oracle_step(_ptr_array(mem), _ptr_array(grad), gd, n, numel, k, beta, lr, step, _p(idx),
                             _p(red))
    if rc:
        raise ValueError("oracle_step: bad arguments")
    return idx, red


def step_layers(mem, grad, offsets, ks, beta: float, lr: float, step: int):
    """One iteration with a separate index set per segment [offsets[s], offsets[s+1])."""
    n = len(mem)
    for m in mem:
        _check_f32(m, "mem[i]")
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    ks = np.ascontiguousarray(ks, dtype=np.int64)
    gd = _grad_dtype(grad[0])
    total = int(ks.sum())
    idx = np.empty(total, dtype=np.int32)
    red = np.empty(total, dtype=np.float32)
    rc = _load().oracle_step_layers(_ptr_array(mem), _ptr_array(grad), gd, n, ks.size, _p(offsets), _p(ks),
                                    beta, lr, step, _p(idx), _p(red))
    if rc:
        raise ValueError("oracle_step_layers: bad arguments")
    return idx, red


def step_layers_chunked(mem, grad, offsets, chunks, beta: float, lr: float, step: int):
    """One iteration with the chunk-wise selector and a chunk size per segment."""
    n = len(mem)
    for m in mem:
        _check_f32(m, "mem[i]")
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    chunks = np.ascontiguousarray(chunks, dtype=np.int64)
    if chunks.size and chunks.min() < 1:
        raise ValueError("chunk sizes must be >= 1")
    lens = np.diff(offsets)
    total = int((-(-lens // chunks)).sum())
    idx = np.empty(total, dtype=np.int32)
    red = np.empty(total, dtype=np.float32)
    rc = _load().oracle_step_layers_chunked(_ptr_array(mem), _ptr_array(grad), _grad_dtype(grad[0]), n, chunks.size,
                                            _p(offsets), _p(chunks), beta, lr, step, _p(idx), _p(red))
    if rc:
        raise ValueError("oracle_step_layers_chunked: bad arguments")
    return idx, red
