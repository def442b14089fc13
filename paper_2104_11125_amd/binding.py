"""Thin Python layer over the C-ABI in ``include/scalecom.h``: argument marshalling only.

Every step of the path runs in the HIP kernels of ``csrc/libscalecom.so``.  PyTorch is used
for device memory and the stream.  If the library has not been built this module raises:
there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "libscalecom.so")

SCALECOM_OK, SCALECOM_EINVAL, SCALECOM_ENOMEM, SCALECOM_EHIP, SCALECOM_EUNSUPPORTED = range(5)
SCALECOM_GRAD_F32, SCALECOM_GRAD_BF16 = 0, 1
SCALECOM_MAX_LEARNERS = 64
SCALECOM_N_PHASES = 5
SCALECOM_N_STATS = 5
SCALECOM_STATIC_NUMEL_MAX, SCALECOM_STATIC_LEARNERS_MAX, SCALECOM_STATIC_K_MAX = 4_194_304, 8, 131_072

_lib = None


class ScaleComError(RuntimeError):
    def __init__(self, status: int, detail: str = ""):
        self.status = status
        text = lib().scalecom_strerror(status).decode()
        super().__init__(f"scalecom status {status} ({text})" + (f": {detail}" if detail else ""))


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library (built by ``paper_2104_11125_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2104_11125_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
        L.scalecom_workspace_bytes.argtypes = [i64, i32, i32, i64]
        L.scalecom_workspace_bytes.restype = sz
        L.scalecom_init.argtypes = [ctypes.POINTER(vp), i32, vp, vp, sz, i32, i64, i64, i32, i32]
        L.scalecom_init.restype = i32
        L.scalecom_step.argtypes = [vp, vp, vp, i32, i64, i64, f32, f32, i64, vp, vp]
        L.scalecom_step.restype = i32
        L.scalecom_step_static.argtypes = [i32, vp, vp, vp, i32, i64, i64, f32, f32, i64, i32, vp, vp]
        L.scalecom_step_static.restype = i32
        L.scalecom_step_chunked.argtypes = [vp, vp, vp, i32, i64, i64, f32, f32, i64, vp, vp]
        L.scalecom_step_chunked.restype = i32
        L.scalecom_step_layers.argtypes = [vp, vp, vp, i32, i32, vp, vp, f32, f32, i64, vp, vp]
        L.scalecom_step_layers.restype = i32
        L.scalecom_step_layers_chunked.argtypes = [vp, vp, vp, i32, i32, vp, vp, f32, f32, i64, vp, vp]
        L.scalecom_step_layers_chunked.restype = i32
        L.scalecom_timing_begin.argtypes = [vp, i32, i32, i32]
        L.scalecom_timing_begin.restype = i32
        L.scalecom_timing_read.argtypes = [vp, vp, i32, ctypes.POINTER(i32)]
        L.scalecom_timing_read.restype = i32
        L.scalecom_selection_stats.argtypes = [vp, vp, i32]
        L.scalecom_selection_stats.restype = i32
        L.scalecom_apply_update.argtypes = [vp, vp, i64, vp, vp, i64, f32]
        L.scalecom_apply_update.restype = i32
        L.scalecom_hamming_scratch_bytes.argtypes = [i64, i32]
        L.scalecom_hamming_scratch_bytes.restype = sz
        L.scalecom_hamming_distance.argtypes = [vp, vp, vp, i32, i32, vp, vp, f32, i64, vp, sz, vp]
        L.scalecom_hamming_distance.restype = i32
        L.scalecom_cosine_distance.argtypes = [vp, vp, vp, i64, vp]
        L.scalecom_cosine_distance.restype = i32
        L.scalecom_layer_ks.argtypes = [i32, vp, vp, vp, vp, vp]
        L.scalecom_layer_ks.restype = i32
        L.scalecom_stream_copy.argtypes = [vp, vp, vp, sz]
        L.scalecom_stream_copy.restype = i32
        L.scalecom_strerror.argtypes = [i32]
        L.scalecom_strerror.restype = ctypes.c_char_p
        L.scalecom_last_error.argtypes = [vp]
        L.scalecom_last_error.restype = ctypes.c_char_p
        L.scalecom_destroy.argtypes = [vp]
        L.scalecom_destroy.restype = None
        _lib = L
    return _lib


def scalecom_workspace_bytes(numel_max: int, n_tensors_max: int, n_learners_max: int, k_max: int) -> int:
    return int(lib().scalecom_workspace_bytes(numel_max, n_tensors_max, n_learners_max, k_max))


def _ptrs(tensors: Sequence[torch.Tensor]):
    return (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def scalecom_layer_ks(flops_per_gradient: Sequence[float], sizes: Sequence[int],
                      uncompressed: Optional[Sequence[bool]] = None):
    """``scalecom_layer_ks`` of the C-ABI: (ks, rates) per layer from the paper's rate guidance."""
    n = len(sizes)
    if len(flops_per_gradient) != n or (uncompressed is not None and len(uncompressed) != n):
        raise ValueError("one ratio (and one flag) per layer")
    c_u = (ctypes.c_uint8 * n)(*[1 if v else 0 for v in uncompressed]) if uncompressed is not None else None
    c_r = (ctypes.c_double * n)(*[float(v) for v in flops_per_gradient])
    c_s = (ctypes.c_int64 * n)(*[int(v) for v in sizes])
    c_k = (ctypes.c_int64 * n)()
    c_rate = (ctypes.c_int64 * n)()
    st = lib().scalecom_layer_ks(n, c_r, c_s, c_u, c_k, c_rate)
    if st != SCALECOM_OK:
        raise ScaleComError(st)
    return list(c_k), list(c_rate)


def scalecom_step_static(mem: Sequence[torch.Tensor], grad: Sequence[torch.Tensor], k: int, beta: float, lr: float,
                         step: int, idx_out: torch.Tensor, reduced_vals_out: torch.Tensor,
                         stream: Optional[torch.cuda.Stream] = None) -> None:
    """``scalecom_step_static`` of the C-ABI: no context, no workspace, nothing allocated (so the
    outputs must be passed in).  Marshalling only; sizes beyond the static limits raise."""
    dev = mem[0].device
    numel = mem[0].numel()
    for m, g in zip(mem, grad):
        if m.dtype != torch.float32 or g.dtype not in (torch.float32, torch.bfloat16) or g.dtype != grad[0].dtype:
            raise TypeError("mem must be float32 and grad float32 or bfloat16")
        if not (m.is_contiguous() and g.is_contiguous() and m.device == dev and g.device == dev):
            raise ValueError("buffers must be contiguous tensors on one device")
        if m.numel() != numel or g.numel() != numel:
            raise ValueError("every learner's mem and grad must have the same number of elements")
    if idx_out.dtype != torch.int32 or reduced_vals_out.dtype != torch.float32 or \
            idx_out.numel() < k or reduced_vals_out.numel() < k:
        raise TypeError("idx_out must be int32[k] and reduced_vals_out float32[k]")
    s = stream if stream is not None else torch.cuda.current_stream(dev)
    index = dev.index if dev.index is not None else torch.cuda.current_device()
    st = lib().scalecom_step_static(index, ctypes.c_void_p(s.cuda_stream), _ptrs(mem), _ptrs(grad), len(mem), numel, k,
                                    beta, lr, step,
                                    SCALECOM_GRAD_BF16 if grad[0].dtype == torch.bfloat16 else SCALECOM_GRAD_F32,
                                    ctypes.c_void_p(idx_out.data_ptr()), ctypes.c_void_p(reduced_vals_out.data_ptr()))
    if st != SCALECOM_OK:
        raise ScaleComError(st, lib().scalecom_last_error(None).decode())


class ScaleCom:
    """One context: a device, a stream and a caller-owned workspace (a torch tensor held here)."""

    def __init__(self, numel_max: int, n_learners_max: int, grad_dtype: torch.dtype = torch.float32,
                 n_tensors_max: int = 1, device: Optional[torch.device] = None,
                 stream: Optional[torch.cuda.Stream] = None, k_max: Optional[int] = None):
        L = lib()
        self.device = torch.device(device if device is not None else "cuda:0")
        if grad_dtype not in (torch.float32, torch.bfloat16):
            raise TypeError("grad_dtype must be torch.float32 or torch.bfloat16")
        self.grad_dtype = grad_dtype
        self.numel_max, self.n_tensors_max = numel_max, n_tensors_max
        self._diag_scratch = None
        k_max = numel_max if k_max is None else k_max
        nbytes = scalecom_workspace_bytes(numel_max, n_tensors_max, n_learners_max, k_max)
        if nbytes == 0:
            raise ScaleComError(SCALECOM_EINVAL, "numel_max / n_tensors_max / n_learners_max / k_max out of range")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self._ctx = ctypes.c_void_p()
        index = self.device.index if self.device.index is not None else torch.cuda.current_device()
        st = L.scalecom_init(ctypes.byref(self._ctx), index, ctypes.c_void_p(self.stream.cuda_stream),
                             ctypes.c_void_p(self.workspace.data_ptr()), nbytes, n_learners_max, numel_max,
                             k_max, n_tensors_max,
                             SCALECOM_GRAD_BF16 if grad_dtype == torch.bfloat16 else SCALECOM_GRAD_F32)
        if st != SCALECOM_OK:
            self._ctx = ctypes.c_void_p()
            raise ScaleComError(st)

    def _check(self, st: int):
        if st != SCALECOM_OK:
            raise ScaleComError(st, lib().scalecom_last_error(self._ctx).decode())

    def _check_buffers(self, mem, grad, extent=None):
        """Every learner's buffers have one length (and reach `extent`, the end of the last segment)."""
        if len(mem) != len(grad) or len(mem) == 0:
            raise ValueError("one mem and one grad buffer per learner")
        numel = mem[0].numel()
        for m, g in zip(mem, grad):
            if m.dtype != torch.float32 or g.dtype != self.grad_dtype:
                raise TypeError("mem must be float32 and grad must have the context's grad_dtype")
            if not (m.is_contiguous() and g.is_contiguous() and m.device == self.device and g.device == self.device):
                raise ValueError("buffers must be contiguous tensors on the context's device")
            if m.numel() != numel or g.numel() != numel:
                raise ValueError("every learner's mem and grad must have the same number of elements")
        if extent is not None and int(extent) > numel:
            raise ValueError("the last segment ends beyond the learners' buffers")

    def scalecom_step(self, mem: Sequence[torch.Tensor], grad: Sequence[torch.Tensor], k: int, beta: float,
                      lr: float, step: int, idx_out: Optional[torch.Tensor] = None,
                      reduced_vals_out: Optional[torch.Tensor] = None):
        """``scalecom_step`` of the C-ABI; allocates the two outputs if they are not given."""
        self._check_buffers(mem, grad)
        numel = mem[0].numel()
        if idx_out is None:
            idx_out = torch.empty(max(k, 0), dtype=torch.int32, device=self.device)
        if reduced_vals_out is None:
            reduced_vals_out = torch.empty(max(k, 0), dtype=torch.float32, device=self.device)
        st = lib().scalecom_step(self._ctx, _ptrs(mem), _ptrs(grad), len(mem), numel, k, beta, lr, step,
                                 ctypes.c_void_p(idx_out.data_ptr()), ctypes.c_void_p(reduced_vals_out.data_ptr()))
        self._check(st)
        return idx_out, reduced_vals_out

    def scalecom_step_chunked(self, mem: Sequence[torch.Tensor], grad: Sequence[torch.Tensor], chunk: int,
                              beta: float, lr: float, step: int, idx_out: Optional[torch.Tensor] = None,
                              reduced_vals_out: Optional[torch.Tensor] = None):
        """``scalecom_step_chunked`` of the C-ABI: one position per chunk of ``chunk`` elements."""
        self._check_buffers(mem, grad)
        numel = mem[0].numel()
        k = -(-numel // chunk) if chunk >= 1 else 0
        if idx_out is None:
            idx_out = torch.empty(k, dtype=torch.int32, device=self.device)
        if reduced_vals_out is None:
            reduced_vals_out = torch.empty(k, dtype=torch.float32, device=self.device)
        st = lib().scalecom_step_chunked(self._ctx, _ptrs(mem), _ptrs(grad), len(mem), numel, chunk, beta, lr, step,
                                         ctypes.c_void_p(idx_out.data_ptr()),
                                         ctypes.c_void_p(reduced_vals_out.data_ptr()))
        self._check(st)
        return idx_out, reduced_vals_out

    def scalecom_step_layers(self, mem: Sequence[torch.Tensor], grad: Sequence[torch.Tensor],
                             offsets: Sequence[int], ks: Sequence[int], beta: float, lr: float, step: int,
                             idx_out: Optional[torch.Tensor] = None,
                             reduced_vals_out: Optional[torch.Tensor] = None):
        """``scalecom_step_layers`` of the C-ABI."""
        self._check_buffers(mem, grad, offsets[-1] if len(offsets) else None)
        n_tensors = len(ks)
        if len(offsets) != n_tensors + 1:
            raise ValueError("offsets must have len(ks) + 1 entries")
        c_off = (ctypes.c_int64 * (n_tensors + 1))(*[int(o) for o in offsets])
        c_ks = (ctypes.c_int64 * n_tensors)(*[int(v) for v in ks])
        total = max(int(sum(int(v) for v in ks)), 0)
        if idx_out is None:
            idx_out = torch.empty(total, dtype=torch.int32, device=self.device)
        if reduced_vals_out is None:
            reduced_vals_out = torch.empty(total, dtype=torch.float32, device=self.device)
        st = lib().scalecom_step_layers(self._ctx, _ptrs(mem), _ptrs(grad), len(mem), n_tensors, c_off, c_ks, beta,
                                        lr, step, ctypes.c_void_p(idx_out.data_ptr()),
                                        ctypes.c_void_p(reduced_vals_out.data_ptr()))
        self._check(st)
        return idx_out, reduced_vals_out

    def scalecom_step_layers_chunked(self, mem: Sequence[torch.Tensor], grad: Sequence[torch.Tensor],
                                     offsets: Sequence[int], chunks: Sequence[int], beta: float, lr: float, step: int,
                                     idx_out: Optional[torch.Tensor] = None,
                                     reduced_vals_out: Optional[torch.Tensor] = None):
        """``scalecom_step_layers_chunked`` of the C-ABI: one position per chunk, a chunk size per tensor."""
        self._check_buffers(mem, grad, offsets[-1] if len(offsets) else None)
        n_tensors = len(chunks)
        if len(offsets) != n_tensors + 1:
            raise ValueError("offsets must have len(chunks) + 1 entries")
        c_off = (ctypes.c_int64 * (n_tensors + 1))(*[int(o) for o in offsets])
        c_ch = (ctypes.c_int64 * n_tensors)(*[int(v) for v in chunks])
        total = sum(-(-(int(b) - int(a)) // int(c)) for a, b, c in zip(offsets[:-1], offsets[1:], chunks)
                    if int(c) >= 1 and int(b) >= int(a))
        if idx_out is None:
            idx_out = torch.empty(total, dtype=torch.int32, device=self.device)
        if reduced_vals_out is None:
            reduced_vals_out = torch.empty(total, dtype=torch.float32, device=self.device)
        st = lib().scalecom_step_layers_chunked(self._ctx, _ptrs(mem), _ptrs(grad), len(mem), n_tensors, c_off, c_ch,
                                                beta, lr, step, ctypes.c_void_p(idx_out.data_ptr()),
                                                ctypes.c_void_p(reduced_vals_out.data_ptr()))
        self._check(st)
        return idx_out, reduced_vals_out

    def scalecom_timing_begin(self, max_steps: int, all_phases: bool = False, every: int = 1) -> None:
        self._check(lib().scalecom_timing_begin(self._ctx, max_steps, 1 if all_phases else 0, every))

    def scalecom_timing_read(self, capacity_steps: int):
        """Per-step lists of SCALECOM_N_PHASES phase durations in milliseconds."""
        buf = (ctypes.c_float * (max(capacity_steps, 1) * SCALECOM_N_PHASES))()
        n = ctypes.c_int(0)
        self._check(lib().scalecom_timing_read(self._ctx, buf, capacity_steps, ctypes.byref(n)))
        return [[buf[t * SCALECOM_N_PHASES + p] for p in range(SCALECOM_N_PHASES)] for t in range(n.value)]

    def scalecom_selection_stats(self, reset: bool = False) -> dict:
        """``scalecom_selection_stats`` of the C-ABI as a dict (waits for the context's stream)."""
        buf = (ctypes.c_uint64 * SCALECOM_N_STATS)()
        self._check(lib().scalecom_selection_stats(self._ctx, buf, 1 if reset else 0))
        names = ("missed", "no_prediction", "full_mode", "wide_range", "steps")
        return {name: int(buf[j]) for j, name in enumerate(names)}

    def scalecom_apply_update(self, theta: torch.Tensor, idx: torch.Tensor, vals: torch.Tensor, scale: float) -> None:
        """``scalecom_apply_update`` of the C-ABI: theta[idx] -= scale * vals, in place."""
        if theta.dtype != torch.float32 or idx.dtype != torch.int32 or vals.dtype != torch.float32:
            raise TypeError("theta/vals must be float32 and idx int32")
        if idx.numel() != vals.numel():
            raise ValueError("idx and vals must have the same length")
        self._check(lib().scalecom_apply_update(self._ctx, ctypes.c_void_p(theta.data_ptr()), theta.numel(),
                                                ctypes.c_void_p(idx.data_ptr()), ctypes.c_void_p(vals.data_ptr()),
                                                idx.numel(), scale))

    def scalecom_hamming_distance(self, mem: Sequence[torch.Tensor], grad: Sequence[torch.Tensor],
                                  offsets: Sequence[int], ks: Sequence[int], lr: float, step: int,
                                  d_out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """``scalecom_hamming_distance`` of the C-ABI; the scratch buffer is allocated on first use and kept."""
        self._check_buffers(mem, grad, offsets[-1] if len(offsets) else None)
        n_tensors = len(ks)
        if len(offsets) != n_tensors + 1:
            raise ValueError("offsets must have len(ks) + 1 entries")
        c_off = (ctypes.c_int64 * (n_tensors + 1))(*[int(o) for o in offsets])
        c_ks = (ctypes.c_int64 * n_tensors)(*[int(v) for v in ks])
        if self._diag_scratch is None:
            nbytes = lib().scalecom_hamming_scratch_bytes(self.numel_max, self.n_tensors_max)
            self._diag_scratch = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        if d_out is None:
            d_out = torch.empty(n_tensors, dtype=torch.int32, device=self.device)
        elif d_out.dtype != torch.int32 or d_out.numel() < n_tensors:
            raise TypeError("d_out must be int32 with one entry per tensor")
        st = lib().scalecom_hamming_distance(self._ctx, _ptrs(mem), _ptrs(grad), len(mem), n_tensors, c_off, c_ks, lr,
                                             step, ctypes.c_void_p(self._diag_scratch.data_ptr()),
                                             self._diag_scratch.numel(), ctypes.c_void_p(d_out.data_ptr()))
        self._check(st)
        return d_out

    def scalecom_cosine_distance(self, a: torch.Tensor, b: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """``scalecom_cosine_distance`` of the C-ABI; returns the 4 doubles (distance, a.b, a.a, b.b)."""
        if a.dtype != torch.float32 or b.dtype != torch.float32 or a.numel() != b.numel():
            raise TypeError("a and b must be float32 vectors of one length")
        if not (a.is_contiguous() and b.is_contiguous() and a.device == self.device and b.device == self.device):
            raise ValueError("a and b must be contiguous tensors on the context's device")
        if out is None:
            out = torch.empty(4, dtype=torch.float64, device=self.device)
        elif out.dtype != torch.float64 or out.numel() < 4:
            raise TypeError("out must hold 4 float64 values")
        self._check(lib().scalecom_cosine_distance(self._ctx, ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(b.data_ptr()),
                                                   a.numel(), ctypes.c_void_p(out.data_ptr())))
        return out

    def scalecom_stream_copy(self, dst: torch.Tensor, src: torch.Tensor) -> None:
        nbytes = src.numel() * src.element_size()
        if dst.numel() * dst.element_size() != nbytes:
            raise ValueError("dst and src must have the same size in bytes")
        self._check(lib().scalecom_stream_copy(self._ctx, ctypes.c_void_p(dst.data_ptr()),
                                               ctypes.c_void_p(src.data_ptr()), nbytes))

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx:
            lib().scalecom_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def scalecom_init(numel_max: int, n_learners_max: int, grad_dtype: torch.dtype = torch.float32,
                  n_tensors_max: int = 1, device=None, stream=None, k_max: Optional[int] = None) -> ScaleCom:
    """``scalecom_init`` of the C-ABI, with the workspace taken from torch (``k_max`` defaults to
    ``numel_max``: any k is then accepted, at the price of a larger workspace)."""
    return ScaleCom(numel_max, n_learners_max, grad_dtype, n_tensors_max, device, stream, k_max)
