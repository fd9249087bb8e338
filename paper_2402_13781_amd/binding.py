"""Thin ctypes binding over libexdyna.so (the C ABI declared in include/exdyna.h).

Argument marshalling only.  torch supplies device memory (gradient, residual,
workspace) and the HIP stream; every step of the path runs in the library's
kernels.  There is no CPU fallback: a missing library raises at first use.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libexdyna.so")

EXDYNA_F32, EXDYNA_BF16, EXDYNA_F16 = 0, 1, 2
EXDYNA_OK, EXDYNA_EINVAL, EXDYNA_ENULL, EXDYNA_EALIGN, EXDYNA_ESTATE, EXDYNA_ENOMEM, EXDYNA_EHIP = (
    0, -1, -2, -3, -4, -5, -6)

# every symbol include/exdyna.h declares
SYMBOLS = (
    "exdyna_default_config", "exdyna_block_size_from_nb", "exdyna_workspace_bytes", "exdyna_init",
    "exdyna_init_static",
    "exdyna_step", "exdyna_step_scaled", "exdyna_worker_select", "exdyna_worker_exchange",
    "exdyna_apply_update", "exdyna_get_selected", "exdyna_get_count_pointers", "exdyna_get_partitions", "exdyna_get_block_counts",
    "exdyna_get_part_counts", "exdyna_get_stats", "exdyna_get_dims", "exdyna_set_profiling",
    "exdyna_get_kernel_ms", "exdyna_state_bytes", "exdyna_get_state", "exdyna_set_state",
    "exdyna_strerror", "exdyna_last_hip_error", "exdyna_destroy",
)


class Config(C.Structure):
    _fields_ = [
        ("n_g", C.c_uint64), ("block_size", C.c_uint32), ("n_parts", C.c_uint32),
        ("density", C.c_double), ("threshold0", C.c_float), ("cmp_mode", C.c_uint32),
        ("alpha", C.c_double), ("beta", C.c_double), ("gamma", C.c_double),
        ("blk_move", C.c_uint32), ("min_blk", C.c_uint32), ("max_selected", C.c_uint64),
        ("want_err_norm", C.c_uint32), ("reserved", C.c_uint32),
    ]


class Stats(C.Structure):
    _fields_ = [
        ("t", C.c_uint64), ("k_actual", C.c_uint64), ("k_emitted", C.c_uint64),
        ("k_max_part", C.c_uint64), ("density_error", C.c_double), ("traffic_ratio", C.c_double),
        ("err_norm", C.c_double), ("delta_used", C.c_float), ("delta_next", C.c_float),
        ("overflow", C.c_uint32), ("moves", C.c_uint32),
        ("bad_index", C.c_uint32), ("reserved", C.c_uint32), ("padding_overhead", C.c_uint64),
    ]


class ExDynaError(RuntimeError):
    def __init__(self, code: int, what: str, detail: str = ""):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code}){' -- ' + detail if detail else ''}")


_lib = None


def load() -> C.CDLL:
    """Load libexdyna.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2402_13781_amd.build` "
            "(hipcc --offload-arch=gfx950).  There is no CPU fallback.")
    L = C.CDLL(LIB_PATH)
    vp, u64, u32, P = C.c_void_p, C.c_uint64, C.c_uint32, C.POINTER
    L.exdyna_default_config.argtypes = [P(Config)]
    L.exdyna_block_size_from_nb.argtypes = [u64, u64, u32, P(u32)]
    L.exdyna_workspace_bytes.argtypes = [P(Config), P(C.c_size_t)]
    L.exdyna_init.argtypes = [P(vp), P(Config), vp, vp, C.c_size_t, vp]
    L.exdyna_init_static.argtypes = [P(vp), P(Config), vp, vp, vp, vp]
    L.exdyna_step.argtypes = [vp, vp, vp]
    L.exdyna_step_scaled.argtypes = [vp, vp, C.c_int, C.c_float, vp]
    L.exdyna_worker_select.argtypes = [vp, vp, C.c_int, C.c_float, u32, vp]
    L.exdyna_worker_exchange.argtypes = [vp, vp, vp, u64, vp, vp]
    L.exdyna_get_selected.argtypes = [vp, P(vp), P(vp), P(vp), P(u64), P(u64)]
    L.exdyna_apply_update.argtypes = [vp, vp, vp, vp, vp, u32, u64, C.c_float, vp]
    L.exdyna_get_count_pointers.argtypes = [vp, P(vp), P(vp)]
    L.exdyna_get_partitions.argtypes = [vp, C.c_int, P(u32), P(u32), P(u64), P(u64), P(u32)]
    L.exdyna_get_block_counts.argtypes = [vp, P(u32)]
    L.exdyna_get_part_counts.argtypes = [vp, P(u64)]
    L.exdyna_get_stats.argtypes = [vp, P(Stats)]
    L.exdyna_get_dims.argtypes = [vp, P(u64), P(u64)]
    L.exdyna_set_profiling.argtypes = [vp, u32, u32]
    L.exdyna_get_kernel_ms.argtypes = [vp, u64, P(C.c_float)]
    L.exdyna_state_bytes.argtypes = [vp, P(C.c_size_t)]
    L.exdyna_get_state.argtypes = [vp, vp, C.c_size_t]
    L.exdyna_set_state.argtypes = [vp, vp, C.c_size_t, vp]
    L.exdyna_strerror.argtypes = [C.c_int]
    L.exdyna_strerror.restype = C.c_char_p
    L.exdyna_last_hip_error.argtypes = [vp]
    L.exdyna_last_hip_error.restype = C.c_char_p
    L.exdyna_destroy.argtypes = [vp]
    for name in SYMBOLS:
        fn = getattr(L, name)
        if name not in ("exdyna_strerror", "exdyna_last_hip_error"):
            fn.restype = C.c_int
    _lib = L
    return L


def strerror(code: int) -> str:
    return load().exdyna_strerror(code).decode()


def default_config(**kw) -> Config:
    cfg = Config()
    rc = load().exdyna_default_config(C.byref(cfg))
    if rc:
        raise ExDynaError(rc, "exdyna_default_config")
    for k, v in kw.items():
        if not hasattr(cfg, k):
            raise AttributeError(k)
        setattr(cfg, k, v)
    return cfg


def block_size_from_nb(n_g: int, n_b: int, multiple: int = 256) -> int:
    out = C.c_uint32()
    rc = load().exdyna_block_size_from_nb(n_g, n_b, multiple, C.byref(out))
    if rc:
        raise ExDynaError(rc, "exdyna_block_size_from_nb")
    return out.value


def workspace_bytes(cfg: Config) -> int:
    out = C.c_size_t()
    rc = load().exdyna_workspace_bytes(C.byref(cfg), C.byref(out))
    if rc:
        raise ExDynaError(rc, "exdyna_workspace_bytes")
    return out.value


class ExDyna:
    """One sparsifier context on the current torch device.

    Owns (through torch) the residual vector and the workspace the library lays
    its state, counters, staging slots and output pairs in.
    """

    def __init__(self, cfg: Config, device="cuda:0", stream=None, static_scratch: bool = False):
        """static_scratch: create the context with exdyna_init_static (the library's built-in
        device array instead of a torch workspace; cfg.max_selected must be set)."""
        import torch

        self._torch = torch
        self._L = load()
        self.cfg = cfg
        self.device = torch.device(device)
        self._h = C.c_void_p()
        nbytes = workspace_bytes(cfg)            # validates the configuration on the host
        self.workspace = self.out_idx = self.out_val = None
        with torch.cuda.device(self.device):
            self.residual = torch.empty(cfg.n_g, dtype=torch.float32, device=self.device)
            if static_scratch:
                self.out_idx = torch.empty(max(cfg.max_selected, 1), dtype=torch.int32, device=self.device)
                self.out_val = torch.empty(max(cfg.max_selected, 1), dtype=torch.float32, device=self.device)
                rc = self._L.exdyna_init_static(C.byref(self._h), C.byref(cfg), self.residual.data_ptr(),
                                                self.out_idx.data_ptr(), self.out_val.data_ptr(),
                                                self._stream_ptr(stream))
            else:
                self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
                rc = self._L.exdyna_init(C.byref(self._h), C.byref(cfg), self.residual.data_ptr(),
                                         self.workspace.data_ptr(), nbytes, self._stream_ptr(stream))
        if rc:
            raise ExDynaError(rc, "exdyna_init_static" if static_scratch else "exdyna_init")
        nb, cap = C.c_uint64(), C.c_uint64()
        self._L.exdyna_get_dims(self._h, C.byref(nb), C.byref(cap))
        self.n_blocks, self.capacity = nb.value, cap.value
        self.P = cfg.n_parts

    # -- plumbing ---------------------------------------------------------
    def _stream_ptr(self, stream):
        if stream is None:
            stream = self._torch.cuda.current_stream(self.device)
        return C.c_void_p(stream.cuda_stream)

    def _check(self, rc, what):
        if rc:
            detail = self._L.exdyna_last_hip_error(self._h).decode() if rc == EXDYNA_EHIP else ""
            raise ExDynaError(rc, what, detail)

    def _view(self, ptr: int, n: int, dtype):
        """A torch view of `n` items of device memory the library handed out at address `ptr`:
        inside the torch workspace, inside the caller's output arrays, or (built-in context)
        inside the library's own device array."""
        torch = self._torch
        item = torch.empty((), dtype=dtype).element_size()
        for base in (self.workspace, self.out_idx, self.out_val):
            if base is None:
                continue
            off = ptr - base.data_ptr()
            if 0 <= off and off + n * item <= base.numel() * base.element_size():
                return base.view(torch.uint8)[off: off + n * item].view(dtype)
        assert self.workspace is None, "pointer outside the workspace"
        if n == 0:
            return torch.empty(0, dtype=dtype, device=self.device)

        class _Raw:          # memory torch did not allocate, described by its address
            __cuda_array_interface__ = {"shape": (n * item,), "typestr": "|u1", "data": (ptr, False),
                                        "version": 2}
        return torch.as_tensor(_Raw(), device=self.device).view(dtype)

    def close(self):
        if self._h:
            self._torch.cuda.synchronize(self.device)
            self._L.exdyna_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the C ABI, same names ---------------------------------------------
    def step(self, grad, stream=None):
        """exdyna_step: enqueue one iteration on `grad` (n_g fp32 on this device)."""
        torch = self._torch
        if grad.dtype != torch.float32 or grad.device != self.device or not grad.is_contiguous() \
                or grad.numel() != self.cfg.n_g:
            raise ValueError("grad must be a contiguous fp32 tensor of n_g elements on the context's device")
        self._check(self._L.exdyna_step(self._h, C.c_void_p(grad.data_ptr()), self._stream_ptr(stream)),
                    "exdyna_step")

    def step_scaled(self, grad, eta: float, stream=None):
        """exdyna_step_scaled: acc = e + eta * grad with fp32, bf16 or fp16 gradients."""
        torch = self._torch
        dt = {torch.float32: EXDYNA_F32, torch.bfloat16: EXDYNA_BF16, torch.float16: EXDYNA_F16}.get(grad.dtype)
        if dt is None or grad.device != self.device or not grad.is_contiguous() \
                or grad.numel() != self.cfg.n_g:
            raise ValueError("grad must be a contiguous fp32/bf16/fp16 tensor of n_g elements on the context's device")
        self._check(self._L.exdyna_step_scaled(self._h, C.c_void_p(grad.data_ptr()), dt, float(eta),
                                               self._stream_ptr(stream)), "exdyna_step_scaled")

    def _grad_dtype(self, grad):
        torch = self._torch
        dt = {torch.float32: EXDYNA_F32, torch.bfloat16: EXDYNA_BF16, torch.float16: EXDYNA_F16}.get(grad.dtype)
        if dt is None or grad.device != self.device or not grad.is_contiguous() \
                or grad.numel() != self.cfg.n_g:
            raise ValueError("grad must be a contiguous fp32/bf16/fp16 tensor of n_g elements on the context's device")
        return dt

    def worker_select(self, grad, rank: int, eta: float = 1.0, stream=None):
        """exdyna_worker_select: worker `rank`'s accumulate and selection of its own partition."""
        self._check(self._L.exdyna_worker_select(self._h, C.c_void_p(grad.data_ptr()), self._grad_dtype(grad),
                                                 float(eta), int(rank), self._stream_ptr(stream)),
                    "exdyna_worker_select")

    def worker_exchange(self, idx_all, counts_by_rank, val_all, stream=None):
        """exdyna_worker_exchange.  idx_all: int32/uint32-bits tensor [P, stride]; counts_by_rank: int64 [P];
        val_all: float32 [P, stride], written.  All on the context's device, contiguous."""
        torch = self._torch
        P = self.P
        if counts_by_rank.dtype != torch.int64 or counts_by_rank.numel() != P or not counts_by_rank.is_contiguous() \
                or counts_by_rank.device != self.device:
            raise ValueError("counts_by_rank must be a contiguous int64 tensor of n_parts entries on the device")
        if idx_all.dim() != 2 or idx_all.shape[0] != P or idx_all.dtype != torch.int32 or not idx_all.is_contiguous() \
                or idx_all.device != self.device:
            raise ValueError("idx_all must be a contiguous int32 tensor [n_parts, stride] on the device")
        if val_all.shape != idx_all.shape or val_all.dtype != torch.float32 or not val_all.is_contiguous() \
                or val_all.device != self.device:
            raise ValueError("val_all must be a contiguous float32 tensor shaped like idx_all on the device")
        stride = int(idx_all.shape[1])
        self._check(self._L.exdyna_worker_exchange(
            self._h, C.c_void_p(idx_all.data_ptr() if stride else None), C.c_void_p(counts_by_rank.data_ptr()),
            stride, C.c_void_p(val_all.data_ptr() if stride else None), self._stream_ptr(stream)),
            "exdyna_worker_exchange")

    def get_selected(self):
        """exdyna_get_selected: (idx[int32 view of u32], val[fp32], part_off[int64], k_actual, k_emitted)."""
        torch = self._torch
        pi, pv, po = C.c_void_p(), C.c_void_p(), C.c_void_p()
        ka, ke = C.c_uint64(), C.c_uint64()
        self._check(self._L.exdyna_get_selected(self._h, C.byref(pi), C.byref(pv), C.byref(po),
                                                C.byref(ka), C.byref(ke)), "exdyna_get_selected")
        idx = self._view(pi.value, ke.value, torch.int32)
        val = self._view(pv.value, ke.value, torch.float32)
        off = self._view(po.value, self.P + 1, torch.int64)
        return idx, val, off, ka.value, ke.value

    def apply_update(self, model, idx, val, counts, scale: float, stream=None):
        """exdyna_apply_update: model[idx] -= scale * val for the first counts[r] entries of every row.
        idx int32 [rows, stride], val float32 [rows, stride], counts int64 [rows], all on the device."""
        torch = self._torch
        if model.dtype != torch.float32 or model.numel() != self.cfg.n_g or not model.is_contiguous() \
                or model.device != self.device:
            raise ValueError("model must be a contiguous fp32 tensor of n_g elements on the context's device")
        if idx.dim() != 2 or idx.dtype != torch.int32 or not idx.is_contiguous() or val.shape != idx.shape \
                or val.dtype != torch.float32 or not val.is_contiguous() or counts.dtype != torch.int64 \
                or counts.numel() != idx.shape[0] or not counts.is_contiguous():
            raise ValueError("idx int32 [rows, stride], val float32 [rows, stride], counts int64 [rows], contiguous")
        rows, stride = int(idx.shape[0]), int(idx.shape[1])
        self._check(self._L.exdyna_apply_update(
            self._h, C.c_void_p(model.data_ptr()), C.c_void_p(idx.data_ptr() if stride else None),
            C.c_void_p(val.data_ptr() if stride else None), C.c_void_p(counts.data_ptr()), rows, stride,
            float(scale), self._stream_ptr(stream)), "exdyna_apply_update")

    def count_tensors(self):
        """exdyna_get_count_pointers as two 1-element int64 views of the workspace: (k_actual, k_emitted)
        of the last selection pass, readable on the device without a host round trip."""
        torch = self._torch
        pa, pe = C.c_void_p(), C.c_void_p()
        self._check(self._L.exdyna_get_count_pointers(self._h, C.byref(pa), C.byref(pe)),
                    "exdyna_get_count_pointers")
        return self._view(pa.value, 1, torch.int64), self._view(pe.value, 1, torch.int64)

    def get_partitions(self, which: int = 0):
        """exdyna_get_partitions: dict of numpy arrays (blk_pos, blk_part, elem_start, elem_end, owner_rank)."""
        import numpy as np
        P = self.P
        pos, part, own = (np.empty(P, np.uint32) for _ in range(3))
        st, en = (np.empty(P, np.uint64) for _ in range(2))
        u32p, u64p = C.POINTER(C.c_uint32), C.POINTER(C.c_uint64)
        self._check(self._L.exdyna_get_partitions(
            self._h, which, pos.ctypes.data_as(u32p), part.ctypes.data_as(u32p),
            st.ctypes.data_as(u64p), en.ctypes.data_as(u64p), own.ctypes.data_as(u32p)),
            "exdyna_get_partitions")
        return dict(blk_pos=pos, blk_part=part, elem_start=st, elem_end=en, owner_rank=own)

    def get_block_counts(self):
        import numpy as np
        out = np.empty(self.n_blocks, np.uint32)
        self._check(self._L.exdyna_get_block_counts(self._h, out.ctypes.data_as(C.POINTER(C.c_uint32))),
                    "exdyna_get_block_counts")
        return out

    def get_part_counts(self):
        import numpy as np
        out = np.empty(self.P, np.uint64)
        self._check(self._L.exdyna_get_part_counts(self._h, out.ctypes.data_as(C.POINTER(C.c_uint64))),
                    "exdyna_get_part_counts")
        return out

    def get_stats(self) -> Stats:
        st = Stats()
        self._check(self._L.exdyna_get_stats(self._h, C.byref(st)), "exdyna_get_stats")
        return st

    def get_state(self) -> bytes:
        """exdyna_get_state: the saved state as bytes (the residual is `self.residual`)."""
        n = C.c_size_t()
        self._check(self._L.exdyna_state_bytes(self._h, C.byref(n)), "exdyna_state_bytes")
        buf = (C.c_char * n.value)()
        self._check(self._L.exdyna_get_state(self._h, buf, n.value), "exdyna_get_state")
        return bytes(buf)

    def set_state(self, state: bytes, stream=None):
        """exdyna_set_state: resume from `state`; restore `self.residual` separately."""
        buf = (C.c_char * len(state)).from_buffer_copy(state)
        self._check(self._L.exdyna_set_state(self._h, buf, len(state), self._stream_ptr(stream)),
                    "exdyna_set_state")

    def set_profiling(self, n_slots: int, every: int = 1):
        self._check(self._L.exdyna_set_profiling(self._h, int(n_slots), int(every)), "exdyna_set_profiling")

    def get_kernel_ms(self, iteration: int):
        """[streaming pass, finishing kernel] milliseconds of a profiled iteration."""
        out = (C.c_float * 2)()
        self._check(self._L.exdyna_get_kernel_ms(self._h, iteration, out), "exdyna_get_kernel_ms")
        return [out[0], out[1]]
