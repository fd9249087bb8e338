"""ctypes access to the C oracle (exdyna_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Argument marshalling only: every number the oracle reports is computed by the
C file, whose functions cite the passages of the paper they follow.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "exdyna_oracle.c")
_LIB = os.path.join(_HERE, "libexdyna_oracle.so")

_lib = None


def lib_path() -> str:
    return _LIB


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(
        os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "exdyna_oracle.h"))
    ):
        cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = C.CDLL(_LIB)
    u64, u32, i64, f32, f64, vp = C.c_uint64, C.c_uint32, C.c_int64, C.c_float, C.c_double, C.c_void_p
    P = C.POINTER
    L.exo_block_size.restype = u64
    L.exo_block_size.argtypes = [u64, u64]
    L.exo_partition.restype = None
    L.exo_partition.argtypes = [u64, u32, P(i64), P(i64)]
    L.exo_allocate.restype = C.c_int
    L.exo_allocate.argtypes = [P(f64), P(i64), P(i64), u32, u64, u64, i64, i64, f64]
    L.exo_owner.restype = u32
    L.exo_owner.argtypes = [u64, u32, u32]
    L.exo_select.restype = u64
    L.exo_select.argtypes = [P(f32), u64, u64, f32, C.c_int, P(u32), u64]
    L.exo_scale_factor.restype = f32
    L.exo_scale_factor.argtypes = [f64, f64, f64, f64]
    L.exo_estimate.restype = f32
    L.exo_estimate.argtypes = [f64, f64, f32, f64, f64]
    L.exo_create.restype = vp
    L.exo_create.argtypes = [u64, u32, u32, f64, f32, f64, f64, f64, u32, u32, u32, u64]
    L.exo_destroy.restype = None
    L.exo_destroy.argtypes = [vp]
    L.exo_step.restype = None
    L.exo_step.argtypes = [vp, P(f32)]
    L.exo_step_scaled.restype = None
    L.exo_step_scaled.argtypes = [vp, vp, C.c_int, f32]
    for name, rt in [("exo_n_blocks", u64), ("exo_capacity", u64), ("exo_iteration", u64),
                     ("exo_threshold", f32), ("exo_threshold_used", f32),
                     ("exo_residual", P(f32)), ("exo_out_idx", P(u32)), ("exo_out_val", P(f32)),
                     ("exo_part_off", P(u64)), ("exo_part_count", P(u64)),
                     ("exo_block_count", P(u32)), ("exo_k_actual", u64), ("exo_k_emitted", u64),
                     ("exo_err_norm", f64), ("exo_density_error", f64),
                     ("exo_traffic_ratio", f64)]:
        fn = getattr(L, name)
        fn.restype = rt
        fn.argtypes = [vp]
    for name in ("exo_blk_part", "exo_blk_pos", "exo_workers_blk_part", "exo_workers_blk_pos"):
        fn = getattr(L, name)
        fn.restype = P(i64)
        fn.argtypes = [vp, C.c_int]
    L.exo_padding_overhead.restype = u64
    L.exo_padding_overhead.argtypes = [P(u64), u32]
    L.exo_apply_update.restype = None
    L.exo_apply_update.argtypes = [P(f32), P(u32), P(f32), u64, f32]
    L.exo_reindex.restype = None
    L.exo_reindex.argtypes = [P(f64), u32, u64, P(f64)]
    L.exo_workers_create.restype = vp
    L.exo_workers_create.argtypes = [u64, u32, u32, f64, f32, f64, f64, f64, u32, u32, u32, u64]
    L.exo_workers_destroy.restype = None
    L.exo_workers_destroy.argtypes = [vp]
    L.exo_workers_step.restype = None
    L.exo_workers_step.argtypes = [vp, P(P(f32))]
    for name, rt in [("exo_workers_capacity", u64), ("exo_workers_n_blocks", u64),
                     ("exo_workers_iteration", u64), ("exo_workers_threshold", f32),
                     ("exo_workers_threshold_used", f32), ("exo_workers_k_rank", P(u64)),
                     ("exo_workers_rank_off", P(u64)), ("exo_workers_idx", P(u32)),
                     ("exo_workers_sum", P(f32)), ("exo_workers_k_actual", u64),
                     ("exo_workers_traffic_ratio", f64)]:
        fn = getattr(L, name)
        fn.restype = rt
        fn.argtypes = [vp]
    for name, rt in [("exo_workers_residual", P(f32)), ("exo_workers_values", P(f32)),
                     ("exo_workers_err_norm", f64)]:
        fn = getattr(L, name)
        fn.restype = rt
        fn.argtypes = [vp, u32]
    _lib = L
    return L


def _ptr(a: np.ndarray, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def block_size(n_g: int, n_b: int) -> int:
    return int(_load().exo_block_size(n_g, n_b))


def partition(n_b: int, n: int):
    bp = np.empty(n, np.int64)
    pos = np.empty(n, np.int64)
    _load().exo_partition(n_b, n, _ptr(bp, C.c_int64), _ptr(pos, C.c_int64))
    return bp, pos


def allocate(kvec, blk_part, blk_pos, n_g, sz_blk, blk_move=1, min_blk=1, alpha=1.0):
    """Returns (kvec', blk_part', blk_pos', moves); inputs are not modified."""
    kv = np.array(kvec, np.float64)
    bp = np.array(blk_part, np.int64)
    pos = np.array(blk_pos, np.int64)
    moves = _load().exo_allocate(_ptr(kv, C.c_double), _ptr(bp, C.c_int64), _ptr(pos, C.c_int64),
                                 len(kv), n_g, sz_blk, blk_move, min_blk, alpha)
    return kv, bp, pos, int(moves)


def owner(t: int, rank: int, n: int) -> int:
    return int(_load().exo_owner(t, rank, n))


def select(acc: np.ndarray, st: int, end: int, delta: float, cmp_mode: int = 0):
    acc = np.ascontiguousarray(acc, np.float32)
    cap = max(end - st, 1)
    out = np.empty(cap, np.uint32)
    cnt = _load().exo_select(_ptr(acc, C.c_float), st, end, np.float32(delta), cmp_mode,
                             _ptr(out, C.c_uint32), cap)
    return out[: int(cnt)].copy()


def scale_factor(k, k_actual, beta, gamma) -> float:
    return float(_load().exo_scale_factor(k, k_actual, beta, gamma))


def estimate(k, k_actual, delta, beta, gamma) -> float:
    return float(_load().exo_estimate(k, k_actual, np.float32(delta), beta, gamma))


def padding_overhead(counts) -> int:
    """Eq. 2-4: C_t from the per-worker (= per-partition) selection counts."""
    k = np.ascontiguousarray(counts, np.uint64)
    return int(_load().exo_padding_overhead(_ptr(k, C.c_uint64), k.size))


def apply_update(x: np.ndarray, idx_t: np.ndarray, g_t: np.ndarray, scale: float):
    """Alg. 1 (model update) on the sent entries, in place on the float32 array x."""
    assert x.dtype == np.float32 and x.flags.c_contiguous
    idx = np.ascontiguousarray(idx_t, np.uint32)
    g = np.ascontiguousarray(g_t, np.float32)
    assert idx.size == g.size
    _load().exo_apply_update(_ptr(x, C.c_float), _ptr(idx, C.c_uint32), _ptr(g, C.c_float), idx.size,
                             np.float32(scale))


def reindex(k_rank, t: int):
    """Alg. 3 (re-indexing of the partial-k vector): partial-k vector from rank order to partition order."""
    kr = np.array(k_rank, np.float64)
    out = np.empty_like(kr)
    _load().exo_reindex(_ptr(kr, C.c_double), len(kr), t, _ptr(out, C.c_double))
    return out


class Workers:
    """Alg. 1 for n workers with their own gradients and residuals (exo_workers_*)."""

    def __init__(self, n_g, block_size, n, density, threshold0, alpha=1.0, beta=1.1,
                 gamma=0.01, blk_move=1, min_blk=1, cmp_mode=0, max_selected=0):
        self._L = _load()
        self._h = self._L.exo_workers_create(n_g, block_size, n, density, np.float32(threshold0),
                                             alpha, beta, gamma, blk_move, min_blk, cmp_mode,
                                             max_selected)
        if not self._h:
            raise ValueError("exo_workers_create rejected the configuration")
        self.n_g, self.b, self.n = n_g, block_size, n
        self.n_b = int(self._L.exo_workers_n_blocks(self._h))
        self.cap = int(self._L.exo_workers_capacity(self._h))

    def close(self):
        if self._h:
            self._L.exo_workers_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, grads):
        """grads: n contiguous float32 arrays of n_g elements, one per worker."""
        assert len(grads) == self.n
        for g in grads:
            assert g.dtype == np.float32 and g.flags.c_contiguous and g.size == self.n_g
        arr = (C.POINTER(C.c_float) * self.n)(*[_ptr(g, C.c_float) for g in grads])
        self._L.exo_workers_step(self._h, arr)

    def _arr(self, p, n, dtype):
        if n == 0:
            return np.empty(0, dtype)
        return np.ctypeslib.as_array(p, shape=(n,)).astype(dtype, copy=True)

    @property
    def t(self): return int(self._L.exo_workers_iteration(self._h))
    @property
    def threshold(self): return np.float32(self._L.exo_workers_threshold(self._h))
    @property
    def threshold_used(self): return np.float32(self._L.exo_workers_threshold_used(self._h))
    @property
    def k_actual(self): return int(self._L.exo_workers_k_actual(self._h))

    def residual(self, i, copy=True):
        a = np.ctypeslib.as_array(self._L.exo_workers_residual(self._h, i), shape=(self.n_g,))
        return a.copy() if copy else a

    def k_rank(self): return self._arr(self._L.exo_workers_k_rank(self._h), self.n, np.uint64)
    def rank_off(self): return self._arr(self._L.exo_workers_rank_off(self._h), self.n + 1, np.uint64)
    def idx(self): return self._arr(self._L.exo_workers_idx(self._h), int(self.rank_off()[-1]), np.uint32)
    def values(self, i): return self._arr(self._L.exo_workers_values(self._h, i), int(self.rank_off()[-1]), np.float32)
    def sum(self): return self._arr(self._L.exo_workers_sum(self._h), int(self.rank_off()[-1]), np.float32)
    def blk_part(self, which=0): return self._arr(self._L.exo_workers_blk_part(self._h, which), self.n, np.int64)
    def blk_pos(self, which=0): return self._arr(self._L.exo_workers_blk_pos(self._h, which), self.n, np.int64)
    def err_norm(self, i=None): return float(self._L.exo_workers_err_norm(self._h, self.n if i is None else i))
    def traffic_ratio(self): return float(self._L.exo_workers_traffic_ratio(self._h))


class Oracle:
    """The whole-step state machine (Alg. 1 (initialisation and iteration body)) behind exo_create/exo_step."""

    def __init__(self, n_g, block_size, n_parts, density, threshold0, alpha=1.0, beta=1.1,
                 gamma=0.01, blk_move=1, min_blk=1, cmp_mode=0, max_selected=0):
        self._L = _load()
        self._h = self._L.exo_create(n_g, block_size, n_parts, density, np.float32(threshold0),
                                     alpha, beta, gamma, blk_move, min_blk, cmp_mode, max_selected)
        if not self._h:
            raise ValueError("exo_create rejected the configuration")
        self.n_g, self.b, self.P = n_g, block_size, n_parts
        self.n_b = int(self._L.exo_n_blocks(self._h))
        self.cap = int(self._L.exo_capacity(self._h))

    def close(self):
        if self._h:
            self._L.exo_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, g: np.ndarray):
        assert g.dtype == np.float32 and g.flags.c_contiguous and g.size == self.n_g
        self._L.exo_step(self._h, _ptr(g, C.c_float))

    def step_scaled(self, g: np.ndarray, dtype: int, eta: float):
        """g: float32 array (dtype 0) or uint16 array of bf16 (1) / fp16 (2) bit patterns."""
        assert g.flags.c_contiguous and g.size == self.n_g
        assert g.dtype == (np.float32 if dtype == 0 else np.uint16)
        self._L.exo_step_scaled(self._h, g.ctypes.data_as(C.c_void_p), dtype, np.float32(eta))

    # --- views (copied so they survive the next step) ---
    def _arr(self, p, n, dtype):
        if n == 0:
            return np.empty(0, dtype)
        return np.ctypeslib.as_array(p, shape=(n,)).astype(dtype, copy=True)

    @property
    def t(self): return int(self._L.exo_iteration(self._h))
    @property
    def threshold(self): return np.float32(self._L.exo_threshold(self._h))
    @property
    def threshold_used(self): return np.float32(self._L.exo_threshold_used(self._h))
    @property
    def k_actual(self): return int(self._L.exo_k_actual(self._h))
    @property
    def k_emitted(self): return int(self._L.exo_k_emitted(self._h))

    def residual(self, copy=True):
        a = np.ctypeslib.as_array(self._L.exo_residual(self._h), shape=(self.n_g,))
        return a.copy() if copy else a

    def set_residual(self, e: np.ndarray):
        a = np.ctypeslib.as_array(self._L.exo_residual(self._h), shape=(self.n_g,))
        a[:] = e

    def out_idx(self): return self._arr(self._L.exo_out_idx(self._h), self.k_emitted, np.uint32)
    def out_val(self): return self._arr(self._L.exo_out_val(self._h), self.k_emitted, np.float32)
    def part_off(self): return self._arr(self._L.exo_part_off(self._h), self.P + 1, np.uint64)
    def part_count(self): return self._arr(self._L.exo_part_count(self._h), self.P, np.uint64)
    def block_count(self): return self._arr(self._L.exo_block_count(self._h), self.n_b, np.uint32)
    def blk_part(self, which=0): return self._arr(self._L.exo_blk_part(self._h, which), self.P, np.int64)
    def blk_pos(self, which=0): return self._arr(self._L.exo_blk_pos(self._h, which), self.P, np.int64)
    def err_norm(self): return float(self._L.exo_err_norm(self._h))
    def density_error(self): return float(self._L.exo_density_error(self._h))
    def traffic_ratio(self): return float(self._L.exo_traffic_ratio(self._h))
