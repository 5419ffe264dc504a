"""ctypes front end of the plain CPU oracle (``asyncmesh_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the benchmark's CPU
baseline leg.  The product path never imports this module, and this module imports nothing of
the product.
"""
from __future__ import annotations

import ctypes as C
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "asyncmesh_oracle.c"
_LIB = _HERE / "libasyncmesh_oracle.so"

OPT_SGD, OPT_ADAMW, OPT_NADAMW = 0, 1, 2
CORR_NONE, CORR_EMA, CORR_EAGER = 0, 1, 2
SUBSET_BERNOULLI, SUBSET_STRATIFIED = 0, 1
MSG_F32, MSG_BF16, MSG_E4M3 = 0, 1, 2


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (OpenMP over coordinates, no fast-math, no FMA contraction)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", str(_LIB), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Config(C.Structure):
    _fields_ = [
        ("n", C.c_uint64), ("mu0", C.c_uint64),
        ("replicas", C.c_uint32), ("delay", C.c_uint32), ("avg_interval", C.c_uint32),
        ("optimizer", C.c_uint32),
        ("fraction", C.c_double), ("seed", C.c_uint64),
        ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double), ("weight_decay", C.c_double),
        ("gamma", C.c_double),
        ("lookahead", C.c_uint32), ("correction", C.c_uint32),
        ("fwd_bf16", C.c_uint32), ("grad_bf16", C.c_uint32),
        ("momentum_decay", C.c_double),
        ("granule", C.c_uint32), ("msg_dtype", C.c_uint32),
        ("stratified", C.c_uint32), ("reserved", C.c_uint32),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(str(_LIB))
        L.amo_philox4x32_10.argtypes = [C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        L.amo_threshold.argtypes = [C.c_double]; L.amo_threshold.restype = C.c_uint64
        L.amo_member.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32]; L.amo_member.restype = C.c_int
        L.amo_subset.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64, C.c_double, C.c_uint32, C.c_uint32,
                                 C.c_void_p, C.c_uint64]
        L.amo_subset.restype = C.c_uint64
        L.amo_block_size.argtypes = [C.c_double]; L.amo_block_size.restype = C.c_uint64
        L.amo_member_stratified.argtypes = [C.c_uint64] * 4; L.amo_member_stratified.restype = C.c_int
        L.amo_bf16_to_float.argtypes = [C.c_uint16]; L.amo_bf16_to_float.restype = C.c_float
        L.amo_double_to_bf16.argtypes = [C.c_double]; L.amo_double_to_bf16.restype = C.c_uint16
        L.amo_create.argtypes = [C.POINTER(_Config)]; L.amo_create.restype = C.c_void_p
        L.amo_destroy.argtypes = [C.c_void_p]
        for name in ("amo_w", "amo_m", "amo_v", "amo_d", "amo_fwd"):
            f = getattr(L, name)
            f.argtypes = [C.c_void_p, C.c_uint32]
            f.restype = C.POINTER(C.c_float)
        L.amo_step.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p), C.c_double, C.c_double, C.c_double]
        L.amo_step.restype = C.c_int
        L.amo_step_scaled.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p), C.c_double, C.c_double, C.c_double, C.c_void_p]
        L.amo_step_scaled.restype = C.c_int
        L.amo_step_masked.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p), C.c_double, C.c_double, C.c_double,
                                      C.c_void_p, C.c_uint32]
        L.amo_step_masked.restype = C.c_int
        L.amo_grad_sqnorm.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32]; L.amo_grad_sqnorm.restype = C.c_double
        L.amo_sparse_average.argtypes = [C.c_void_p, C.c_uint64, C.c_double]; L.amo_sparse_average.restype = C.c_int
        L.amo_lookahead.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_double]
        L.amo_consensus_error.argtypes = [C.c_void_p]; L.amo_consensus_error.restype = C.c_double
        L.amo_quantize_e4m3.argtypes = [C.c_double]; L.amo_quantize_e4m3.restype = C.c_double
        L.amo_quantize_message.argtypes = [C.c_float, C.c_uint32]; L.amo_quantize_message.restype = C.c_double
        L.amo_set_delay.argtypes = [C.c_void_p, C.c_uint32]; L.amo_set_delay.restype = C.c_int
        L.amo_ema_variance.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        _lib = L
    return _lib


def f32(x) -> float:
    """A Python float holding exactly the fp32 value nearest to x (hyper-parameters cross the
    product's C ABI as fp32; the oracle must be given those very values)."""
    return float(np.float32(x))


def philox4x32_10(counter, key):
    c = (C.c_uint32 * 4)(*counter)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    lib().amo_philox4x32_10(c, k, o)
    return tuple(int(x) for x in o)


def threshold(p: float) -> int:
    return int(lib().amo_threshold(p))


def member(seed: int, s: int, mu: int, p: float, granule: int = 1) -> bool:
    return bool(lib().amo_member(seed, s, mu, threshold(p), granule))


def block_size(p: float) -> int:
    """B = round(1/p) of the stratified sampling variant."""
    return int(lib().amo_block_size(p))


def member_stratified(seed: int, s: int, mu: int, p: float) -> bool:
    return bool(lib().amo_member_stratified(seed, s, mu, block_size(p)))


def subset(seed: int, s: int, n: int, p: float, mu0: int = 0, granule: int = 1, stratified: bool = False) -> np.ndarray:
    """Ascending global indices of S^s inside [mu0, mu0+n)."""
    L = lib()
    count = L.amo_subset(seed, s, mu0, n, p, granule, int(stratified), None, 0)
    out = np.empty(count, dtype=np.uint64)
    if count:
        L.amo_subset(seed, s, mu0, n, p, granule, int(stratified), out.ctypes.data, count)
    return out


def quantize_e4m3(x: float) -> float:
    return float(lib().amo_quantize_e4m3(x))


def quantize_message(x: float, msg_dtype: int) -> float:
    return float(lib().amo_quantize_message(x, msg_dtype))


def grad_sqnorm(g: np.ndarray) -> float:
    """Sum of squares of a gradient array (fp32, or bf16 given as uint16 bit patterns)."""
    g = np.ascontiguousarray(g)
    return float(lib().amo_grad_sqnorm(g.ctypes.data, g.size, int(g.dtype == np.uint16)))


def double_to_bf16(x: float) -> int:
    return int(lib().amo_double_to_bf16(x))


def bf16_to_float(h: int) -> float:
    return float(lib().amo_bf16_to_float(h))


def lookahead(w: np.ndarray, w_prev: np.ndarray, gamma: float, bf16: bool = False) -> np.ndarray:
    w = np.ascontiguousarray(w, dtype=np.float32)
    w_prev = np.ascontiguousarray(w_prev, dtype=np.float32)
    if bf16:
        out = np.empty(w.shape, dtype=np.uint16)
        lib().amo_lookahead(None, out.ctypes.data, w.ctypes.data, w_prev.ctypes.data, w.size, gamma)
    else:
        out = np.empty(w.shape, dtype=np.float32)
        lib().amo_lookahead(out.ctypes.data, None, w.ctypes.data, w_prev.ctypes.data, w.size, gamma)
    return out


class Oracle:
    """One pipeline stage replicated R times, advanced one step at a time on the CPU."""

    def __init__(self, n, replicas, delay=0, avg_interval=1, fraction=0.05, seed=0,
                 optimizer=OPT_ADAMW, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01,
                 lookahead=False, gamma=0.0, correction=CORR_EMA, fwd_bf16=False, grad_bf16=False,
                 momentum_decay=0.004, mu0=0, subset_granule=1, msg_dtype=MSG_F32, subset_kind=SUBSET_BERNOULLI):
        self.cfg = _Config(
            n=n, mu0=mu0, replicas=replicas, delay=delay, avg_interval=avg_interval, optimizer=optimizer,
            fraction=fraction, seed=seed, beta1=f32(beta1), beta2=f32(beta2), eps=f32(eps),
            weight_decay=f32(weight_decay), gamma=f32(gamma), lookahead=int(bool(lookahead)),
            correction=correction, fwd_bf16=int(bool(fwd_bf16)), grad_bf16=int(bool(grad_bf16)),
            momentum_decay=momentum_decay, granule=subset_granule, msg_dtype=msg_dtype,
            stratified=int(subset_kind == SUBSET_STRATIFIED), reserved=0)
        self.n, self.R = n, replicas
        self._h = lib().amo_create(C.byref(self.cfg))
        if not self._h:
            raise MemoryError("amo_create failed")

    def close(self):
        if self._h:
            lib().amo_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _view(self, name, i) -> np.ndarray:
        p = getattr(lib(), name)(self._h, i)
        if self.n == 0:
            return np.empty(0, dtype=np.float32)
        return np.ctypeslib.as_array(p, shape=(self.n,))

    def w(self, i): return self._view("amo_w", i)
    def m(self, i): return self._view("amo_m", i)
    def v(self, i): return self._view("amo_v", i)
    def d(self, i): return self._view("amo_d", i)
    def fwd(self, i): return self._view("amo_fwd", i)

    def set_w(self, w0):
        """Same starting point for every replica (1-D array), or one row per replica (2-D)."""
        w0 = np.asarray(w0, dtype=np.float32)
        for i in range(self.R):
            self.w(i)[:] = w0 if w0.ndim == 1 else w0[i]

    def step(self, t, grads, lr, lam=0.5, grad_scale=1.0, replica_scale=None):
        want = np.uint16 if self.cfg.grad_bf16 else np.float32
        keep = [np.ascontiguousarray(g, dtype=want) for g in grads]
        assert len(keep) == self.R and all(g.size == self.n for g in keep)
        ptrs = (C.c_void_p * self.R)(*[g.ctypes.data for g in keep])
        if replica_scale is not None:
            rs = np.ascontiguousarray(replica_scale, dtype=np.float32)
            assert rs.size == self.R
            rc = lib().amo_step_scaled(self._h, t, ptrs, f32(lr), f32(lam), f32(grad_scale), rs.ctypes.data)
        else:
            rc = lib().amo_step(self._h, t, ptrs, f32(lr), f32(lam), f32(grad_scale))
        if rc != 0:
            raise ValueError(f"oracle step out of order: t={t}")

    def step_masked(self, t, grads, lr, lam, active: int, grad_scale=1.0, replica_scale=None):
        """One tick of the heterogeneous set-up: replica i makes a local step iff bit i of `active`
        is set (grads[i] of the others may be None)."""
        want = np.uint16 if self.cfg.grad_bf16 else np.float32
        keep = [None if g is None else np.ascontiguousarray(g, dtype=want) for g in grads]
        assert len(keep) == self.R and all(g is None or g.size == self.n for g in keep)
        assert all(keep[i] is not None for i in range(self.R) if (active >> i) & 1)
        ptrs = (C.c_void_p * self.R)(*[None if g is None else g.ctypes.data for g in keep])
        rs = None if replica_scale is None else np.ascontiguousarray(replica_scale, dtype=np.float32)
        rc = lib().amo_step_masked(self._h, t, ptrs, f32(lr), f32(lam), f32(grad_scale),
                                   None if rs is None else rs.ctypes.data, active)
        if rc != 0:
            raise ValueError(f"oracle step out of order: t={t}")

    def sparse_average(self, t, lam=0.5):
        rc = lib().amo_sparse_average(self._h, t, f32(lam))
        if rc != 0:
            raise ValueError(f"oracle sparse_average out of order: t={t}")

    def consensus_error(self) -> float:
        return float(lib().amo_consensus_error(self._h))

    def ema_variance(self):
        """(mean, max) over the coordinates of the variance of d_i over the replicas."""
        a, b = C.c_double(0), C.c_double(0)
        lib().amo_ema_variance(self._h, C.byref(a), C.byref(b))
        return float(a.value), float(b.value)

    def set_delay(self, tau: int):
        if lib().amo_set_delay(self._h, tau) != 0:
            raise ValueError(f"delay {tau} exceeds the delay the oracle was created with")


def threads() -> int:
    """How many OpenMP threads the oracle's coordinate loops use."""
    L = lib()
    L.amo_threads.restype = C.c_int
    return int(L.amo_threads())
