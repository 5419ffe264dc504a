"""Thin ctypes binding of libasyncmesh.so (include/asyncmesh.h).

Argument marshalling only: every step of the update runs in the library's HIP kernels.  PyTorch
is used to own device memory and to name the stream.  There is no CPU fallback: importing this
module without the built library raises.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
_LIB_PATH = _PKG / "libasyncmesh.so"

MAX_REPLICAS = 32
OPT_SGD, OPT_ADAMW, OPT_NADAMW = 0, 1, 2
CORR_NONE, CORR_EMA, CORR_EAGER = 0, 1, 2
F32, BF16 = 0, 1
MSG_F32, MSG_BF16, MSG_E4M3 = 0, 1, 2
SUBSET_BERNOULLI, SUBSET_STRATIFIED = 0, 1
D_PER_REPLICA, D_INTERLEAVED = 0, 1

EXPORTS = (
    "am_workspace_bytes", "am_d_layout_info", "am_init_state", "am_step", "am_step_scaled", "am_step_masked", "am_grad_sqnorm", "am_sparse_average",
    "am_lookahead",
    "am_subset_indices", "am_subset_indices_static", "am_set_delay", "am_diagnostics", "am_read_flags", "am_set_profiling", "am_get_profile", "am_get_profile_times", "am_ring_info",
    "am_export_state", "am_resume_state",
    "am_destroy", "am_last_error", "am_version",
)


class AsyncMeshError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"asyncmesh error {status}: {message}")
        self.status = status


class Config(C.Structure):
    """Mirror of am_config."""
    _fields_ = [
        ("n", C.c_uint64),
        ("replicas", C.c_uint32), ("delay", C.c_uint32), ("avg_interval", C.c_uint32), ("optimizer", C.c_uint32),
        ("fraction", C.c_double), ("seed", C.c_uint64),
        ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("weight_decay", C.c_float),
        ("gamma", C.c_float),
        ("lookahead", C.c_uint32), ("correction", C.c_uint32), ("fwd_dtype", C.c_uint32), ("grad_dtype", C.c_uint32),
        ("momentum_decay", C.c_double),
        ("subset_granule", C.c_uint32), ("msg_dtype", C.c_uint32),
        ("subset_kind", C.c_uint32), ("d_layout", C.c_uint32),
        ("ring_cap_lines", C.c_uint64),
    ]


class Buffers(C.Structure):
    """Mirror of am_buffers."""
    _fields_ = [
        ("w", C.POINTER(C.c_void_p)), ("m", C.POINTER(C.c_void_p)), ("v", C.POINTER(C.c_void_p)),
        ("d", C.POINTER(C.c_void_p)), ("fwd", C.POINTER(C.c_void_p)),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_uint64),
    ]


class Snapshot(C.Structure):
    """Mirror of am_snapshot: what the library itself remembers between steps."""
    _fields_ = [
        ("magic", C.c_uint64), ("config_digest", C.c_uint64), ("last_t", C.c_uint64),
        ("next_lines_step", C.c_uint64),
        ("delay_now", C.c_uint32), ("reserved", C.c_uint32),
        ("opt_steps", C.c_uint64 * MAX_REPLICAS), ("mu_product", C.c_double * MAX_REPLICAS),
    ]


def _load():
    if not _LIB_PATH.exists():
        raise ImportError(
            f"{_LIB_PATH} is missing: build it first (python -m paper_2601_22442_amd.build, or "
            "__graft_entry__.build()).  There is no fallback path.")
    L = C.CDLL(str(_LIB_PATH))
    L.am_workspace_bytes.argtypes = [C.POINTER(Config), C.POINTER(C.c_uint64)]
    L.am_d_layout_info.argtypes = [C.POINTER(Config), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint64)]
    L.am_init_state.argtypes = [C.POINTER(Config), C.POINTER(Buffers), C.c_void_p, C.POINTER(C.c_void_p)]
    L.am_step.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p), C.c_float, C.c_float, C.c_float]
    L.am_step_scaled.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p), C.c_float, C.c_float, C.c_float, C.c_void_p]
    L.am_step_masked.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p), C.c_float, C.c_float, C.c_float, C.c_void_p, C.c_uint32]
    L.am_grad_sqnorm.argtypes = [C.c_void_p, C.POINTER(C.c_void_p), C.c_void_p]
    L.am_sparse_average.argtypes = [C.c_void_p, C.c_uint64, C.c_float]
    L.am_lookahead.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint64, C.c_float, C.c_void_p]
    L.am_subset_indices.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p]
    L.am_subset_indices_static.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p]
    L.am_set_delay.argtypes = [C.c_void_p, C.c_uint32]
    L.am_diagnostics.argtypes = [C.c_void_p, C.c_void_p]
    L.am_read_flags.argtypes = [C.c_void_p, C.POINTER(C.c_uint32)]
    L.am_set_profiling.argtypes = [C.c_void_p, C.c_int]
    L.am_get_profile.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
    L.am_get_profile_times.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.c_uint64, C.POINTER(C.c_uint64)]
    L.am_ring_info.argtypes = [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)]
    L.am_export_state.argtypes = [C.c_void_p, C.POINTER(Snapshot)]
    L.am_resume_state.argtypes = [C.POINTER(Config), C.POINTER(Buffers), C.c_void_p, C.POINTER(Snapshot), C.POINTER(C.c_void_p)]
    L.am_destroy.argtypes = [C.c_void_p]
    for name in EXPORTS:
        getattr(L, name).restype = C.c_int
    L.am_last_error.restype = C.c_char_p
    L.am_last_error.argtypes = []
    L.am_version.restype = C.c_char_p
    L.am_version.argtypes = []
    return L


lib = _load()


def _check(status: int):
    if status != 0:
        raise AsyncMeshError(status, lib.am_last_error().decode())


def version() -> str:
    return lib.am_version().decode()


def make_config(n, replicas, delay=0, avg_interval=1, fraction=0.05, seed=0, optimizer=OPT_ADAMW,
                beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, lookahead=False, gamma=0.0,
                correction=CORR_EMA, fwd_dtype=F32, grad_dtype=F32, momentum_decay=0.004,
                subset_granule=1, msg_dtype=MSG_F32, subset_kind=SUBSET_BERNOULLI, d_layout=D_PER_REPLICA,
                ring_cap_lines=0) -> Config:
    return Config(n=n, replicas=replicas, delay=delay, avg_interval=avg_interval, optimizer=optimizer,
                  fraction=fraction, seed=seed, beta1=beta1, beta2=beta2, eps=eps, weight_decay=weight_decay,
                  gamma=gamma, lookahead=int(bool(lookahead)), correction=correction,
                  fwd_dtype=fwd_dtype, grad_dtype=grad_dtype, momentum_decay=momentum_decay,
                  subset_granule=subset_granule, msg_dtype=msg_dtype, subset_kind=subset_kind, d_layout=d_layout,
                  ring_cap_lines=ring_cap_lines)


def workspace_bytes(cfg: Config) -> int:
    out = C.c_uint64(0)
    _check(lib.am_workspace_bytes(C.byref(cfg), C.byref(out)))
    return int(out.value)


def d_layout_info(cfg: Config):
    """(replicas per block, number of arrays, floats per array) of the EMA vectors (am_d_layout_info)."""
    rb, arrays, floats = C.c_uint32(0), C.c_uint32(0), C.c_uint64(0)
    _check(lib.am_d_layout_info(C.byref(cfg), C.byref(rb), C.byref(arrays), C.byref(floats)))
    return int(rb.value), int(arrays.value), int(floats.value)


def _check_tensors(name, tensors, count, numel, dtype, device):
    if len(tensors) != count:
        raise ValueError(f"{name}: {len(tensors)} tensors, {count} expected")
    for i, x in enumerate(tensors):
        if not (x.is_cuda and x.device == device and x.is_contiguous() and x.numel() == numel and x.dtype == dtype):
            raise ValueError(f"{name}[{i}] must be a contiguous {dtype} tensor of {numel} elements on {device}")


def _ptr_table(tensors):
    return (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def _stream_handle(device) -> int:
    return int(torch.cuda.current_stream(device).cuda_stream)


class Stage:
    """State of one pipeline stage replicated R times on one GPU (am_state plus the device
    tensors it is bound to).  Methods carry the names of the C entry points."""

    def __init__(self, cfg: Config, w0: torch.Tensor | None = None, device="cuda:0", with_fwd: bool | None = None):
        self.cfg = cfg
        self.device = torch.device(device)
        n, R = int(cfg.n), int(cfg.replicas)
        self.n, self.R = n, R
        f32 = dict(dtype=torch.float32, device=self.device)
        need_m = not (cfg.optimizer == OPT_SGD and cfg.beta1 == 0.0)
        need_v = cfg.optimizer != OPT_SGD
        need_d = cfg.correction != CORR_NONE
        need_fwd = bool(cfg.lookahead) or cfg.fwd_dtype == BF16
        if with_fwd is None:
            with_fwd = need_fwd
        self.w = [torch.empty(n, **f32) for _ in range(R)]
        self.m = [torch.empty(n, **f32) for _ in range(R)] if need_m else None
        self.v = [torch.empty(n, **f32) for _ in range(R)] if need_v else None
        self._alloc_d(need_d, f32)
        fdt = torch.bfloat16 if cfg.fwd_dtype == BF16 else torch.float32
        self.fwd = [torch.empty(n, dtype=fdt, device=self.device) for _ in range(R)] if with_fwd else None
        if w0 is not None:
            self.set_w(w0)
        self.workspace = torch.empty(workspace_bytes(cfg), dtype=torch.uint8, device=self.device)
        self._handle = C.c_void_p(None)
        self._init()

    def _alloc_d(self, need_d: bool, f32):
        """d_storage: the arrays handed to the library (one per replica, or one per block of
        replicas in the interleaved layout); d: one view per replica, for reading."""
        if not need_d:
            self.d_storage = self.d = None
            return
        rb, arrays, floats = d_layout_info(self.cfg)
        self.d_storage = [torch.empty(floats, **f32) for _ in range(arrays)]
        self._d_views(rb)

    def _d_views(self, rb: int):
        if self.cfg.d_layout == D_INTERLEAVED:
            self.d = [self.d_storage[i // rb].view(-1, rb)[:self.n, i % rb] for i in range(self.R)]
        else:
            self.d = self.d_storage

    @classmethod
    def resume(cls, cfg: Config, snapshot: Snapshot, w, m, v, d, fwd, workspace, device="cuda:0"):
        """A stage bound to arrays whose bytes were restored from a checkpoint (am_resume_state);
        nothing is cleared.  m, v, d, fwd are lists of tensors or None, as the config needs (d: what
        d_storage held: one array per replica, or per block in the interleaved layout)."""
        self = cls.__new__(cls)
        self.cfg, self.device = cfg, torch.device(device)
        self.n, self.R = int(cfg.n), int(cfg.replicas)
        self.w, self.m, self.v, self.fwd, self.workspace = w, m, v, fwd, workspace
        self.d_storage = d
        if d is None:
            self.d = None
        else:
            rb, arrays, floats = d_layout_info(cfg)
            _check_tensors("d", d, arrays, floats, torch.float32, self.device)
            self._d_views(rb)
        fdt = torch.bfloat16 if cfg.fwd_dtype == BF16 else torch.float32
        for name, ts, dt in (("w", w, torch.float32), ("m", m, torch.float32), ("v", v, torch.float32), ("fwd", fwd, fdt)):
            if ts is not None:
                _check_tensors(name, ts, self.R, self.n, dt, self.device)
        if not (workspace.is_cuda and workspace.is_contiguous() and workspace.dtype == torch.uint8
                and workspace.numel() >= workspace_bytes(cfg)):
            raise ValueError("workspace must be a contiguous uint8 device tensor of at least workspace_bytes(cfg) bytes")
        self._handle = C.c_void_p(None)
        self._init(snapshot)
        return self

    def export_state(self) -> Snapshot:
        """The library's own record for a checkpoint (am_export_state).  The caller lets the stream
        drain and saves w, m, v, d, (fwd) and the workspace alongside it."""
        snap = Snapshot()
        _check(lib.am_export_state(self._handle, C.byref(snap)))
        return snap

    def _init(self, snapshot: Snapshot | None = None):
        bufs = Buffers()
        self._tables = {}
        for name in ("w", "m", "v", "d", "fwd"):
            ts = self.d_storage if name == "d" else getattr(self, name)
            if ts is not None:
                self._tables[name] = _ptr_table(ts)
                setattr(bufs, name, C.cast(self._tables[name], C.POINTER(C.c_void_p)))
        bufs.workspace = self.workspace.data_ptr()
        bufs.workspace_bytes = self.workspace.numel()
        with torch.cuda.device(self.device):
            if snapshot is None:
                _check(lib.am_init_state(C.byref(self.cfg), C.byref(bufs), _stream_handle(self.device), C.byref(self._handle)))
            else:
                _check(lib.am_resume_state(C.byref(self.cfg), C.byref(bufs), _stream_handle(self.device),
                                           C.byref(snapshot), C.byref(self._handle)))

    def set_w(self, w0: torch.Tensor):
        """Copy the starting weights in: one row for all replicas (1-D) or one row per replica (2-D)."""
        w0 = torch.as_tensor(w0)
        for i in range(self.R):
            self.w[i].copy_(w0 if w0.dim() == 1 else w0[i])

    def _check_grads(self, grads, allow_none: bool = False):
        """The C side sees raw pointers only: everything that could make a kernel read past an
        allocation is refused here, before any launch."""
        if len(grads) != self.R:
            raise ValueError(f"{len(grads)} gradient tensors for {self.R} replicas")
        want = torch.bfloat16 if self.cfg.grad_dtype == BF16 else torch.float32
        for i, g in enumerate(grads):
            if g is None:
                if allow_none:
                    continue
                raise ValueError(f"grads[{i}] is None")
            if not (g.is_cuda and g.device == self.device and g.is_contiguous() and g.numel() == self.n and g.dtype == want):
                raise ValueError(f"grads[{i}] must be a contiguous {want} tensor of {self.n} elements on {self.device}, "
                                 f"got {tuple(g.shape)} {g.dtype} on {g.device}, contiguous={g.is_contiguous()}")

    # ---- entry points -------------------------------------------------------------------
    def step(self, t: int, grads, lr: float, lambda_t: float = 0.5, grad_scale: float = 1.0):
        self._check_grads(grads)
        table = _ptr_table(grads)
        with torch.cuda.device(self.device):
            _check(lib.am_step(self._handle, t, table, lr, lambda_t, grad_scale))

    def step_scaled(self, t: int, grads, lr: float, lambda_t: float, grad_scale: float, replica_scale: torch.Tensor):
        """am_step_scaled: replica_scale is a device tensor of R fp32 factors."""
        self._check_grads(grads)
        assert replica_scale.is_cuda and replica_scale.dtype == torch.float32
        assert replica_scale.numel() == self.R and replica_scale.is_contiguous()
        table = _ptr_table(grads)
        with torch.cuda.device(self.device):
            _check(lib.am_step_scaled(self._handle, t, table, lr, lambda_t, grad_scale, replica_scale.data_ptr()))

    def step_masked(self, t: int, grads, lr: float, lambda_t: float, active_mask: int, grad_scale: float = 1.0,
                    replica_scale: torch.Tensor | None = None):
        """One tick in which only the replicas named by active_mask make a local step (am_step_masked);
        grads[i] of an idle replica may be None."""
        self._check_grads([g if (active_mask >> i) & 1 else None for i, g in enumerate(grads)], allow_none=True)
        table = (C.c_void_p * self.R)(*[None if g is None else g.data_ptr() for g in grads])
        with torch.cuda.device(self.device):
            _check(lib.am_step_masked(self._handle, t, table, lr, lambda_t, grad_scale,
                                      None if replica_scale is None else replica_scale.data_ptr(), active_mask))

    def grad_sqnorm(self, grads) -> torch.Tensor:
        """am_grad_sqnorm: device tensor of R doubles, sum of squares of each replica's gradient."""
        self._check_grads(grads)
        out = torch.empty(self.R, dtype=torch.float64, device=self.device)
        table = _ptr_table(grads)
        with torch.cuda.device(self.device):
            _check(lib.am_grad_sqnorm(self._handle, table, out.data_ptr()))
        return out

    def sparse_average(self, t: int, lambda_t: float = 0.5):
        with torch.cuda.device(self.device):
            _check(lib.am_sparse_average(self._handle, t, lambda_t))

    def subset_indices(self, t: int, capacity: int | None = None) -> torch.Tensor:
        cap = self.n if capacity is None else capacity
        out = torch.empty(max(cap, 1), dtype=torch.int64, device=self.device)
        count = torch.zeros(1, dtype=torch.int64, device=self.device)
        with torch.cuda.device(self.device):
            _check(lib.am_subset_indices(self._handle, t, out.data_ptr(), cap, count.data_ptr()))
        k = int(count.item())
        return out[:min(k, cap)], k

    def subset_indices_static(self, t: int, out: torch.Tensor, count: torch.Tensor):
        """am_subset_indices_static: the variant that allocates nothing.  out (int64, its length is
        the capacity) and count (int64, one element) are the caller's device tensors; nothing is
        read back."""
        assert out.is_cuda and out.dtype == torch.int64 and out.is_contiguous()
        assert count.is_cuda and count.dtype == torch.int64 and count.numel() == 1
        with torch.cuda.device(self.device):
            _check(lib.am_subset_indices_static(self._handle, t, out.data_ptr(), out.numel(), count.data_ptr()))

    def set_delay(self, tau: int):
        _check(lib.am_set_delay(self._handle, tau))

    def diagnostics(self):
        """(consensus error, mean EMA variance, max EMA variance) as Python floats (synchronises)."""
        out = torch.zeros(3, dtype=torch.float64, device=self.device)
        with torch.cuda.device(self.device):
            _check(lib.am_diagnostics(self._handle, out.data_ptr()))
        return tuple(float(x) for x in out.cpu())

    def read_flags(self) -> int:
        f = C.c_uint32(0)
        _check(lib.am_read_flags(self._handle, C.byref(f)))
        return int(f.value)

    def set_profiling(self, on: bool):
        _check(lib.am_set_profiling(self._handle, int(on)))

    def get_profile(self):
        ms, k = C.c_double(0), C.c_uint64(0)
        _check(lib.am_get_profile(self._handle, C.byref(ms), C.byref(k)))
        return float(ms.value), int(k.value)

    def get_profile_times(self):
        """Per-launch times (ms) of the fused kernel since profiling was switched on (am_get_profile_times)."""
        buf = (C.c_float * 4096)()
        k = C.c_uint64(0)
        _check(lib.am_get_profile_times(self._handle, buf, 4096, C.byref(k)))
        return [float(buf[i]) for i in range(min(int(k.value), 4096))]

    def ring_info(self):
        cap, slots = C.c_uint64(0), C.c_uint32(0)
        _check(lib.am_ring_info(self._handle, C.byref(cap), C.byref(slots)))
        return int(cap.value), int(slots.value)

    def close(self):
        if self._handle:
            lib.am_destroy(self._handle)
            self._handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def init_state(cfg: Config, w0=None, device="cuda:0", with_fwd=None) -> Stage:
    return Stage(cfg, w0=w0, device=device, with_fwd=with_fwd)


def lookahead(w: torch.Tensor, w_prev: torch.Tensor, gamma: float, out_dtype=F32) -> torch.Tensor:
    """Stateless out = w + gamma (w - w_prev) (am_lookahead)."""
    assert w.is_cuda and w_prev.is_cuda and w.dtype == torch.float32 and w_prev.dtype == torch.float32
    assert w.is_contiguous() and w_prev.is_contiguous() and w.numel() == w_prev.numel()
    out = torch.empty(w.numel(), dtype=torch.bfloat16 if out_dtype == BF16 else torch.float32, device=w.device)
    with torch.cuda.device(w.device):
        _check(lib.am_lookahead(out.data_ptr(), out_dtype, w.data_ptr(), w_prev.data_ptr(), w.numel(), gamma,
                                _stream_handle(w.device)))
    return out
