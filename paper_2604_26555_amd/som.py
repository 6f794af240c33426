"""Thin ctypes binding of libsom's C ABI: argument marshalling only, every step runs in the HIP kernels.

The functions keep the C names (som_bmu, som_accumulate, som_neighborhood_update, som_epoch, som_epoch_host)
and take torch tensors that live on the GPU; torch is used for device memory and streams, nothing else.
There is no CPU fallback: if the shared library is missing or no gfx950 device is present, loading or
``Som()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SOM_LIB") or os.path.join(_HERE, "libsom.so")   # SOM_LIB: another build of the library

SOM_OK, SOM_EINVAL, SOM_ENOMEM, SOM_EHIP, SOM_EIO, SOM_ESTATE = 0, -1, -2, -3, -4, -5
SOM_KERNEL_GAUSSIAN = 0
SOM_SAFEGUARD_THRESHOLD = 0
SOM_SAFEGUARD_SHIFT = 1
SOM_SEARCH_AUTO = 0
SOM_SEARCH_FLOAT32 = 1
SOM_TOPOLOGY_MST = 1
SOM_TOPOLOGY_RNG = 2

EXPORTS = [
    "som_create", "som_destroy", "som_strerror", "som_last_error", "som_sync", "som_bmu", "som_accumulate",
    "som_neighborhood_update", "som_epoch", "som_epoch_host", "som_profile", "som_profile_read",
    "som_set_update_rule", "som_topology", "som_set_safeguard", "som_set_reproducible", "som_set_search",
    "som_matrix_pipe_probe", "som_neighborhood_update_static", "som_epoch_file", "som_read_probe", "som_mfma_rate_probe",
]


class SomStats(C.Structure):
    _fields_ = [
        ("sum_dist", C.c_double), ("sum_dist2", C.c_double), ("m", C.c_int64), ("n_recheck", C.c_int64),
        ("n_empty", C.c_int32), ("n_guarded", C.c_int32), ("ms_bmu_acc", C.c_float), ("ms_update", C.c_float),
        ("ms_h2d", C.c_float),
    ]


class SomError(RuntimeError):
    def __init__(self, code: int, what: str, detail: str):
        super().__init__(f"{what} failed: {detail} (code {code})")
        self.code = code


_lib = None


def load_library(path: str = LIB_PATH) -> C.CDLL:
    """Load libsom.so and declare the prototypes.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2604_26555_amd.build`")
    lib = C.CDLL(path)
    vp, i32, i64, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_double
    lib.som_create.argtypes = [C.POINTER(vp), C.c_int, vp]
    lib.som_create.restype = C.c_int
    lib.som_destroy.argtypes = [vp]
    lib.som_destroy.restype = None
    lib.som_strerror.argtypes = [C.c_int]
    lib.som_strerror.restype = C.c_char_p
    lib.som_last_error.argtypes = [vp]
    lib.som_last_error.restype = C.c_char_p
    lib.som_sync.argtypes = [vp]
    lib.som_sync.restype = C.c_int
    lib.som_set_update_rule.argtypes = [vp, f64, f64, vp]
    lib.som_set_update_rule.restype = C.c_int
    lib.som_profile.argtypes = [vp, C.c_int]
    lib.som_profile.restype = C.c_int
    lib.som_profile_read.argtypes = [vp, C.POINTER(C.c_float), i32, C.POINTER(i32)]
    lib.som_profile_read.restype = C.c_int
    lib.som_bmu.argtypes = [vp, vp, i64, i32, i64, vp, i64, vp, i32, vp, vp, vp]
    lib.som_bmu.restype = C.c_int
    lib.som_accumulate.argtypes = [vp, vp, i64, i32, i64, vp, i64, vp, i32, vp, vp, C.c_int]
    lib.som_accumulate.restype = C.c_int
    lib.som_neighborhood_update.argtypes = [vp, vp, vp, vp, i32, i32, f64, C.c_int, f64, vp, vp]
    lib.som_neighborhood_update.restype = C.c_int
    lib.som_neighborhood_update_static.argtypes = [vp, vp, vp, vp, i32, i32, f64, C.c_int, f64, vp, vp]
    lib.som_neighborhood_update_static.restype = C.c_int
    lib.som_set_reproducible.argtypes = [vp, C.c_int]
    lib.som_set_reproducible.restype = C.c_int
    lib.som_set_search.argtypes = [vp, C.c_int]
    lib.som_set_search.restype = C.c_int
    lib.som_set_safeguard.argtypes = [vp, C.c_int]
    lib.som_set_safeguard.restype = C.c_int
    lib.som_topology.argtypes = [vp, vp, i32, i32, C.c_int, vp]
    lib.som_topology.restype = C.c_int
    lib.som_matrix_pipe_probe.argtypes = [vp, vp, vp, vp, vp, i64]
    lib.som_matrix_pipe_probe.restype = C.c_int
    lib.som_epoch.argtypes = [vp, vp, i64, i32, i64, vp, i64, vp, i32, vp, f64, C.c_int, f64, C.POINTER(SomStats)]
    lib.som_epoch.restype = C.c_int
    lib.som_epoch_host.argtypes = [vp, vp, i64, i32, i64, C.c_int, vp, i32, vp, f64, C.c_int, f64,
                                   C.POINTER(SomStats)]
    lib.som_epoch_host.restype = C.c_int
    lib.som_mfma_rate_probe.argtypes = [vp, C.c_int, C.c_int, C.c_int]
    lib.som_mfma_rate_probe.restype = C.c_int
    lib.som_read_probe.argtypes = [vp, vp, i64]
    lib.som_read_probe.restype = C.c_int
    lib.som_epoch_file.argtypes = [vp, C.c_int, i64, i64, i32, i64, vp, i32, vp, f64, C.c_int, f64, C.POINTER(SomStats)]
    lib.som_epoch_file.restype = C.c_int
    _lib = lib
    return lib


# same-width signed types are accepted for the unsigned arguments (row numbers below 2^31, counts below 2^63)
_ALIASES = {torch.uint32: (torch.uint32, torch.int32), torch.uint64: (torch.uint64, torch.int64)}


def _ptr(t: Optional[torch.Tensor], dtype: torch.dtype, name: str, device=None) -> Optional[int]:
    if t is None:
        return None
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name} must be a torch tensor")
    if t.dtype not in _ALIASES.get(dtype, (dtype,)):
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if t.dim() and not t.is_contiguous() and t.dim() == 1:
        raise ValueError(f"{name} must be contiguous")
    if device is not None and t.device != device:
        raise ValueError(f"{name} lives on {t.device}, the context is on {device}")
    return t.data_ptr()


def _matrix(t: torch.Tensor, name: str):
    if t.dim() != 2 or t.stride(1) != 1 or (t.shape[0] > 1 and t.stride(0) < t.shape[1]):
        raise ValueError(f"{name} must be a row-major 2-D tensor")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0))
    return t.shape[0], t.shape[1], ld


@dataclass
class EpochStats:
    sum_dist: float
    sum_dist2: float
    m: int
    n_recheck: int
    n_empty: int
    n_guarded: int
    ms_bmu_acc: float
    ms_update: float
    ms_h2d: float

    @property
    def qe(self) -> float:
        return self.sum_dist / self.m if self.m else 0.0


def _stats(s: SomStats) -> EpochStats:
    return EpochStats(s.sum_dist, s.sum_dist2, s.m, s.n_recheck, s.n_empty, s.n_guarded, s.ms_bmu_acc, s.ms_update,
                      s.ms_h2d)


class Som:
    """One libsom context bound to a GPU and to the torch stream that is current when it is created."""

    def __init__(self, device: int | str | torch.device = 0, stream: Optional[torch.cuda.Stream] = None):
        self.lib = load_library()
        dev = torch.device("cuda", device) if isinstance(device, int) else torch.device(device)
        if dev.type != "cuda":
            raise ValueError("libsom runs on a GPU only")
        self.device = torch.device("cuda", dev.index or 0)
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: libsom has no CPU path")
        with torch.cuda.device(self.device):
            self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        handle = C.c_void_p()
        rc = self.lib.som_create(C.byref(handle), self.device.index, C.c_void_p(self.stream.cuda_stream))
        if rc != SOM_OK:
            raise SomError(rc, "som_create", self.lib.som_strerror(rc).decode())
        self._h = handle

    def close(self):
        if getattr(self, "_h", None):
            self.lib.som_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def _check(self, rc: int, what: str):
        if rc != SOM_OK:
            detail = self.lib.som_last_error(self._h).decode() or self.lib.som_strerror(rc).decode()
            raise SomError(rc, what, detail)

    def som_sync(self):
        self._check(self.lib.som_sync(self._h), "som_sync")

    def som_set_update_rule(self, eta: float = 1.0, mu: float = 0.0, velocity=None):
        """Learning rate and momentum of every later update on this context; velocity is a K x D float32 GPU tensor."""
        if velocity is not None and not velocity.is_contiguous():
            raise ValueError("velocity must be contiguous")
        self._velocity = velocity                       # keep the caller's buffer alive while the library uses it
        self._check(self.lib.som_set_update_rule(self._h, float(eta), float(mu),
                                                 _ptr(velocity, torch.float32, "velocity", self.device)),
                    "som_set_update_rule")

    def som_profile(self, enable: bool):
        self._check(self.lib.som_profile(self._h, 1 if enable else 0), "som_profile")

    def som_profile_read(self, capacity: int = 4096):
        """Durations (ms) of the main BMU kernel launches recorded since the last read."""
        buf = (C.c_float * capacity)()
        count = C.c_int32(0)
        self._check(self.lib.som_profile_read(self._h, buf, capacity, C.byref(count)), "som_profile_read")
        return [buf[i] for i in range(min(capacity, count.value))]

    def som_mfma_rate_probe(self, fold_steps=0, waves_per_simd=2, iters=20000):
        """Enqueue a loop of 8 * iters bf16 MFMAs per wavefront on random operands (time it from outside)."""
        self._check(self.lib.som_mfma_rate_probe(self._h, int(fold_steps), int(waves_per_simd), int(iters)), "som_mfma_rate_probe")

    def som_read_probe(self, t):
        """One plain streaming read of tensor t's bytes on the context's stream (time it from outside)."""
        nbytes = t.numel() * t.element_size() // 16 * 16
        self._check(self.lib.som_read_probe(self._h, C.c_void_p(t.data_ptr()), nbytes), "som_read_probe")

    def som_matrix_pipe_probe(self, A, Bt, Cm, Dout=None):
        """One bf16 MFMA per problem: Dout = Cm + A @ Bt^T.  A, Bt: (n, 32, 16) bf16; Cm: (n, 32, 32) float32."""
        n = A.shape[0]
        if A.shape != (n, 32, 16) or Bt.shape != (n, 32, 16) or Cm.shape != (n, 32, 32) or not (
                A.is_contiguous() and Bt.is_contiguous() and Cm.is_contiguous()):
            raise ValueError("shapes: A, Bt (n, 32, 16) bf16, C (n, 32, 32) float32, all contiguous")
        if Dout is None:
            Dout = torch.empty_like(Cm)
        rc = self.lib.som_matrix_pipe_probe(self._h, _ptr(A, torch.bfloat16, "A", self.device),
                                            _ptr(Bt, torch.bfloat16, "Bt", self.device),
                                            _ptr(Cm, torch.float32, "C", self.device),
                                            _ptr(Dout, torch.float32, "Dout", self.device), n)
        self._check(rc, "som_matrix_pipe_probe")
        return Dout

    # ------------------------------------------------------------------ stage 1
    def som_bmu(self, X, W, idx=None, bmu=None, d2=None, qe=None):
        """bmu[i] = best-matching unit of presented sample i; returns (bmu, d2, qe) tensors (those requested)."""
        N, D, ldx = _matrix(X, "X")
        K, Dw, _ = _matrix(W, "W")
        if Dw != D or not W.is_contiguous():
            raise ValueError("W must be a contiguous K x D tensor with X's D")
        m = N if idx is None else idx.numel()
        if bmu is None:
            bmu = torch.empty(m, dtype=torch.int32, device=self.device)
        rc = self.lib.som_bmu(self._h, _ptr(X, torch.float32, "X", self.device), N, D, ldx,
                              _ptr(idx, torch.uint32, "idx", self.device) if idx is not None else None, m,
                              _ptr(W, torch.float32, "W", self.device), K,
                              _ptr(bmu, torch.int32, "bmu", self.device), _ptr(d2, torch.float32, "d2", self.device),
                              _ptr(qe, torch.float64, "qe", self.device))
        self._check(rc, "som_bmu")
        return bmu, d2, qe

    # ------------------------------------------------------------------ stage 2
    def som_accumulate(self, X, bmu, K, S, n, idx=None, zero_first=True):
        N, D, ldx = _matrix(X, "X")
        m = N if idx is None else idx.numel()
        if bmu.numel() != m:
            raise ValueError("bmu must have one entry per presented sample")
        if S.shape != (K, D) or not S.is_contiguous() or n.numel() != K:
            raise ValueError("S must be K x D contiguous and n of length K")
        rc = self.lib.som_accumulate(self._h, _ptr(X, torch.float32, "X", self.device), N, D, ldx,
                                     _ptr(idx, torch.uint32, "idx", self.device) if idx is not None else None, m,
                                     _ptr(bmu, torch.int32, "bmu", self.device), K,
                                     _ptr(S, torch.float64, "S", self.device), _ptr(n, torch.uint64, "n", self.device),
                                     1 if zero_first else 0)
        self._check(rc, "som_accumulate")
        return S, n

    # ------------------------------------------------------------------ stage 3
    def som_neighborhood_update(self, S, n, G, sigma, W, eps_h=0.0, n_guarded=None, kernel=SOM_KERNEL_GAUSSIAN):
        K, D, _ = _matrix(W, "W")
        if not W.is_contiguous() or S.shape != (K, D) or not S.is_contiguous() or G.shape != (K, K) \
                or not G.is_contiguous() or n.numel() != K:
            raise ValueError("shapes: W K x D, S K x D, G K x K, n K (all contiguous)")
        rc = self.lib.som_neighborhood_update(self._h, _ptr(S, torch.float64, "S", self.device),
                                              _ptr(n, torch.uint64, "n", self.device),
                                              _ptr(G, torch.float32, "G", self.device), K, D, float(sigma), kernel,
                                              float(eps_h), _ptr(W, torch.float32, "W", self.device),
                                              _ptr(n_guarded, torch.int32, "n_guarded", self.device))
        self._check(rc, "som_neighborhood_update")
        return W

    def som_neighborhood_update_static(self, S, n, G, sigma, W, eps_h=0.0, n_guarded=None, kernel=SOM_KERNEL_GAUSSIAN):
        """som_neighborhood_update without any device allocation (fixed per-GPU workspace; K * (D + 1) <= 65536)."""
        K, D, _ = _matrix(W, "W")
        if not W.is_contiguous() or S.shape != (K, D) or not S.is_contiguous() or G.shape != (K, K) \
                or not G.is_contiguous() or n.numel() != K:
            raise ValueError("shapes: W K x D, S K x D, G K x K, n K (all contiguous)")
        rc = self.lib.som_neighborhood_update_static(self._h, _ptr(S, torch.float64, "S", self.device),
                                                     _ptr(n, torch.uint64, "n", self.device),
                                                     _ptr(G, torch.float32, "G", self.device), K, D, float(sigma), kernel,
                                                     float(eps_h), _ptr(W, torch.float32, "W", self.device),
                                                     _ptr(n_guarded, torch.int32, "n_guarded", self.device))
        self._check(rc, "som_neighborhood_update_static")
        return W

    def som_set_reproducible(self, on=True):
        self._check(self.lib.som_set_reproducible(self._h, 1 if on else 0), "som_set_reproducible")

    def som_set_search(self, mode):
        if isinstance(mode, str):
            mode = {"auto": SOM_SEARCH_AUTO, "float32": SOM_SEARCH_FLOAT32}[mode]
        self._check(self.lib.som_set_search(self._h, int(mode)), "som_set_search")

    def som_set_safeguard(self, mode):
        if isinstance(mode, str):
            mode = {"threshold": SOM_SAFEGUARD_THRESHOLD, "shift": SOM_SAFEGUARD_SHIFT}[mode]
        self._check(self.lib.som_set_safeguard(self._h, int(mode)), "som_set_safeguard")

    # ------------------------------------------------------------------ topology rebuild
    def som_topology(self, W, kind, G=None):
        K, D, _ = _matrix(W, "W")
        if not W.is_contiguous():
            raise ValueError("W must be contiguous")
        if isinstance(kind, str):
            kind = {"mst": SOM_TOPOLOGY_MST, "rng": SOM_TOPOLOGY_RNG}[kind]
        if G is None:
            G = torch.empty((K, K), dtype=torch.float32, device=W.device)
        elif G.shape != (K, K) or not G.is_contiguous():
            raise ValueError("G must be K x K contiguous")
        rc = self.lib.som_topology(self._h, _ptr(W, torch.float32, "W", self.device), K, D, int(kind),
                                   _ptr(G, torch.float32, "G", self.device))
        self._check(rc, "som_topology")
        return G

    # ------------------------------------------------------------------ whole epoch
    def som_epoch(self, X, W, G, sigma, idx=None, eps_h=0.0, want_stats=True, kernel=SOM_KERNEL_GAUSSIAN):
        N, D, ldx = _matrix(X, "X")
        K, Dw, _ = _matrix(W, "W")
        if Dw != D or not W.is_contiguous() or G.shape != (K, K) or not G.is_contiguous():
            raise ValueError("shapes: W K x D contiguous with X's D, G K x K contiguous")
        m = N if idx is None else idx.numel()
        st = SomStats()
        rc = self.lib.som_epoch(self._h, _ptr(X, torch.float32, "X", self.device), N, D, ldx,
                                _ptr(idx, torch.uint32, "idx", self.device) if idx is not None else None, m,
                                _ptr(W, torch.float32, "W", self.device), K, _ptr(G, torch.float32, "G", self.device),
                                float(sigma), kernel, float(eps_h), C.byref(st) if want_stats else None)
        self._check(rc, "som_epoch")
        return _stats(st) if want_stats else None

    def som_epoch_host(self, Xhost, W, G, sigma, chunk_rows, eps_h=0.0, pinned=None, kernel=SOM_KERNEL_GAUSSIAN):
        """Xhost: CPU float32 tensor or numpy array (C order, N x D), e.g. backed by a memory-mapped file."""
        import numpy as np
        if isinstance(Xhost, torch.Tensor):
            if Xhost.device.type != "cpu" or Xhost.dtype != torch.float32 or not Xhost.is_contiguous() or Xhost.dim() != 2:
                raise ValueError("Xhost must be a contiguous CPU float32 matrix")
            N, D = Xhost.shape
            addr = Xhost.data_ptr()
            if pinned is None:
                pinned = Xhost.is_pinned()
        else:
            a = Xhost
            if not isinstance(a, np.ndarray) or a.dtype != np.float32 or a.ndim != 2 or not a.flags["C_CONTIGUOUS"]:
                raise ValueError("Xhost must be a C-contiguous float32 numpy matrix")
            N, D = a.shape
            addr = a.ctypes.data
            pinned = bool(pinned)
        K, Dw, _ = _matrix(W, "W")
        if Dw != D or not W.is_contiguous() or G.shape != (K, K) or not G.is_contiguous():
            raise ValueError("shapes: W K x D contiguous with X's D, G K x K contiguous")
        st = SomStats()
        rc = self.lib.som_epoch_host(self._h, C.c_void_p(addr), N, D, int(chunk_rows), 1 if pinned else 0,
                                     _ptr(W, torch.float32, "W", self.device), K,
                                     _ptr(G, torch.float32, "G", self.device), float(sigma), kernel, float(eps_h),
                                     C.byref(st))
        self._check(rc, "som_epoch_host")
        return _stats(st)

    def som_epoch_file(self, fd, offset, N, D, W, G, sigma, chunk_rows, eps_h=0.0, kernel=SOM_KERNEL_GAUSSIAN):
        """One epoch on the N x D float32 rows stored from byte ``offset`` of the open file descriptor ``fd``."""
        K, Dw, _ = _matrix(W, "W")
        if Dw != D or not W.is_contiguous() or G.shape != (K, K) or not G.is_contiguous():
            raise ValueError("shapes: W K x D contiguous with the file's D, G K x K contiguous")
        st = SomStats()
        rc = self.lib.som_epoch_file(self._h, int(fd), int(offset), int(N), int(D), int(chunk_rows),
                                     _ptr(W, torch.float32, "W", self.device), K,
                                     _ptr(G, torch.float32, "G", self.device), float(sigma), kernel, float(eps_h),
                                     C.byref(st))
        self._check(rc, "som_epoch_file")
        return _stats(st)
