"""Thin ctypes binding of the C-ABI library (``include/regtopk.h``).

Argument marshalling only: every step of the round runs in the HIP kernels of
``libregtopk.so``.  PyTorch is used for device memory (the arena and the views
on the results) and for the current stream.  There is no CPU fallback: if the
library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libregtopk.so")

OK, INVALID_ARG, BAD_STATE, HIP_ERROR, NO_MEMORY = 0, -1, -2, -3, -4
OPT_FORCE_DENSE, OPT_CAND_TARGET, OPT_PROFILE, OPT_PRIOR_ROOTS, OPT_LIKELIHOOD, OPT_PRIOR_EXPONENT = 1, 2, 3, 4, 5, 6

# every symbol include/regtopk.h declares
SYMBOLS = [
    "regtopk_workspace_bytes", "regtopk_create", "regtopk_create_in", "regtopk_step", "regtopk_step_bf16", "regtopk_step_global",
    "regtopk_global_workspace_bytes", "regtopk_bind_global",
    "regtopk_destroy", "regtopk_reset", "regtopk_get_state", "regtopk_set_state",
    "regtopk_get_stats", "regtopk_set_option", "regtopk_get_timings", "regtopk_tanh_f32", "regtopk_erf_f32", "regtopk_pow_f32",
    "regtopk_copy_f32", "regtopk_set_weights", "regtopk_set_worker_k", "regtopk_mask_overlap", "regtopk_mask_overlap_static", "regtopk_sgd_update",
    "regtopk_last_error",
]


class Result(ctypes.Structure):
    _fields_ = [("idx", c_void_p), ("val", c_void_p), ("agg", c_void_p)]


class WorkerStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in (
        "tau_lo_bits", "n_candidates", "used_dense", "tau_bits", "n_greater",
        "n_ties_taken", "n_ties_total", "overflow", "used_window", "n_boundary", "n_valid",
        "window_half")]


class RegTopkError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("regtopk error %d: %s" % (code, msg))
        self.code = code


_lib = None


def load():
    """Loads libregtopk.so (built beforehand by ``build.build_library``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: run `python -m paper_2501_05633_amd.build` "
                           "(or __graft_entry__.build()) first" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    lib.regtopk_workspace_bytes.restype = c_size_t
    lib.regtopk_workspace_bytes.argtypes = [c_int32, c_int64, c_int64]
    lib.regtopk_create.argtypes = [ctypes.POINTER(c_void_p), c_int32, c_int64, c_int64, c_float]
    lib.regtopk_create_in.argtypes = [ctypes.POINTER(c_void_p), c_int32, c_int64, c_int64, c_float,
                                      c_void_p, c_size_t, c_void_p]
    lib.regtopk_step.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, ctypes.POINTER(Result)]
    lib.regtopk_step_bf16.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, ctypes.POINTER(Result)]
    lib.regtopk_step_global.argtypes = [c_void_p, c_void_p, c_void_p, ctypes.POINTER(Result)]
    lib.regtopk_global_workspace_bytes.restype = c_size_t
    lib.regtopk_global_workspace_bytes.argtypes = [c_int64, c_int64]
    lib.regtopk_bind_global.argtypes = [c_void_p, c_void_p, c_size_t, c_void_p]
    lib.regtopk_destroy.argtypes = [c_void_p]
    lib.regtopk_reset.argtypes = [c_void_p, c_void_p]
    lib.regtopk_get_state.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p,
                                      ctypes.POINTER(c_int64), c_void_p]
    lib.regtopk_set_state.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_void_p]
    lib.regtopk_get_stats.argtypes = [c_void_p, ctypes.POINTER(WorkerStats), c_void_p]
    lib.regtopk_set_option.argtypes = [c_void_p, c_int, c_double]
    lib.regtopk_get_timings.argtypes = [c_void_p, ctypes.POINTER(c_float), c_int32, ctypes.POINTER(c_int32)]
    lib.regtopk_copy_f32.argtypes = [c_void_p, c_void_p, c_int64, c_void_p]
    lib.regtopk_tanh_f32.argtypes = [c_void_p, c_void_p, c_int64, c_void_p]
    lib.regtopk_erf_f32.argtypes = [c_void_p, c_void_p, c_int64, c_void_p]
    lib.regtopk_pow_f32.argtypes = [c_void_p, c_float, c_void_p, c_int64, c_void_p]
    lib.regtopk_set_weights.argtypes = [c_void_p, ctypes.POINTER(c_float), c_void_p]
    lib.regtopk_set_worker_k.argtypes = [c_void_p, ctypes.POINTER(c_int64), c_void_p]
    lib.regtopk_mask_overlap.argtypes = [c_void_p, c_void_p, c_void_p]
    lib.regtopk_mask_overlap_static.argtypes = [c_void_p, c_void_p, c_void_p]
    lib.regtopk_sgd_update.argtypes = [c_void_p, c_void_p, c_float, c_int64, c_void_p]
    lib.regtopk_last_error.restype = c_char_p
    _lib = lib
    return lib


def _check(rc: int):
    if rc != OK:
        raise RegTopkError(rc, load().regtopk_last_error().decode())


def _stream_ptr(torch):
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def workspace_bytes(N: int, d: int, k: int) -> int:
    return int(load().regtopk_workspace_bytes(N, d, k))


def _view(torch, ptr: int, shape, dtype, device, arena=None):
    """Zero-copy torch view of device memory owned by the context."""
    n = 1
    for s in shape:
        n *= s
    itemsize = torch.empty(0, dtype=dtype).element_size()
    if arena is not None:                     # torch owns the arena: slice it
        off = ptr - arena.data_ptr()
        return arena[off:off + n * itemsize].view(dtype).view(*shape)

    class _Holder:
        pass

    h = _Holder()
    h.__cuda_array_interface__ = {
        "shape": tuple(shape), "typestr": {4: "<f4" if dtype.is_floating_point else "<i4"}[itemsize],
        "data": (ptr, False), "version": 2,
    }
    return torch.as_tensor(h, device=device)


class RegTopk:
    """regtopk_create / regtopk_step / regtopk_destroy with torch tensors.

    ``step(grads, prev_aggregate)`` takes CUDA tensors ([N,d] float32 or bfloat16, and [d] float32)
    and returns ``(idx [N,k] int32, val [N,k] float32, agg [d] float32)`` as
    views into the context's memory, valid until the next step.
    """

    def __init__(self, N: int, d: int, k: int, mu: float, device="cuda:0", own_arena: bool = False):
        import torch
        self._torch = torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the RegTop-k path runs only as HIP kernels")
        self.lib = load()
        self.N, self.d, self.k, self.mu = int(N), int(d), int(k), float(mu)
        self.device = torch.device(device)
        self._h = c_void_p()
        self._arena = None
        self._garena = None          # memory of the global Top-k round's selector (torch-owned arenas only)
        self._own_arena = own_arena
        with torch.cuda.device(self.device):
            if own_arena:
                _check(self.lib.regtopk_create(ctypes.byref(self._h), self.N, self.d, self.k, self.mu))
            else:
                nbytes = workspace_bytes(self.N, self.d, self.k)
                if nbytes == 0:
                    _check(self.lib.regtopk_create(ctypes.byref(self._h), self.N, self.d, self.k, self.mu))
                self._arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
                base = self._arena.data_ptr()
                aligned = (base + 255) // 256 * 256
                _check(self.lib.regtopk_create_in(ctypes.byref(self._h), self.N, self.d, self.k, self.mu,
                                                  c_void_p(aligned), nbytes, _stream_ptr(torch)))

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            self.lib.regtopk_destroy(self._h)
            self._h = c_void_p()
            self._arena = None
            self._garena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, grads, prev_aggregate=None):
        torch = self._torch
        if grads.device != self.device or grads.dtype not in (torch.float32, torch.bfloat16) \
                or not grads.is_contiguous() or tuple(grads.shape) != (self.N, self.d):
            raise ValueError("grads must be a contiguous float32 or bfloat16 [N,d] tensor on %s" % self.device)
        fn = self.lib.regtopk_step if grads.dtype == torch.float32 else self.lib.regtopk_step_bf16
        gp = c_void_p(0)
        if prev_aggregate is not None:
            if prev_aggregate.device != self.device or prev_aggregate.dtype != torch.float32 \
                    or not prev_aggregate.is_contiguous() or tuple(prev_aggregate.shape) != (self.d,):
                raise ValueError("prev_aggregate must be a contiguous float32 [d] tensor on %s" % self.device)
            gp = c_void_p(prev_aggregate.data_ptr())
        res = Result()
        with torch.cuda.device(self.device):
            _check(fn(self._h, c_void_p(grads.data_ptr()), gp, _stream_ptr(torch), ctypes.byref(res)))
        idx = _view(torch, res.idx, (self.N, self.k), torch.int32, self.device, self._arena)
        val = _view(torch, res.val, (self.N, self.k), torch.float32, self.device, self._arena)
        agg = _view(torch, res.agg, (self.d,), torch.float32, self.device, self._arena)
        return idx, val, agg

    def step_global(self, grads):
        """One round of the genie-aided global Top-k baseline; returns like ``step``."""
        torch = self._torch
        if grads.device != self.device or grads.dtype != torch.float32 or not grads.is_contiguous() \
                or tuple(grads.shape) != (self.N, self.d):
            raise ValueError("grads must be a contiguous float32 [N,d] tensor on %s" % self.device)
        res = Result()
        with torch.cuda.device(self.device):
            if self._arena is not None and self._garena is None:
                # the context lives in torch's memory, so the selector of the global round does too
                nbytes = int(self.lib.regtopk_global_workspace_bytes(self.d, self.k))
                self._garena = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
                aligned = (self._garena.data_ptr() + 255) // 256 * 256
                _check(self.lib.regtopk_bind_global(self._h, c_void_p(aligned), nbytes, _stream_ptr(torch)))
            _check(self.lib.regtopk_step_global(self._h, c_void_p(grads.data_ptr()), _stream_ptr(torch),
                                                ctypes.byref(res)))
        idx = _view(torch, res.idx, (self.N, self.k), torch.int32, self.device, self._arena)
        val = _view(torch, res.val, (self.N, self.k), torch.float32, self.device, self._arena)
        agg = _view(torch, res.agg, (self.d,), torch.float32, self.device, self._garena)
        return idx, val, agg

    def reset(self):
        with self._torch.cuda.device(self.device):
            _check(self.lib.regtopk_reset(self._h, _stream_ptr(self._torch)))

    def set_weights(self, weights):
        """Aggregation weights omega_n (sequence of N floats; default 1/N each)."""
        ws = [float(x) for x in weights]
        if len(ws) != self.N:
            raise ValueError("need N weights")
        arr = (c_float * self.N)(*ws)
        with self._torch.cuda.device(self.device):
            _check(self.lib.regtopk_set_weights(self._h, arr, _stream_ptr(self._torch)))

    def set_worker_k(self, kn):
        """Entries kept by each worker (N integers in [1, k]); unused list positions hold (-1, 0)."""
        ks = [int(x) for x in kn]
        if len(ks) != self.N:
            raise ValueError("need N values")
        arr = (c_int64 * self.N)(*ks)
        with self._torch.cuda.device(self.device):
            _check(self.lib.regtopk_set_worker_k(self._h, arr, _stream_ptr(self._torch)))

    def mask_overlap(self):
        """int64 [N+1] CUDA tensor: entry c = number of indices that exactly c workers selected last round."""
        torch = self._torch
        counts = torch.empty(self.N + 1, dtype=torch.int64, device=self.device)
        with torch.cuda.device(self.device):
            _check(self.lib.regtopk_mask_overlap(self._h, c_void_p(counts.data_ptr()), _stream_ptr(torch)))
        return counts

    def mask_overlap_static(self, counts):
        """``mask_overlap`` into the caller's int64 [N+1] CUDA tensor through the entry point that allocates nothing."""
        torch = self._torch
        if counts.dtype != torch.int64 or counts.numel() != self.N + 1 or counts.device != self.device \
                or not counts.is_contiguous():
            raise ValueError("counts must be a contiguous int64 [N+1] tensor on %s" % self.device)
        with torch.cuda.device(self.device):
            _check(self.lib.regtopk_mask_overlap_static(self._h, c_void_p(counts.data_ptr()), _stream_ptr(torch)))
        return counts

    def set_option(self, option: int, value: float):
        _check(self.lib.regtopk_set_option(self._h, option, float(value)))

    def get_state(self):
        """Returns (e [N,d], prev_idx [N,k] or None, prev_val [N,k] or None, t)."""
        torch = self._torch
        e = torch.empty(self.N, self.d, dtype=torch.float32, device=self.device)
        pidx = torch.full((self.N, self.k), -1, dtype=torch.int32, device=self.device)
        pval = torch.zeros(self.N, self.k, dtype=torch.float32, device=self.device)
        t = c_int64(0)
        with torch.cuda.device(self.device):
            _check(self.lib.regtopk_get_state(self._h, c_void_p(e.data_ptr()), c_void_p(pidx.data_ptr()),
                                              c_void_p(pval.data_ptr()), ctypes.byref(t), _stream_ptr(torch)))
        if t.value == 0:
            return e, None, None, 0
        return e, pidx, pval, int(t.value)

    def set_state(self, e, prev_idx=None, prev_val=None, t: int = 0):
        torch = self._torch
        if tuple(e.shape) != (self.N, self.d) or e.dtype != torch.float32 or not e.is_contiguous():
            raise ValueError("e must be contiguous float32 [N,d]")
        pi = pv = c_void_p(0)
        if t > 0:
            if prev_idx is None or prev_val is None:
                raise ValueError("previous lists are required when t > 0")
            if tuple(prev_idx.shape) != (self.N, self.k) or prev_idx.dtype != torch.int32 \
                    or tuple(prev_val.shape) != (self.N, self.k) or prev_val.dtype != torch.float32:
                raise ValueError("prev_idx/prev_val must be [N,k] int32/float32")
            pi, pv = c_void_p(prev_idx.contiguous().data_ptr()), c_void_p(prev_val.contiguous().data_ptr())
        with torch.cuda.device(self.device):
            _check(self.lib.regtopk_set_state(self._h, c_void_p(e.data_ptr()), pi, pv, int(t), _stream_ptr(torch)))
            torch.cuda.current_stream().synchronize()   # inputs may be temporaries of the caller

    def timings(self, max_rounds: int = 64):
        """Per-round stage times in ms: rows of (sweep, select, compact+aggregate, total)."""
        buf = (c_float * (4 * max_rounds))()
        n = c_int32(0)
        _check(self.lib.regtopk_get_timings(self._h, buf, max_rounds, ctypes.byref(n)))
        return [tuple(buf[4 * i + j] for j in range(4)) for i in range(n.value)]

    def stats(self):
        arr = (WorkerStats * self.N)()
        with self._torch.cuda.device(self.device):
            _check(self.lib.regtopk_get_stats(self._h, arr, _stream_ptr(self._torch)))
        return [{f: getattr(s, f) for f, _ in WorkerStats._fields_} for s in arr]


def copy_f32(dst, src):
    """Plain copy kernel of known size (reference dispatch for traffic counters)."""
    import torch
    with torch.cuda.device(src.device):
        _check(load().regtopk_copy_f32(c_void_p(dst.data_ptr()), c_void_p(src.data_ptr()), src.numel(),
                                       _stream_ptr(torch)))


def tanh_f32(x):
    """tanh step alone on a CUDA float32 tensor (test hook)."""
    import torch
    y = torch.empty_like(x)
    with torch.cuda.device(x.device):
        _check(load().regtopk_tanh_f32(c_void_p(x.data_ptr()), c_void_p(y.data_ptr()), x.numel(),
                                       _stream_ptr(torch)))
    return y


def pow_f32(x, y: float):
    """x**y correctly rounded, on a CUDA float32 tensor of non-negative values (test hook)."""
    import torch
    out = torch.empty_like(x)
    with torch.cuda.device(x.device):
        _check(load().regtopk_pow_f32(c_void_p(x.data_ptr()), float(y), c_void_p(out.data_ptr()), x.numel(),
                                      _stream_ptr(torch)))
    return out


def erf_f32(x):
    """erf step alone on a CUDA float32 tensor (test hook)."""
    import torch
    y = torch.empty_like(x)
    with torch.cuda.device(x.device):
        _check(load().regtopk_erf_f32(c_void_p(x.data_ptr()), c_void_p(y.data_ptr()), x.numel(),
                                      _stream_ptr(torch)))
    return y


def sgd_update(theta, g, eta: float):
    """theta <- theta - eta * g in place (CUDA float32 vectors of one length)."""
    import torch
    if theta.dtype != torch.float32 or g.dtype != torch.float32 or theta.shape != g.shape or theta.dim() != 1 \
            or not theta.is_contiguous() or not g.is_contiguous() or theta.device != g.device:
        raise ValueError("theta and g must be contiguous float32 vectors of one length on one device")
    with torch.cuda.device(theta.device):
        _check(load().regtopk_sgd_update(c_void_p(theta.data_ptr()), c_void_p(g.data_ptr()), float(eta),
                                         theta.numel(), _stream_ptr(torch)))
    return theta
