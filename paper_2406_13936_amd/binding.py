"""ctypes binding of the C ABI (include/abs.h): argument marshalling only.

Every step of the hot path runs in the HIP kernels of libabs.so; this module moves
pointers and sizes across the boundary and keeps the torch tensors that own the
device memory alive.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libabs.so")
_lib = None

STATS_NORM, STATS_IP = 1, 2
PREC_F32, PREC_BF16 = 0, 1

EXPORTS = [
    "abs_workspace_bytes", "abs_init_replicas", "abs_local_step", "abs_norm_test",
    "abs_inner_product_test", "abs_cross_worker_test", "abs_next_batch_size",
    "abs_average_replicas", "abs_get_params", "abs_set_params", "abs_get_grad",
    "abs_get_per_sample", "abs_n_params", "abs_layer_stats",
    "abs_layer_stats_workspace_bytes", "abs_average_bf16", "abs_destroy", "abs_last_error",
    "abs_profile_enable", "abs_profile_read", "abs_copy_probe", "abs_lr_schedule",
    "abs_lr_linear_scaling", "abs_norm_test_fpc", "abs_local_step_ragged", "abs_norm_test_per_worker",
    "abs_local_step_accumulated", "abs_profile_pause", "abs_local_step_graphed", "abs_graph_count",
    "abs_get_counters", "abs_get_opt_state", "abs_average_bf16_static",
    "abs_set_fused_update", "abs_set_gram_ip_max_batch",
]


class AbsError(RuntimeError):
    pass


class _Config(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("dims", C.POINTER(C.c_int)), ("act", C.c_int),
                ("has_bias", C.c_int), ("prec", C.c_int), ("M", C.c_int), ("b_cap", C.c_int),
                ("opt", C.c_int), ("momentum", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("eps", C.c_float), ("weight_decay", C.c_float),
                ("stats_mask", C.c_int), ("hip_stream", C.c_void_p), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t)]


class TestResult(C.Structure):
    __test__ = False            # not a pytest class
    _fields_ = [("b", C.c_int), ("sum_sq", C.c_double), ("gbar_sq", C.c_double),
                ("sum_q", C.c_double), ("sum_q2", C.c_double), ("loss_sum", C.c_double),
                ("var", C.c_double), ("var_perp", C.c_double), ("lhs", C.c_double),
                ("rhs", C.c_double), ("ratio", C.c_double), ("T", C.c_longlong),
                ("pass_", C.c_int)]


class ProfileEntry(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("calls", C.c_longlong), ("total_ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double)]


def load_library(reload: bool = False):
    """Load libabs.so (built by __graft_entry__.build()); raises if it is missing."""
    global _lib
    if _lib is not None and not reload:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise AbsError(f"{_LIB_PATH} is not built: run `python __graft_entry__.py` first "
                       "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    for name in EXPORTS:
        getattr(lib, name)          # fail loudly on a missing export
    for name in EXPORTS:
        getattr(lib, name).restype = C.c_int
    lib.abs_last_error.restype = C.c_char_p
    lib.abs_last_error.argtypes = [C.c_void_p]
    lib.abs_workspace_bytes.argtypes = [C.POINTER(_Config), C.c_int64, C.POINTER(C.c_size_t)]
    lib.abs_init_replicas.argtypes = [C.POINTER(_Config), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_int64, C.POINTER(C.c_void_p)]
    lib.abs_local_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_float]
    lib.abs_norm_test.argtypes = [C.c_void_p, C.c_double, C.POINTER(TestResult)]
    lib.abs_inner_product_test.argtypes = [C.c_void_p, C.c_double, C.c_double, C.POINTER(TestResult)]
    lib.abs_cross_worker_test.argtypes = [C.c_void_p, C.c_double, C.POINTER(TestResult)]
    lib.abs_next_batch_size.argtypes = [C.POINTER(TestResult), C.c_int, C.POINTER(C.c_int), C.c_int,
                                        C.c_int, C.POINTER(C.c_int)]
    lib.abs_average_replicas.argtypes = [C.c_void_p]
    lib.abs_get_params.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
    lib.abs_set_params.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
    lib.abs_get_grad.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
    lib.abs_get_counters.argtypes = [C.c_void_p, C.POINTER(C.c_longlong), C.POINTER(C.c_longlong),
                                     C.POINTER(C.c_longlong)]
    lib.abs_set_fused_update.argtypes = [C.c_void_p, C.c_int]
    lib.abs_set_gram_ip_max_batch.argtypes = [C.c_void_p, C.c_int]
    lib.abs_get_opt_state.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    lib.abs_get_per_sample.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
    lib.abs_n_params.argtypes = [C.POINTER(_Config), C.POINTER(C.c_int64)]
    lib.abs_layer_stats.argtypes = [C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int), C.c_int, C.c_int,
                                    C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p,
                                    C.c_size_t, C.c_void_p, C.POINTER(TestResult), C.c_void_p,
                                    C.c_void_p, C.c_void_p]
    lib.abs_layer_stats_workspace_bytes.argtypes = [C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int),
                                                    C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    lib.abs_average_bf16.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_void_p, C.c_void_p]
    lib.abs_average_bf16_static.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_void_p]
    lib.abs_destroy.argtypes = [C.c_void_p]
    lib.abs_lr_schedule.argtypes = [C.c_longlong, C.c_longlong, C.c_longlong, C.c_double, C.c_double,
                                    C.POINTER(C.c_double)]
    lib.abs_lr_linear_scaling.argtypes = [C.c_double, C.c_int64, C.c_int64, C.POINTER(C.c_double)]
    lib.abs_local_step_graphed.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_float]
    lib.abs_graph_count.argtypes = [C.c_void_p, C.POINTER(C.c_int)]
    lib.abs_local_step_accumulated.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float]
    lib.abs_local_step_ragged.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_int), C.c_float]
    lib.abs_norm_test_per_worker.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(TestResult)]
    lib.abs_norm_test_fpc.argtypes = [C.c_void_p, C.c_double, C.c_int64, C.POINTER(TestResult)]
    lib.abs_copy_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    lib.abs_profile_enable.argtypes = [C.c_void_p, C.c_int]
    lib.abs_profile_pause.argtypes = [C.c_void_p, C.c_int]
    lib.abs_profile_read.argtypes = [C.c_void_p, C.c_int, C.POINTER(ProfileEntry), C.POINTER(C.c_int)]
    _lib = lib
    return lib


def _check(st: int, ctx=None):
    if st != 0:
        msg = load_library().abs_last_error(ctx)
        raise AbsError(f"abs status {st}: {msg.decode() if msg else ''}")


def _stream_ptr():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def next_batch_size(results: Sequence[TestResult], b_cur: Sequence[int], b_cap: int,
                    sync_max: bool = True) -> List[int]:
    lib = load_library()
    M = len(results)
    arr = (TestResult * M)(*results)
    cur = (C.c_int * M)(*[int(v) for v in b_cur])
    nxt = (C.c_int * M)()
    _check(lib.abs_next_batch_size(arr, M, cur, int(b_cap), int(bool(sync_max)), nxt))
    return list(nxt)


class Replicas:
    """M replicas of one MLP on the current CUDA (HIP) device."""

    def __init__(self, dims, act, has_bias, prec, M, b_cap, opt, X, y, x0, momentum=0.0,
                 beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, stats_mask=STATS_NORM):
        import torch
        self._lib = load_library()
        self._torch = torch
        self.M, self.b_cap, self.dims = int(M), int(b_cap), tuple(int(d) for d in dims)
        self._dims_arr = (C.c_int * len(self.dims))(*self.dims)
        dev = torch.device("cuda")
        self._X = torch.as_tensor(np.ascontiguousarray(X, dtype=np.float32)).to(dev)
        self._y = torch.as_tensor(np.ascontiguousarray(y, dtype=np.int32)).to(dev)
        N = int(self._X.shape[0])
        cfg = _Config(len(self.dims) - 1, self._dims_arr, int(act), int(bool(has_bias)), int(prec),
                      self.M, self.b_cap, int(opt), momentum, beta1, beta2, eps, weight_decay,
                      int(stats_mask), _stream_ptr(), None, 0)
        nbytes = C.c_size_t(0)
        _check(self._lib.abs_workspace_bytes(C.byref(cfg), N, C.byref(nbytes)))
        # 4 KiB of canary bytes behind the workspace: guard_intact() tells whether a kernel wrote past its end
        self._guard = 4096
        self._ws = torch.empty(nbytes.value + 256 + self._guard, dtype=torch.uint8, device=dev)
        self._ws[-self._guard:].fill_(0xA5)
        base = (self._ws.data_ptr() + 255) // 256 * 256
        cfg.workspace, cfg.workspace_bytes = base, nbytes.value
        self.workspace_bytes = nbytes.value
        npar = C.c_int64(0)
        _check(self._lib.abs_n_params(C.byref(cfg), C.byref(npar)))
        self.n_params = int(npar.value)
        x0 = np.ascontiguousarray(x0, dtype=np.float32)
        assert x0.size == self.n_params, (x0.size, self.n_params)
        self._ctx = C.c_void_p(None)
        _check(self._lib.abs_init_replicas(C.byref(cfg), x0.ctypes.data, self._X.data_ptr(),
                                           self._y.data_ptr(), N, C.byref(self._ctx)))
        self._idx = torch.empty((self.M, self.b_cap), dtype=torch.int32, device=dev)
        self._idx_keep = None

    @classmethod
    def from_workload(cls, w, X, y, x0, b_cap: Optional[int] = None):
        from . import workloads as W
        mask = STATS_NORM | (STATS_IP if w.test != W.TEST_NORM else 0)
        return cls(w.dims, w.act, w.has_bias, w.prec, w.M, b_cap or w.b_cap, w.opt, X, y, x0,
                   momentum=w.momentum, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                   weight_decay=w.weight_decay, stats_mask=mask)

    # -- the hot path ------------------------------------------------------
    def upload_indices(self, idx: np.ndarray):
        """Copy an int32 [M, b] index array to the device; returns (device tensor, b)."""
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        assert idx.ndim == 2 and idx.shape[0] == self.M
        t = self._torch.as_tensor(idx).to(self._X.device)
        return t, int(idx.shape[1])

    def local_step_dev(self, idx_dev, b: int, lr: float):
        """idx_dev: device int32 tensor holding M*b contiguous indices."""
        self._idx_keep = idx_dev
        _check(self._lib.abs_local_step(self._ctx, idx_dev.data_ptr(), int(b), float(lr)), self._ctx)

    def local_step_graphed_dev(self, idx_dev, b: int, lr: float):
        """As local_step_dev, replaying a captured HIP graph once this batch size has been seen twice."""
        self._idx_keep = idx_dev
        _check(self._lib.abs_local_step_graphed(self._ctx, idx_dev.data_ptr(), int(b), float(lr)), self._ctx)

    def graph_count(self) -> int:
        n = C.c_int(0)
        _check(self._lib.abs_graph_count(self._ctx, C.byref(n)), self._ctx)
        return n.value

    def local_step(self, idx: np.ndarray, lr: float):
        t, b = self.upload_indices(idx)
        self.local_step_dev(t, b, lr)

    def local_step_accumulated(self, idx: np.ndarray, micro_b: int, lr: float):
        """One step on an int32 [M, b] index array, processed micro_b samples at a time."""
        t, b = self.upload_indices(idx)
        self._idx_keep = t
        _check(self._lib.abs_local_step_accumulated(self._ctx, t.data_ptr(), b, int(micro_b), float(lr)), self._ctx)

    def local_step_ragged(self, idx_rows, lr: float):
        """idx_rows: M index arrays of (possibly) different lengths, one per worker."""
        assert len(idx_rows) == self.M
        bs = [int(len(r)) for r in idx_rows]
        ldi = max(bs)
        host = np.zeros((self.M, ldi), dtype=np.int32)
        for m, r in enumerate(idx_rows):
            host[m, :bs[m]] = np.asarray(r, dtype=np.int32)
        t = self._torch.as_tensor(host).to(self._X.device)
        self._idx_keep = t
        _check(self._lib.abs_local_step_ragged(self._ctx, t.data_ptr(), ldi, (C.c_int * self.M)(*bs), float(lr)),
               self._ctx)

    def norm_test_per_worker(self, etas) -> List[TestResult]:
        out = (TestResult * self.M)()
        assert len(etas) == self.M
        _check(self._lib.abs_norm_test_per_worker(self._ctx, (C.c_double * self.M)(*[float(e) for e in etas]), out),
               self._ctx)
        return list(out)

    def norm_test(self, eta: float) -> List[TestResult]:
        out = (TestResult * self.M)()
        _check(self._lib.abs_norm_test(self._ctx, float(eta), out), self._ctx)
        return list(out)

    def norm_test_fpc(self, eta: float, n_total: int) -> List[TestResult]:
        out = (TestResult * self.M)()
        _check(self._lib.abs_norm_test_fpc(self._ctx, float(eta), int(n_total), out), self._ctx)
        return list(out)

    def inner_product_test(self, theta: float, nu: float = 0.0) -> List[TestResult]:
        out = (TestResult * self.M)()
        _check(self._lib.abs_inner_product_test(self._ctx, float(theta), float(nu), out), self._ctx)
        return list(out)

    def test_and_next_batch_size(self, b_cur: int, b_cap: int, eta: float = 0.0, theta: float = 0.0, nu: float = 0.0,
                                 sync_max: bool = True) -> List[int]:
        """The batch test of the last step followed by the batch-size rule, for tight loops: the same two library
        calls as norm_test / inner_product_test + next_batch_size, on argument arrays that are kept between calls
        (theta > 0 selects the inner-product test, augmented when nu > 0; otherwise the norm test with eta).  The
        test results of the call stay readable in `self.last_results`."""
        M = self.M
        if getattr(self, "_loop_args", None) is None:
            self._loop_args = ((TestResult * M)(), (C.c_int * M)(), (C.c_int * M)())
        out, cur, nxt = self._loop_args
        if theta > 0.0:
            _check(self._lib.abs_inner_product_test(self._ctx, theta, nu, out), self._ctx)
        else:
            _check(self._lib.abs_norm_test(self._ctx, eta, out), self._ctx)
        for m in range(M):
            cur[m] = b_cur
        _check(self._lib.abs_next_batch_size(out, M, cur, b_cap, 1 if sync_max else 0, nxt))
        self.last_results = out
        return nxt

    def cross_worker_test(self, eta: float) -> TestResult:
        out = TestResult()
        _check(self._lib.abs_cross_worker_test(self._ctx, float(eta), C.byref(out)), self._ctx)
        return out

    def average_replicas(self):
        _check(self._lib.abs_average_replicas(self._ctx), self._ctx)

    # -- parity helpers ----------------------------------------------------
    def get_params(self, m: int) -> np.ndarray:
        out = np.empty(self.n_params, dtype=np.float32)
        _check(self._lib.abs_get_params(self._ctx, int(m), out.ctypes.data), self._ctx)
        return out

    def set_params(self, m: int, x: np.ndarray):
        x = np.ascontiguousarray(x, dtype=np.float32)
        assert x.size == self.n_params
        _check(self._lib.abs_set_params(self._ctx, int(m), x.ctypes.data), self._ctx)

    def get_grad(self, m: int) -> np.ndarray:
        out = np.empty(self.n_params, dtype=np.float32)
        _check(self._lib.abs_get_grad(self._ctx, int(m), out.ctypes.data), self._ctx)
        return out

    def get_opt_state(self, m: int, which: int = 0) -> np.ndarray:
        out = np.empty(self.n_params, dtype=np.float32)
        _check(self._lib.abs_get_opt_state(self._ctx, int(m), int(which), out.ctypes.data), self._ctx)
        return out

    def set_fused_update(self, on: bool = True):
        """The optimizer step inside the weight-gradient epilogue (bf16 default) or as a kernel of its own."""
        _check(self._lib.abs_set_fused_update(self._ctx, int(bool(on))), self._ctx)

    def set_gram_ip_max_batch(self, b_max: int):
        """Largest local batch whose inner products <g_i, gbar> come from Gram matrices (0: never)."""
        _check(self._lib.abs_set_gram_ip_max_batch(self._ctx, int(b_max)), self._ctx)

    def counters(self):
        """(rounds k, local steps, samples B) of Alg. 1 as kept by the library."""
        k, h, B = C.c_longlong(0), C.c_longlong(0), C.c_longlong(0)
        _check(self._lib.abs_get_counters(self._ctx, C.byref(k), C.byref(h), C.byref(B)), self._ctx)
        return k.value, h.value, B.value

    def get_per_sample(self, m: int, b: int, want_q: bool = False):
        n = np.empty(b, dtype=np.float32)
        q = np.empty(b, dtype=np.float32) if want_q else None
        _check(self._lib.abs_get_per_sample(self._ctx, int(m), n.ctypes.data,
                                            q.ctypes.data if want_q else None), self._ctx)
        return n, q

    def profile_enable(self, on: bool = True):
        _check(self._lib.abs_profile_enable(self._ctx, int(bool(on))), self._ctx)

    def guard_intact(self) -> bool:
        """True if the canary bytes behind the workspace still hold their pattern."""
        self._torch.cuda.synchronize()
        return bool((self._ws[-self._guard:] == 0xA5).all().item())

    def profile_pause(self, paused: bool = True):
        _check(self._lib.abs_profile_pause(self._ctx, int(bool(paused))), self._ctx)

    def profile_read(self):
        """{kernel class: dict(calls, total_ms, flops, bytes)} accumulated since profile_enable."""
        buf = (ProfileEntry * 64)()
        n = C.c_int(0)
        _check(self._lib.abs_profile_read(self._ctx, 64, buf, C.byref(n)), self._ctx)
        return {buf[i].name.decode(): dict(calls=buf[i].calls, total_ms=buf[i].total_ms,
                                           flops=buf[i].flops, bytes=buf[i].bytes)
                for i in range(n.value)}

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            self._lib.abs_destroy(self._ctx)
            self._ctx = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def layer_stats(a_list, delta_list, want_per_sample: bool = False, want_gbar: bool = False):
    """Statistics alone on device bf16 tensors a_list[l] [M,b,in_l], delta_list[l] [M,b,out_l]."""
    import torch
    lib = load_library()
    L = len(a_list)
    M, b = int(a_list[0].shape[0]), int(a_list[0].shape[1])
    ins = (C.c_int * L)(*[int(t.shape[2]) for t in a_list])
    outs = (C.c_int * L)(*[int(t.shape[2]) for t in delta_list])
    for t in list(a_list) + list(delta_list):
        assert t.dtype == torch.bfloat16 and t.is_contiguous() and t.is_cuda
    nbytes = C.c_size_t(0)
    _check(lib.abs_layer_stats_workspace_bytes(L, ins, outs, M, b, C.byref(nbytes)))
    ws = torch.empty(nbytes.value + 256, dtype=torch.uint8, device=a_list[0].device)
    base = (ws.data_ptr() + 255) // 256 * 256
    ap = (C.c_void_p * L)(*[t.data_ptr() for t in a_list])
    dp = (C.c_void_p * L)(*[t.data_ptr() for t in delta_list])
    out = (TestResult * M)()
    n_out = torch.empty((M, b), dtype=torch.float32, device=ws.device) if want_per_sample else None
    q_out = torch.empty((M, b), dtype=torch.float32, device=ws.device) if want_per_sample else None
    Wsum = sum(int(i) * int(o) for i, o in zip(ins, outs))
    gbar = torch.empty((M, Wsum), dtype=torch.float32, device=ws.device) if want_gbar else None
    _check(lib.abs_layer_stats(L, ins, outs, M, b, ap, dp, base, nbytes.value, _stream_ptr(), out,
                               n_out.data_ptr() if want_per_sample else None,
                               q_out.data_ptr() if want_per_sample else None,
                               gbar.data_ptr() if want_gbar else None))
    return list(out), n_out, q_out, gbar


def lr_schedule(step: int, total_steps: int, warmup_steps: int, peak: float, floor: float) -> float:
    lib = load_library()
    out = C.c_double(0.0)
    _check(lib.abs_lr_schedule(int(step), int(total_steps), int(warmup_steps), float(peak), float(floor),
                               C.byref(out)))
    return out.value


def lr_linear_scaling(lr_ref: float, b: int, b_ref: int) -> float:
    lib = load_library()
    out = C.c_double(0.0)
    _check(lib.abs_lr_linear_scaling(float(lr_ref), int(b), int(b_ref), C.byref(out)))
    return out.value


def copy_probe(src, dst):
    """Run the library's plain copy kernel on two equally sized contiguous device tensors."""
    lib = load_library()
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib.abs_copy_probe(src.data_ptr(), dst.data_ptr(), nbytes, _stream_ptr()))


def average_bf16(params, scratch=None):
    """In-place mean over dim 0 of a contiguous bf16 device tensor [M, n]; `scratch` (bf16, n elements,
    optional) lets a large block be averaged in two passes."""
    lib = load_library()
    M, n = int(params.shape[0]), int(params[0].numel())
    if scratch is not None:
        assert scratch.is_contiguous() and scratch.numel() >= n and scratch.element_size() == 2
    _check(lib.abs_average_bf16(params.data_ptr(), M, n, scratch.data_ptr() if scratch is not None else None,
                                _stream_ptr()))


def average_bf16_static(params):
    """average_bf16 through the entry point that allocates nothing (the mean buffer lives in the library)."""
    lib = load_library()
    M, n = int(params.shape[0]), int(params[0].numel())
    _check(lib.abs_average_bf16_static(params.data_ptr(), M, n, _stream_ptr()))
