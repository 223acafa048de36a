"""Python binding of liblpc_hip.so: the same names as include/lpc.h, argument marshalling only.

Every step of the path runs in the HIP kernels of the library; torch is used for device
memory and streams.  There is no CPU fallback: if the library cannot be loaded this module
raises at import time.
"""
import ctypes as C
import os

import torch  # imported first so that the process-wide HIP runtime is torch's

from . import build as _build

LOSS_LOGISTIC, LOSS_SQUARED, LOSS_MLP_SOFTMAX = 0, 1, 2
ALGO_LPC, ALGO_ALPC_SC, ALGO_ALPC_GC = 0, 1, 2
CLIP_LAMBDA, CLIP_CSIGMA = 0, 1
SCHEME_A, SCHEME_B, SCHEME_C = 0, 1, 2
BATCH_WORKER, BATCH_SHARED = 1, 2
OK, EINVAL, ENULL, ESHAPE, EWORKSPACE, ENONFINITE, EDEVICE, EUNSUPPORTED = 0, -1, -2, -3, -4, -5, -6, -7

_vp = C.c_void_p


class EpochStats(C.Structure):
    _fields_ = [("bits_sent", C.c_uint64), ("messages", C.c_uint64), ("clipped", C.c_uint64),
                ("max_delta", C.c_float), ("nonfinite", C.c_int32)]


class Problem(C.Structure):
    _fields_ = [("n", C.c_int64), ("d", C.c_int64), ("loss", C.c_int32),
                ("X", _vp), ("ldx", C.c_int64),
                ("row_ptr", _vp), ("col_idx", _vp), ("vals", _vp), ("nnz", C.c_int64),
                ("y", _vp), ("mlp_dims", C.POINTER(C.c_int32)), ("mlp_nlayers", C.c_int32),
                ("lambda1", C.c_float), ("lambda2", C.c_float)]


class Config(C.Structure):
    _fields_ = [("algo", C.c_int32), ("N", C.c_int32), ("B", C.c_int32), ("m", C.c_int32), ("bits", C.c_int32),
                ("clip_mode", C.c_int32), ("clip", C.c_float), ("scheme", C.c_int32),
                ("eta", C.c_float), ("L", C.c_float), ("sigma", C.c_float), ("tau1", C.c_float),
                ("tau2", C.c_float), ("alpha", C.c_float), ("seed", C.c_uint64), ("n_full", C.c_int64)]


EXPORTS = {
    "lpc_workspace_bytes": (C.c_size_t, [C.POINTER(Problem), C.POINTER(Config)]),
    "lpc_create": (C.c_int, [C.POINTER(_vp), C.POINTER(Problem), C.POINTER(Config), _vp, C.c_size_t]),
    "lpc_destroy": (None, [_vp]),
    "lpc_status_string": (C.c_char_p, [C.c_int]),
    "lpc_d_pad": (C.c_int64, [C.c_int64]),
    "lpc_words_per_msg": (C.c_int64, [C.c_int64, C.c_int32]),
    "lpc_full_grad": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _vp]),
    "lpc_worker_vr_grad": (C.c_int, [_vp, _vp, _vp, _vp, C.c_uint32, C.c_uint32, C.c_int32, C.c_int32, C.c_int32,
                                     _vp, _vp, _vp]),
    "lpc_vector_stats": (C.c_int, [_vp, _vp, C.c_int32, _vp, _vp]),
    "lpc_quantize_clip": (C.c_int, [_vp, _vp, _vp, _vp, C.c_uint32, C.c_uint32, _vp, _vp, _vp, _vp]),
    "lpc_dequantize_avg": (C.c_int, [_vp, _vp, _vp, _vp, _vp]),
    "lpc_dequantize_shared": (C.c_int, [_vp, _vp, _vp, C.c_int32, C.c_uint32, C.c_uint32, _vp, _vp]),
    "lpc_exchange": (C.c_int, [_vp, _vp, C.c_uint32, C.c_uint32, _vp, _vp, _vp, _vp]),
    "lpc_exchange_static": (C.c_int, [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_uint64, _vp,
                                      C.c_uint32, C.c_uint32, _vp, _vp, _vp, _vp, _vp]),
    "lpc_prox_step": (C.c_int, [_vp, _vp, _vp, _vp, C.c_float, _vp]),
    "lpc_epoch": (C.c_int, [_vp, _vp, _vp, _vp, C.c_uint32, _vp]),
    "lpc_epoch_traced": (C.c_int, [_vp, _vp, _vp, _vp, C.c_uint32, _vp, _vp, C.POINTER(C.c_uint64), _vp]),
    "lpc_resident_trace": (C.c_int, [_vp, C.c_int32, _vp, _vp]),
    "lpc_bits_per_iteration": (C.c_int, [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_uint64)]),
    "lpc_epoch_report": (C.c_int, [_vp, _vp, _vp, _vp, C.c_uint32, _vp, _vp]),
    "lpc_clip_sweep": (C.c_int, [_vp, _vp, C.c_int32, C.POINTER(C.c_float), C.c_int32, C.c_uint32, _vp, _vp, _vp,
                                 C.POINTER(C.c_double), C.POINTER(C.c_uint64), _vp]),
    "lpc_objective": (C.c_int, [_vp, _vp, C.POINTER(C.c_double), _vp]),
    "lpc_take_device_flags": (C.c_int, [_vp, _vp]),
    "lpc_gradient_mapping": (C.c_int, [_vp, _vp, C.c_float, C.POINTER(C.c_double), _vp]),
    "lpc_theorem2_lhs": (C.c_int, [C.c_int64, C.c_int32, C.c_double, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                   C.c_double, C.c_int32, C.POINTER(C.c_double)]),
    "lpc_code_histogram": (C.c_int, [_vp, _vp, _vp, _vp]),
    "lpc_huffman_bits": (C.c_int, [_vp, C.c_int32, _vp, C.POINTER(C.c_uint64)]),
    "lpc_huffman_encode": (C.c_int, [_vp, _vp, _vp, _vp, C.c_int64, C.POINTER(C.c_uint64), _vp]),
    "lpc_tune": (C.c_int, [_vp, C.c_int32, C.c_int64]),
    "lpc_debug_gemm": (C.c_int, [_vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_int64,
                                 C.c_int32, C.c_int32, C.c_float, _vp, C.c_int32, C.c_int32, _vp]),
    "lpc_profile_enable": (C.c_int, [_vp, C.c_int32]),
    "lpc_profile_read": (C.c_int, [_vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_int32), _vp]),
}
TUNE_ITER_FORM, TUNE_ITER_TILE, TUNE_ITER_THREADS, TUNE_SPIN_LIMIT = 0, 1, 2, 3
PROF_CLASSES = ("full_rows", "full_fold", "vr_rows", "vr_fold", "exchange", "resident")

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblpc_hip.so")


def _load():
    if not os.path.exists(LIB_PATH):
        _build.build()
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in EXPORTS.items():
        fn = getattr(lib, name)   # AttributeError here means the library lacks a declared entry point
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()


class LpcError(RuntimeError):
    def __init__(self, code, where):
        msg = lib.lpc_status_string(code).decode()
        super().__init__("%s: %s (%d)" % (where, msg, code))
        self.code = code


def _chk(code, where):
    if code != OK:
        raise LpcError(code, where)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def d_pad(d):
    return int(lib.lpc_d_pad(d))


def words_per_msg(d, bits):
    return int(lib.lpc_words_per_msg(d, bits))


def theorem2_lhs(d, bits, lam, d_lambda, N, B, m, rho, scheme=SCHEME_A):
    out = C.c_double()
    _chk(lib.lpc_theorem2_lhs(d, bits, lam, d_lambda, N, B, m, rho, scheme, C.byref(out)), "lpc_theorem2_lhs")
    return out.value


def bits_per_iteration(d, bits, N, scheme=SCHEME_A):
    out = C.c_uint64()
    _chk(lib.lpc_bits_per_iteration(d, bits, N, scheme, C.byref(out)), "lpc_bits_per_iteration")
    return int(out.value)


def huffman_bits(counts):
    """counts: host sequence of symbol counts -> (encoded bits, list of code lengths)."""
    n = len(counts)
    arr = (C.c_uint64 * n)(*[int(c) for c in counts])
    lens = (C.c_int32 * n)()
    out = C.c_uint64()
    _chk(lib.lpc_huffman_bits(arr, n, lens, C.byref(out)), "lpc_huffman_bits")
    return int(out.value), list(lens)


def make_config(algo=ALGO_LPC, N=1, B=1, m=1, bits=32, clip_mode=CLIP_LAMBDA, clip=1.0, scheme=SCHEME_A, eta=0.1,
                L=0.0, sigma=0.0, tau1=0.0, tau2=0.0, alpha=0.0, seed=0, n_full=0):
    return Config(algo, N, B, m, bits, clip_mode, clip, scheme, eta, L, sigma, tau1, tau2, alpha, seed, n_full)


def exchange_static(d, N, bits, clip_mode, clip, seed, U, epoch, iter_, packed, delta_out, u_avg, flags_out=None,
                    stream=None):
    """lpc_exchange without a context: allocates nothing (the library's static device scratch)."""
    _chk(lib.lpc_exchange_static(d, N, bits, clip_mode, clip, seed, _ptr(U), epoch, iter_, _ptr(packed),
                                 _ptr(delta_out), _ptr(u_avg), _ptr(flags_out), _stream(stream)),
         "lpc_exchange_static")


class Context:
    """Owns an lpc_ctx and the torch tensors (data, workspace) it borrows."""

    def __init__(self, loss, y, config, X=None, csr=None, d=None, mlp_dims=None, lambda1=0.0, lambda2=0.0):
        self._keep = [y]
        p = Problem()
        p.loss, p.lambda1, p.lambda2 = loss, lambda1, lambda2
        assert y.is_cuda and y.dtype == torch.float32 and y.is_contiguous()
        p.y = y.data_ptr()
        if X is not None:
            assert X.is_cuda and X.dtype == torch.float32 and X.dim() == 2 and X.stride(1) == 1
            self._keep.append(X)
            p.n, p.X, p.ldx = X.shape[0], X.data_ptr(), X.stride(0)
            p.d = X.shape[1] if d is None else d
        else:
            row_ptr, col_idx, vals, dd = csr
            for t, dt in ((row_ptr, torch.int32), (col_idx, torch.int32), (vals, torch.float32)):
                assert t.is_cuda and t.dtype == dt and t.is_contiguous()
            self._keep += [row_ptr, col_idx, vals]
            p.n, p.d, p.nnz = row_ptr.numel() - 1, dd, vals.numel()
            p.row_ptr, p.col_idx, p.vals = row_ptr.data_ptr(), col_idx.data_ptr(), vals.data_ptr()
        if mlp_dims is not None:
            self._dims = (C.c_int32 * len(mlp_dims))(*mlp_dims)
            p.mlp_dims, p.mlp_nlayers = self._dims, len(mlp_dims) - 1
        self.problem, self.config = p, config
        self.n, self.d, self.N, self.bits = int(p.n), int(p.d), config.N, config.bits
        self.d_pad = d_pad(self.d)
        self.W = words_per_msg(self.d, self.bits) if self.bits < 32 else 0
        self.device = y.device
        need = lib.lpc_workspace_bytes(C.byref(p), C.byref(config))
        self.workspace = torch.empty(max(int(need), 256), dtype=torch.uint8, device=self.device)
        handle = _vp()
        _chk(lib.lpc_create(C.byref(handle), C.byref(p), C.byref(config), self.workspace.data_ptr(),
                            self.workspace.numel()), "lpc_create")
        self._h = handle

    def close(self):
        if getattr(self, "_h", None):
            torch.cuda.synchronize(self.device)
            lib.lpc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the calls of include/lpc.h -------------------------------------------------------
    def full_grad(self, w, mu, z=None, f_out=None, stream=None):
        _chk(lib.lpc_full_grad(self._h, _ptr(w), _ptr(mu), _ptr(z), _ptr(f_out), _stream(stream)), "lpc_full_grad")

    def worker_vr_grad(self, w, w_snap, z_snap, epoch, iter_, U, stats=None, kind=BATCH_WORKER, worker_begin=0,
                       worker_end=None, stream=None):
        we = self.N if worker_end is None else worker_end
        _chk(lib.lpc_worker_vr_grad(self._h, _ptr(w), _ptr(w_snap), _ptr(z_snap), epoch, iter_, kind, worker_begin,
                                    we, _ptr(U), _ptr(stats), _stream(stream)), "lpc_worker_vr_grad")

    def vector_stats(self, U, nvec, stats, stream=None):
        _chk(lib.lpc_vector_stats(self._h, _ptr(U), nvec, _ptr(stats), _stream(stream)), "lpc_vector_stats")

    def quantize_clip(self, U, stats, delta_in, epoch, iter_, packed, delta_out, n_clipped=None, stream=None):
        _chk(lib.lpc_quantize_clip(self._h, _ptr(U), _ptr(stats), _ptr(delta_in), epoch, iter_, _ptr(packed),
                                   _ptr(delta_out), _ptr(n_clipped), _stream(stream)), "lpc_quantize_clip")

    def dequantize_avg(self, packed, delta, u_avg, stream=None):
        _chk(lib.lpc_dequantize_avg(self._h, _ptr(packed), _ptr(delta), _ptr(u_avg), _stream(stream)),
             "lpc_dequantize_avg")

    def dequantize_shared(self, packed, delta, requantize, epoch, iter_, u_avg, stream=None):
        _chk(lib.lpc_dequantize_shared(self._h, _ptr(packed), _ptr(delta), 1 if requantize else 0, epoch, iter_,
                                       _ptr(u_avg), _stream(stream)), "lpc_dequantize_shared")

    def exchange(self, U, epoch, iter_, packed, delta_out, u_avg, stream=None):
        _chk(lib.lpc_exchange(self._h, _ptr(U), epoch, iter_, _ptr(packed), _ptr(delta_out), _ptr(u_avg),
                              _stream(stream)), "lpc_exchange")

    def prox_step(self, w, u_avg, mu, step, stream=None):
        _chk(lib.lpc_prox_step(self._h, _ptr(w), _ptr(u_avg), _ptr(mu), step, _stream(stream)), "lpc_prox_step")

    def epoch(self, w_snap, epoch, y=None, z=None, stream=None):
        _chk(lib.lpc_epoch(self._h, _ptr(w_snap), _ptr(y), _ptr(z), epoch, _stream(stream)), "lpc_epoch")

    def epoch_traced(self, w_snap, epoch, y=None, z=None, stream=None, coded=False):
        """epoch() that also returns (delta_trace float32 [m][N], nclip_trace int32 [m][N]) on the device and,
        with coded=True, the entropy-coded size of every message as a nested host list [m][N]."""
        m = int(self.config.m)
        dtr = torch.empty((m, self.N), dtype=torch.float32, device=self.device)
        ntr = torch.empty((m, self.N), dtype=torch.int32, device=self.device)   # uint32 bit patterns
        sizes = (C.c_uint64 * (m * self.N))() if coded else None
        _chk(lib.lpc_epoch_traced(self._h, _ptr(w_snap), _ptr(y), _ptr(z), epoch, _ptr(dtr), _ptr(ntr), sizes,
                                  _stream(stream)), "lpc_epoch_traced")
        if coded:
            return dtr, ntr, [[int(sizes[t * self.N + i]) for i in range(self.N)] for t in range(m)]
        return dtr, ntr

    def epoch_report(self, w_snap, epoch, y=None, z=None, stream=None):
        """epoch() plus its summary (EpochStats on the host)."""
        st = EpochStats()
        _chk(lib.lpc_epoch_report(self._h, _ptr(w_snap), _ptr(y), _ptr(z), epoch, C.byref(st), _stream(stream)),
             "lpc_epoch_report")
        return st

    def clip_sweep(self, w0, clips, epochs, epoch0=0, stream=None):
        """Objective and total clipped coordinates after `epochs` epochs from w0 for each candidate clip value."""
        k = len(clips)
        arr = (C.c_float * k)(*[float(v) for v in clips])
        P = (C.c_double * k)()
        clipped = (C.c_uint64 * k)()
        work = [torch.empty_like(w0) for _ in range(3)]
        alpc = int(self.config.algo) != 0
        _chk(lib.lpc_clip_sweep(self._h, _ptr(w0), k, arr, epochs, epoch0, _ptr(work[0]),
                                _ptr(work[1]) if alpc else None, _ptr(work[2]) if alpc else None, P, clipped,
                                _stream(stream)), "lpc_clip_sweep")
        return list(P), [int(v) for v in clipped], work[0]

    def objective(self, w, stream=None):
        out = C.c_double()
        _chk(lib.lpc_objective(self._h, _ptr(w), C.byref(out), _stream(stream)), "lpc_objective")
        return out.value

    def gradient_mapping(self, w, eta, stream=None):
        out = C.c_double()
        _chk(lib.lpc_gradient_mapping(self._h, _ptr(w), eta, C.byref(out), _stream(stream)), "lpc_gradient_mapping")
        return out.value

    def huffman_encode(self, packed, lens, capacity_words=None, stream=None):
        """One packed message (device) -> (stream words on the device, total bits) under the canonical code of
        `lens` (host sequence of 2^bits lengths)."""
        lens_arr = (C.c_int32 * len(lens))(*[int(v) for v in lens])
        total = C.c_uint64()
        if capacity_words is None:     # ask for the size first
            code = lib.lpc_huffman_encode(self._h, _ptr(packed), lens_arr, None, 0, C.byref(total), _stream(stream))
            if code not in (OK, ESHAPE):
                raise LpcError(code, "lpc_huffman_encode")
            capacity_words = (total.value + 31) // 32
        out = torch.empty(max(int(capacity_words), 1), dtype=torch.int32, device=self.device)
        _chk(lib.lpc_huffman_encode(self._h, _ptr(packed), lens_arr, _ptr(out), int(capacity_words), C.byref(total),
                                    _stream(stream)), "lpc_huffman_encode")
        return out[:(total.value + 31) // 32], int(total.value)

    def code_histogram(self, packed, counts=None, stream=None):
        """packed: one message (W uint32 words on the device) -> 2^bits int64 counts on the device."""
        if counts is None:
            counts = torch.empty(1 << self.config.bits, dtype=torch.int64, device=packed.device)
        _chk(lib.lpc_code_histogram(self._h, _ptr(packed), _ptr(counts), _stream(stream)), "lpc_code_histogram")
        return counts

    def tune(self, key, value):
        _chk(lib.lpc_tune(self._h, key, value), "lpc_tune")

    def profile_enable(self, on):
        _chk(lib.lpc_profile_enable(self._h, 1 if on else 0), "lpc_profile_enable")

    def resident_trace(self, on, read=False, stream=None):
        """Switches the phase time stamps of the resident inner loop on or off; with read=True first returns the last
        launch's stamps as m rows of 16 counter readings (100 MHz)."""
        out = None
        if read:
            out = (C.c_uint64 * (16 * self.config.m))()
        _chk(lib.lpc_resident_trace(self._h, 1 if on else 0, out, _stream(stream)), "lpc_resident_trace")
        return [list(out[16 * t:16 * t + 16]) for t in range(self.config.m)] if read else None

    def profile_read(self, stream=None):
        """{class: (total ms, launches, exact)} since the last read; exact = every record was one kernel timed by
        its own dispatch (no event-handling overhead in the interval)."""
        ms = (C.c_double * len(PROF_CLASSES))()
        cnt = (C.c_int64 * len(PROF_CLASSES))()
        exact = (C.c_int32 * len(PROF_CLASSES))()
        _chk(lib.lpc_profile_read(self._h, ms, cnt, exact, _stream(stream)), "lpc_profile_read")
        return {k: (ms[i], cnt[i], bool(exact[i])) for i, k in enumerate(PROF_CLASSES)}

    def take_device_flags(self, stream=None):
        return lib.lpc_take_device_flags(self._h, _stream(stream))


def context_from_problem(sp, **over):
    """Upload a synthetic problem description (fields as in lpc_synth.SynthProblem) and create its context.

    `over` overrides run parameters (N, B, m, bits, clip_mode, clip, eta, ...).
    """
    import numpy as np
    dev = torch.device("cuda:0")
    kw = dict(algo=sp.algo, N=sp.N, B=sp.B, m=sp.m, bits=sp.bits, clip_mode=sp.clip_mode, clip=sp.clip, eta=sp.eta,
              L=sp.L, seed=sp.seed, n_full=sp.n_full)
    kw.update(over)
    cfg = make_config(**kw)
    y = torch.from_numpy(sp.y).to(dev)
    if sp.csr is not None:
        rp, ci, va = (torch.from_numpy(np.ascontiguousarray(a)).to(dev) for a in sp.csr)
        return Context(sp.loss, y, cfg, csr=(rp, ci, va, sp.d), lambda1=sp.lambda1, lambda2=sp.lambda2)
    X = torch.from_numpy(sp.X).to(dev)
    return Context(sp.loss, y, cfg, X=X, d=sp.d, mlp_dims=sp.mlp_dims, lambda1=sp.lambda1, lambda2=sp.lambda2)
