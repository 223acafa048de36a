"""ctypes binding of the CPU oracle (oracle/liblpco.so).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg.  The product package never imports this module.
Arrays are numpy, host memory; argument marshalling only.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

LOSS_LOGISTIC, LOSS_SQUARED, LOSS_MLP_SOFTMAX = 0, 1, 2
ALGO_LPC, ALGO_ALPC_SC, ALGO_ALPC_GC = 0, 1, 2
CLIP_LAMBDA, CLIP_CSIGMA = 0, 1
TAG_QUANT, TAG_BATCH, TAG_SHARED, TAG_REQUANT = 0, 1, 2, 3
SCHEME_A, SCHEME_B, SCHEME_C = 0, 1, 2
OK, EINVAL, ENULL, ESHAPE, ENONFINITE, EUNSUPPORTED = 0, -1, -2, -3, -5, -7

_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)
_i32p = C.POINTER(C.c_int32)
_i64p = C.POINTER(C.c_int64)
_u32p = C.POINTER(C.c_uint32)
_u64p = C.POINTER(C.c_uint64)


class Problem(C.Structure):
    _fields_ = [("n", C.c_int64), ("d", C.c_int64), ("loss", C.c_int32),
                ("X", _f32p), ("ldx", C.c_int64),
                ("row_ptr", _i32p), ("col_idx", _i32p), ("vals", _f32p), ("nnz", C.c_int64),
                ("y", _f32p), ("mlp_dims", _i32p), ("mlp_nlayers", C.c_int32),
                ("lambda1", C.c_float), ("lambda2", C.c_float)]


class Config(C.Structure):
    _fields_ = [("algo", C.c_int32), ("N", C.c_int32), ("B", C.c_int32), ("m", C.c_int32), ("bits", C.c_int32),
                ("clip_mode", C.c_int32), ("clip", C.c_float), ("scheme", C.c_int32),
                ("eta", C.c_float), ("L", C.c_float), ("sigma", C.c_float), ("tau1", C.c_float),
                ("tau2", C.c_float), ("alpha", C.c_float), ("seed", C.c_uint64), ("n_full", C.c_int64)]


def _load():
    if _build.needs_build():
        _build.build()
    lib = C.CDLL(os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblpco.so"))
    P, K = C.POINTER(Problem), C.POINTER(Config)
    sig = {
        "lpco_philox4x32_10": (None, [_u32p, _u32p, _u32p]),
        "lpco_stream_word": (C.c_uint32, [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint64]),
        "lpco_sample_batch": (C.c_int, [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int32,
                                        C.c_int64, _i64p]),
        "lpco_d_pad": (C.c_int64, [C.c_int64]),
        "lpco_words_per_msg": (C.c_int64, [C.c_int64, C.c_int32]),
        "lpco_vector_stats": (C.c_int, [_f32p, C.c_int64, _f64p]),
        "lpco_delta_from_stats": (C.c_int, [_f64p, C.c_int64, C.c_int32, C.c_int32, C.c_float, _f32p, _f32p]),
        "lpco_quantize_codes": (C.c_int, [_f32p, C.c_int64, C.c_int32, C.c_float, C.c_float, C.c_uint64, C.c_uint32,
                                          C.c_uint32, C.c_uint32, C.c_uint32, _i32p, _u32p]),
        "lpco_pack": (C.c_int, [_i32p, C.c_int64, C.c_int32, _u32p]),
        "lpco_unpack": (C.c_int, [_u32p, C.c_int64, C.c_int32, _i32p]),
        "lpco_quantize_clip": (C.c_int, [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_uint64,
                                         C.c_uint32, C.c_uint32, _f32p, _f64p, _f32p, _u32p, _f32p, _u32p]),
        "lpco_dequantize_avg": (C.c_int, [C.c_int64, C.c_int32, C.c_int32, _u32p, _f32p, _f32p]),
        "lpco_plain_avg": (C.c_int, [C.c_int64, C.c_int32, _f32p, _f32p]),
        "lpco_dequantize_shared": (C.c_int, [C.c_int64, C.c_int32, C.c_int32, _u32p, C.c_float, C.c_int32,
                                             C.c_uint64, C.c_uint32, C.c_uint32, _f32p, _i32p]),
        "lpco_prox_step": (C.c_int, [C.c_int64, _f32p, _f32p, _f32p, C.c_float, C.c_float, C.c_float]),
        "lpco_full_grad": (C.c_int, [P, _f32p, C.c_int64, _f32p, _f32p, _f64p]),
        "lpco_worker_vr_grad": (C.c_int, [P, K, _f32p, _f32p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int32,
                                          C.c_int32, _f32p, _f64p]),
        "lpco_objective": (C.c_int, [P, _f32p, _f64p]),
        "lpco_mlp_relu_margin": (C.c_int, [P, _f32p, _i64p, C.c_int32, _f64p]),
        "lpco_gradient_mapping": (C.c_int, [P, _f32p, C.c_float, _f64p]),
        "lpco_theorem2_lhs": (C.c_double, [C.c_int64, C.c_int32, C.c_double, C.c_int64, C.c_int32, C.c_int32,
                                           C.c_int32, C.c_double, C.c_int32]),
        "lpco_huffman_bits": (C.c_uint64, [_u64p, C.c_int32, _i32p]),
        "lpco_code_histogram": (C.c_int, [_u32p, C.c_int64, C.c_int32, _u64p]),
        "lpco_huffman_encode": (C.c_int, [_u32p, C.c_int64, C.c_int32, _i32p, _u32p, C.c_int64, _u64p]),
        "lpco_huffman_decode": (C.c_int, [_u32p, C.c_uint64, C.c_int64, C.c_int32, _i32p, _i32p]),
        "lpco_alpc_params": (C.c_int, [P, K, C.c_uint32, _f32p, _f32p, _f32p, _f32p]),
        "lpco_epoch": (C.c_int, [P, K, _f32p, _f32p, _f32p, C.c_uint32, _u64p]),
        "lpco_epoch_traced": (C.c_int, [P, K, _f32p, _f32p, _f32p, C.c_uint32, _f32p, _u32p, _u64p]),
        "lpco_bits_per_message": (C.c_uint64, [C.c_int64, C.c_int32]),
        "lpco_bits_per_iteration": (C.c_uint64, [C.c_int64, C.c_int32, C.c_int32, C.c_int32]),
        "lpco_set_threads": (None, [C.c_int32]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__("oracle returned status %d" % code)
        self.code = code


def _chk(rc, allow=()):
    if rc != OK and rc not in allow:
        raise OracleError(rc)
    return rc


def _p(a, typ):
    return None if a is None else a.ctypes.data_as(typ)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def make_problem(loss, y, lambda1=0.0, lambda2=0.0, X=None, csr=None, d=None, mlp_dims=None):
    """Build a Problem; returns (struct, keepalive).  csr = (row_ptr, col_idx, vals, d)."""
    keep = []
    p = Problem()
    y = _f32(y); keep.append(y)
    p.y = _p(y, _f32p)
    p.loss = loss
    p.lambda1, p.lambda2 = lambda1, lambda2
    if X is not None:
        assert X.dtype == np.float32 and X.ndim == 2 and X.strides[1] == 4
        keep.append(X)
        p.n = X.shape[0]
        p.X = _p(X, _f32p)
        p.ldx = X.strides[0] // 4
        p.d = X.shape[1] if d is None else d
    else:
        rp, ci, va, dd = csr
        rp = np.ascontiguousarray(rp, dtype=np.int32); ci = np.ascontiguousarray(ci, dtype=np.int32)
        va = _f32(va); keep += [rp, ci, va]
        p.n, p.d, p.nnz = len(rp) - 1, dd, len(va)
        p.row_ptr, p.col_idx, p.vals = _p(rp, _i32p), _p(ci, _i32p), _p(va, _f32p)
    if mlp_dims is not None:
        md = np.ascontiguousarray(mlp_dims, dtype=np.int32); keep.append(md)
        p.mlp_dims, p.mlp_nlayers = _p(md, _i32p), len(md) - 1
    return p, keep


def make_config(algo=ALGO_LPC, N=1, B=1, m=1, bits=32, clip_mode=CLIP_LAMBDA, clip=1.0, scheme=SCHEME_A, eta=0.1,
                L=0.0, sigma=0.0, tau1=0.0, tau2=0.0, alpha=0.0, seed=0, n_full=0):
    return Config(algo, N, B, m, bits, clip_mode, clip, scheme, eta, L, sigma, tau1, tau2, alpha, seed, n_full)


# ---- thin wrappers -------------------------------------------------------------------------

def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32); k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib.lpco_philox4x32_10(_p(c, _u32p), _p(k, _u32p), _p(out, _u32p))
    return out


def stream_word(seed, epoch, iter_, tag, worker, index):
    return int(lib.lpco_stream_word(seed, epoch, iter_, tag, worker, index))


def sample_batch(seed, epoch, iter_, tag, worker, B, n):
    out = np.zeros(B, dtype=np.int64)
    _chk(lib.lpco_sample_batch(seed, epoch, iter_, tag, worker, B, n, _p(out, _i64p)))
    return out


def d_pad(d):
    return int(lib.lpco_d_pad(d))


def words_per_msg(d, bits):
    return int(lib.lpco_words_per_msg(d, bits))


def vector_stats(u):
    u = _f32(u)
    st = np.zeros(4, dtype=np.float64)
    rc = lib.lpco_vector_stats(_p(u, _f32p), u.size, _p(st, _f64p))
    _chk(rc, allow=(ENONFINITE,))
    return st


def delta_from_stats(stats, d, bits, clip_mode, clip):
    st = np.ascontiguousarray(stats, dtype=np.float64)
    de, th = C.c_float(), C.c_float()
    _chk(lib.lpco_delta_from_stats(_p(st, _f64p), d, bits, clip_mode, clip, C.byref(de), C.byref(th)))
    return de.value, th.value


def quantize_codes(u, bits, delta, thresh=float("inf"), seed=0, epoch=0, iter_=0, tag=TAG_QUANT, worker=0):
    u = _f32(u)
    codes = np.zeros(u.size, dtype=np.int32)
    nc = C.c_uint32()
    _chk(lib.lpco_quantize_codes(_p(u, _f32p), u.size, bits, delta, thresh, seed, epoch, iter_, tag, worker,
                                 _p(codes, _i32p), C.byref(nc)))
    return codes, nc.value


def pack(codes, bits):
    codes = np.ascontiguousarray(codes, dtype=np.int32)
    words = np.zeros(words_per_msg(codes.size, bits), dtype=np.uint32)
    _chk(lib.lpco_pack(_p(codes, _i32p), codes.size, bits, _p(words, _u32p)))
    return words


def unpack(words, d, bits):
    words = np.ascontiguousarray(words, dtype=np.uint32)
    codes = np.zeros(d, dtype=np.int32)
    _chk(lib.lpco_unpack(_p(words, _u32p), d, bits, _p(codes, _i32p)))
    return codes


def quantize_clip(U, d, bits, clip_mode=CLIP_LAMBDA, clip=1.0, seed=0, epoch=0, iter_=0, stats=None, delta_in=None):
    """U: [N, d_pad] float32.  Returns packed [N, W], delta [N], n_clipped [N], status."""
    U = _f32(U)
    N = U.shape[0]
    assert U.shape[1] == d_pad(d)
    W = words_per_msg(d, bits)
    packed = np.zeros((N, W), dtype=np.uint32)
    delta = np.zeros(N, dtype=np.float32)
    ncl = np.zeros(N, dtype=np.uint32)
    st = None if stats is None else np.ascontiguousarray(stats, dtype=np.float64)
    di = None if delta_in is None else _f32(delta_in)
    rc = lib.lpco_quantize_clip(d, N, bits, clip_mode, clip, seed, epoch, iter_, _p(U, _f32p), _p(st, _f64p),
                                _p(di, _f32p), _p(packed, _u32p), _p(delta, _f32p), _p(ncl, _u32p))
    _chk(rc, allow=(ENONFINITE,))
    return packed, delta, ncl, rc


def dequantize_avg(packed, delta, d, bits):
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    delta = _f32(delta)
    out = np.zeros(d, dtype=np.float32)
    _chk(lib.lpco_dequantize_avg(d, packed.shape[0], bits, _p(packed, _u32p), _p(delta, _f32p), _p(out, _f32p)))
    return out


def plain_avg(U, d):
    U = _f32(U)
    out = np.zeros(d, dtype=np.float32)
    _chk(lib.lpco_plain_avg(d, U.shape[0], _p(U, _f32p), _p(out, _f32p)))
    return out


def dequantize_shared(packed, delta_shared, d, bits, requantize=False, seed=0, epoch=0, iter_=0):
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    out = np.zeros(d, dtype=np.float32)
    sums = np.zeros(d, dtype=np.int32)
    _chk(lib.lpco_dequantize_shared(d, packed.shape[0], bits, _p(packed, _u32p), delta_shared, int(requantize), seed,
                                    epoch, iter_, _p(out, _f32p), _p(sums, _i32p)))
    return out, sums


def prox_step(w, u_avg, mu, step, lambda1, lambda2):
    w = _f32(w).copy(); u_avg = _f32(u_avg); mu = _f32(mu)
    _chk(lib.lpco_prox_step(w.size, _p(w, _f32p), _p(u_avg, _f32p), _p(mu, _f32p), step, lambda1, lambda2))
    return w


def full_grad(problem, w, n_rows=0, want_z=True):
    w = _f32(w)
    mu = np.zeros(problem.d, dtype=np.float32)
    z = np.zeros(problem.n, dtype=np.float32) if (want_z and problem.loss != LOSS_MLP_SOFTMAX) else None
    f = C.c_double()
    _chk(lib.lpco_full_grad(C.byref(problem), _p(w, _f32p), n_rows, _p(mu, _f32p), _p(z, _f32p), C.byref(f)))
    return mu, z, f.value


def worker_vr_grad(problem, config, w, w_snap, epoch, iter_, tag=TAG_BATCH, worker_begin=0, worker_end=None):
    w = _f32(w); w_snap = _f32(w_snap)
    nrow = 1 if tag == TAG_SHARED else config.N
    if worker_end is None:
        worker_end = nrow
    dp = d_pad(problem.d)
    U = np.zeros((nrow, dp), dtype=np.float32)
    stats = np.zeros((nrow, 4), dtype=np.float64)
    rc = lib.lpco_worker_vr_grad(C.byref(problem), C.byref(config), _p(w, _f32p), _p(w_snap, _f32p), epoch, iter_,
                                 tag, worker_begin, worker_end, _p(U, _f32p), _p(stats, _f64p))
    _chk(rc, allow=(ENONFINITE,))
    return U, stats


def objective(problem, w):
    w = _f32(w)
    out = C.c_double()
    _chk(lib.lpco_objective(C.byref(problem), _p(w, _f32p), C.byref(out)))
    return out.value


def mlp_relu_margin(problem, w, idx):
    w = _f32(w)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = C.c_double()
    _chk(lib.lpco_mlp_relu_margin(C.byref(problem), _p(w, _f32p), _p(idx, _i64p), idx.size, C.byref(out)))
    return out.value


def gradient_mapping(problem, w, eta):
    w = _f32(w)
    out = C.c_double()
    _chk(lib.lpco_gradient_mapping(C.byref(problem), _p(w, _f32p), eta, C.byref(out)))
    return out.value


def theorem2_lhs(d, bits, lam, d_lambda, N, B, m, rho, scheme=SCHEME_A):
    return float(lib.lpco_theorem2_lhs(d, bits, lam, d_lambda, N, B, m, rho, scheme))


def huffman_bits(counts):
    counts = np.ascontiguousarray(counts, dtype=np.uint64)
    lens = np.zeros(counts.size, dtype=np.int32)
    bits = lib.lpco_huffman_bits(_p(counts, _u64p), counts.size, _p(lens, _i32p))
    return int(bits), lens


def code_histogram(words, d, bits):
    words = np.ascontiguousarray(words, dtype=np.uint32)
    counts = np.zeros(1 << bits, dtype=np.uint64)
    _chk(lib.lpco_code_histogram(_p(words, _u32p), d, bits, _p(counts, _u64p)))
    return counts


def huffman_encode(words, d, bits, lens, capacity_words=None):
    """(stream words, total bits) of one packed message under the canonical code of `lens`."""
    words = np.ascontiguousarray(words, np.uint32)
    lens = np.ascontiguousarray(lens, np.int32)
    cap = int(capacity_words) if capacity_words is not None else (int(d) * max(int(lens.max()), 1) + 31) // 32
    out = np.zeros(max(cap, 1), np.uint32)
    total = C.c_uint64()
    _chk(lib.lpco_huffman_encode(_p(words, _u32p), d, bits, _p(lens, _i32p), _p(out, _u32p), cap, C.byref(total)))
    return out[:(total.value + 31) // 32].copy(), total.value


def huffman_decode(stream, total_bits, d, bits, lens):
    stream = np.ascontiguousarray(stream, np.uint32)
    if stream.size == 0:
        stream = np.zeros(1, np.uint32)
    lens = np.ascontiguousarray(lens, np.int32)
    codes = np.zeros(d, np.int32)
    _chk(lib.lpco_huffman_decode(_p(stream, _u32p), total_bits, d, bits, _p(lens, _i32p), _p(codes, _i32p)))
    return codes


def alpc_params(problem, config, epoch):
    t1, t2, a, th = C.c_float(), C.c_float(), C.c_float(), C.c_float()
    _chk(lib.lpco_alpc_params(C.byref(problem), C.byref(config), epoch, C.byref(t1), C.byref(t2), C.byref(a),
                              C.byref(th)))
    return t1.value, t2.value, a.value, th.value


def epoch(problem, config, w_snap, epoch_index, y=None, z=None):
    """In-place on w_snap (and y, z for ALPC); returns the Table 1 bit count of the epoch."""
    assert w_snap.dtype == np.float32 and w_snap.flags.c_contiguous
    bits = C.c_uint64()
    _chk(lib.lpco_epoch(C.byref(problem), C.byref(config), _p(w_snap, _f32p), _p(y, _f32p), _p(z, _f32p),
                        epoch_index, C.byref(bits)))
    return bits.value


def epoch_traced(problem, config, w_snap, epoch_index, y=None, z=None, coded=False):
    """epoch() that also returns (delta_trace, nclip_trace), each [m][N]; with coded=True also the entropy-coded
    size of every message."""
    assert w_snap.dtype == np.float32 and w_snap.flags.c_contiguous
    dtr = np.zeros((config.m, config.N), np.float32)
    ntr = np.zeros((config.m, config.N), np.uint32)
    ctr = np.zeros((config.m, config.N), np.uint64) if coded else None
    _chk(lib.lpco_epoch_traced(C.byref(problem), C.byref(config), _p(w_snap, _f32p), _p(y, _f32p), _p(z, _f32p),
                               epoch_index, _p(dtr, _f32p), _p(ntr, _u32p), _p(ctr, _u64p)))
    return (dtr, ntr, ctr) if coded else (dtr, ntr)


def bits_per_message(d, bits):
    return int(lib.lpco_bits_per_message(d, bits))


def bits_per_iteration(d, bits, N, scheme):
    return int(lib.lpco_bits_per_iteration(d, bits, N, scheme))


def set_threads(n):
    lib.lpco_set_threads(n)
