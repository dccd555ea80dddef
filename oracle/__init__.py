"""LAQ oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

ctypes front end of the plain-C reference in this directory (quantizer,
skip rule, server update and Algorithm 2's loop body, model gradients).  Only
tests, the smoke check and the benchmark's CPU-baseline leg may import it.

Parity pins: see the header of laq_oracle.h.  Unpinned: the upload counts,
curves and accuracies of the paper's Tables 2-3 (need MNIST and an unstated
initialisation).
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblaq_oracle.so")
_SOURCES = ["laq_oracle.c", "laq_models.c"]
B_EXACT = 32

OK, EINVAL, ENONFINITE = 0, 1, 4


def build(force=False):
    """Compile the oracle with gcc (-O2, no contraction, no fast-math)."""
    srcs = [os.path.join(_HERE, s) for s in _SOURCES]
    deps = srcs + [os.path.join(_HERE, "laq_oracle.h")]
    if (not force and os.path.exists(_LIB_PATH)
            and all(os.path.getmtime(_LIB_PATH) >= os.path.getmtime(d) for d in deps)):
        return _LIB_PATH
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC",
           "-shared", "-Wall", "-Wextra", "-o", _LIB_PATH] + srcs + ["-lm"]
    subprocess.check_call(cmd)
    return _LIB_PATH


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB_PATH)
        _declare(_lib)
    return _lib


def _p(a, ctype):
    return None if a is None else a.ctypes.data_as(C.POINTER(ctype))


def _declare(L):
    i32, i64, f32, f64 = C.c_int32, C.c_int64, C.c_float, C.c_double
    pf, pd = C.POINTER(f32), C.POINTER(f64)
    pu32, pu8, pi32, pi64, pu64 = (C.POINTER(C.c_uint32), C.POINTER(C.c_uint8),
                                   C.POINTER(i32), C.POINTER(i64), C.POINTER(C.c_uint64))
    L.laq_oracle_eps_K.restype = i32
    L.laq_oracle_eps_K.argtypes = [i64]
    L.laq_oracle_code_words.restype = i64
    L.laq_oracle_code_words.argtypes = [i64, i32]
    L.laq_oracle_quantize.restype = C.c_int
    L.laq_oracle_quantize.argtypes = [pf, pf, i64, i32, pf, pu32, pf, pf, pi64, pd, pd]
    L.laq_oracle_pack.restype = None
    L.laq_oracle_pack.argtypes = [pu32, i64, i32, pu32, i64]
    L.laq_oracle_unpack.restype = None
    L.laq_oracle_unpack.argtypes = [pu32, i64, i32, pu32]
    L.laq_oracle_dequantize.restype = None
    L.laq_oracle_dequantize.argtypes = [pu32, i64, i32, f32, pf]
    L.laq_oracle_skip.restype = C.c_int
    L.laq_oracle_skip.argtypes = [f64, f64, f64, pd, pd, i32, f32, i32, i32, i32, pd]
    L.laq_oracle_server.restype = f64
    L.laq_oracle_server.argtypes = [pf, pu8, i32, i64, f32, pf, pf]
    L.laq_oracle_iteration.restype = C.c_int
    L.laq_oracle_iteration.argtypes = [i32, i64, i32, i32, pd, i32, f32, pf, pf, pf, pf,
                                       pd, pi32, pd, pu64, pu64, pf, pu32, pu8, pi64,
                                       pd, pd, pd, i32]
    L.laq_oracle_grad_binlog.restype = None
    L.laq_oracle_grad_binlog.argtypes = [pf, pf, pi32, i64, i64, i64, i64, f32, pf, pd]
    L.laq_oracle_grad_softmax.restype = None
    L.laq_oracle_grad_softmax.argtypes = [pf, pf, pi32, i64, i64, i64, i32, i64, f32, pf, pd]
    L.laq_oracle_grad_mlp.restype = None
    L.laq_oracle_grad_mlp.argtypes = [pf, pf, pi32, i64, i64, pi32, i32, i64, f32, pf, pd]
    L.laq_oracle_mlp_params.restype = i64
    L.laq_oracle_mlp_params.argtypes = [pi32, i32]
    L.laq_oracle_grads_all.restype = f64
    L.laq_oracle_grads_all.argtypes = [i32, pf, pf, pi32, i32, i64, i64, pi32, i32, f32, pf]
    L.laq_oracle_grads_minibatch.restype = None
    L.laq_oracle_grads_minibatch.argtypes = [i32, pf, pf, pi32, i32, i64, i64, pi32, i32, f32,
                                             pi32, i64, pf]


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def eps_K(p):
    return int(lib().laq_oracle_eps_K(int(p)))


def code_words(p, b):
    return int(lib().laq_oracle_code_words(int(p), int(b)))


def quantize(g, h, b, want_vectors=True):
    """Innovation quantizer of one worker (Sec. 2.1, eqs. 5-6).

    Returns dict(status, R, q, delta, h_new, Sq, E2, lhs)."""
    g, h = _f32(g), _f32(h)
    p = g.size
    R = C.c_float(0)
    Sq = C.c_int64(0)
    E2 = C.c_double(0)
    lhs = C.c_double(0)
    q = np.zeros(p, np.uint32) if want_vectors else None
    d = np.zeros(p, np.float32) if want_vectors else None
    hn = np.zeros(p, np.float32) if want_vectors else None
    st = lib().laq_oracle_quantize(_p(g, C.c_float), _p(h, C.c_float), p, int(b), C.byref(R),
                                   _p(q, C.c_uint32), _p(d, C.c_float), _p(hn, C.c_float),
                                   C.byref(Sq), C.byref(E2), C.byref(lhs))
    return dict(status=st, R=np.float32(R.value), q=q, delta=d, h_new=hn, Sq=Sq.value,
                E2=E2.value, lhs=lhs.value)


def pack(q, b, n_words=None):
    q = np.ascontiguousarray(q, np.uint32)
    n = code_words(q.size, b) if n_words is None else int(n_words)
    w = np.zeros(n, np.uint32)
    lib().laq_oracle_pack(_p(q, C.c_uint32), q.size, int(b), _p(w, C.c_uint32), n)
    return w


def unpack(words, p, b):
    words = np.ascontiguousarray(words, np.uint32)
    q = np.zeros(p, np.uint32)
    lib().laq_oracle_unpack(_p(words, C.c_uint32), int(p), int(b), _p(q, C.c_uint32))
    return q


def dequantize(q, b, R):
    q = np.ascontiguousarray(q, np.uint32)
    d = np.zeros(q.size, np.float32)
    lib().laq_oracle_dequantize(_p(q, C.c_uint32), q.size, int(b), float(R), _p(d, C.c_float))
    return d


def skip(lhs, E2, Ehat2, xi, dtheta2, alpha, M, t_m, t_bar):
    """Skip rule (eqs. 7a-7b): returns (skip?, rhs)."""
    xi = np.ascontiguousarray(xi, np.float64)
    d2 = np.ascontiguousarray(dtheta2, np.float64)
    rhs = C.c_double(0)
    s = lib().laq_oracle_skip(float(lhs), float(E2), float(Ehat2), _p(xi, C.c_double),
                              _p(d2, C.c_double), xi.size, float(alpha), int(M), int(t_m),
                              int(t_bar), C.byref(rhs))
    return bool(s), rhs.value


def server(delta, upload, alpha, nabla, theta):
    """Server update (eq. 4), in place on nabla/theta; returns alpha^2||nabla||^2."""
    delta = _f32(delta)
    M, p = delta.shape
    up = np.ascontiguousarray(upload, np.uint8)
    assert nabla.dtype == np.float32 and theta.dtype == np.float32
    return lib().laq_oracle_server(_p(delta, C.c_float), _p(up, C.c_uint8), M, p, float(alpha),
                                   _p(nabla, C.c_float), _p(theta, C.c_float))


class State:
    """Everything Algorithm 2 carries from one iteration to the next.

    Initial values (the paper leaves them open): Q_m(theta_hat^0) = 0,
    ||eps_hat||^2 = 0, missing parameter differences = 0, clocks = t_bar so
    that the first iteration is a full round."""

    def __init__(self, M, p, b, D, xi, t_bar, alpha, theta0):
        self.M, self.p, self.b, self.D, self.t_bar = int(M), int(p), int(b), int(D), int(t_bar)
        self.alpha = np.float32(alpha)
        self.xi = np.ascontiguousarray(np.broadcast_to(np.asarray(xi, np.float32), (D,)),
                                       np.float32).astype(np.float64)
        self.H = np.zeros((M, p), np.float32)
        self.nabla = np.zeros(p, np.float32)
        self.theta = np.array(theta0, np.float32, copy=True).reshape(p)
        self.Ehat2 = np.zeros(M, np.float64)
        self.t = np.full(M, t_bar, np.int32)
        self.dtheta2 = np.zeros(D, np.float64)
        self.uploads = np.zeros(M, np.uint64)
        self.bits = C.c_uint64(0)

    def copy(self):
        import copy
        s = copy.copy(self)
        for k in ("H", "nabla", "theta", "Ehat2", "t", "dtheta2", "uploads"):
            setattr(s, k, getattr(self, k).copy())
        s.bits = C.c_uint64(self.bits.value)
        return s

    def iteration(self, G, want_codes=True, force_upload=False):
        """One pass of Algorithm 2's loop body given the fresh gradients G[M][p]."""
        G = _f32(G)
        assert G.shape == (self.M, self.p)
        M, p = self.M, self.p
        out = dict(R=np.zeros(M, np.float32),
                   q=np.zeros((M, p), np.uint32) if want_codes else None,
                   upload=np.zeros(M, np.uint8), Sq=np.zeros(M, np.int64),
                   E2=np.zeros(M, np.float64), lhs=np.zeros(M, np.float64),
                   rhs=np.zeros(M, np.float64))
        st = lib().laq_oracle_iteration(
            M, p, self.b, self.D, _p(self.xi, C.c_double), self.t_bar, float(self.alpha),
            _p(G, C.c_float), _p(self.H, C.c_float), _p(self.nabla, C.c_float),
            _p(self.theta, C.c_float), _p(self.Ehat2, C.c_double), _p(self.t, C.c_int32),
            _p(self.dtheta2, C.c_double), _p(self.uploads, C.c_uint64), C.byref(self.bits),
            _p(out["R"], C.c_float), _p(out["q"], C.c_uint32), _p(out["upload"], C.c_uint8),
            _p(out["Sq"], C.c_int64), _p(out["E2"], C.c_double), _p(out["lhs"], C.c_double),
            _p(out["rhs"], C.c_double), int(bool(force_upload)))
        out["status"] = st
        return out


def mlp_params(dims):
    d = np.ascontiguousarray(dims, np.int32)
    return int(lib().laq_oracle_mlp_params(_p(d, C.c_int32), d.size))


def model_params(kind, dims):
    if kind == 1:
        return int(dims[0])
    if kind == 2:
        return int(dims[0]) * int(dims[1])
    return mlp_params(dims)


def grads_all(kind, theta, X, y, dims, lam):
    """All workers' gradients.  X[M][N_m][ldx] float32, y[M][N_m] int32.
    Returns (G[M][p], global loss)."""
    X = _f32(X)
    y = np.ascontiguousarray(y, np.int32)
    theta = _f32(theta)
    M, N_m, ldx = X.shape
    d = np.ascontiguousarray(dims, np.int32)
    p = model_params(kind, dims)
    assert theta.size == p
    G = np.zeros((M, p), np.float32)
    loss = lib().laq_oracle_grads_all(int(kind), _p(theta, C.c_float), _p(X, C.c_float),
                                      _p(y, C.c_int32), M, N_m, ldx, _p(d, C.c_int32), d.size,
                                      float(lam), _p(G, C.c_float))
    return G, loss


def grads_minibatch(kind, theta, X, y, dims, lam, idx):
    """Minibatch gradients of all workers (SLAQ): idx[M][B] int32 indices into each
    worker's own shard.  Returns G[M][p]."""
    X = _f32(X)
    y = np.ascontiguousarray(y, np.int32)
    theta = _f32(theta)
    idx = np.ascontiguousarray(idx, np.int32)
    M, N_m, ldx = X.shape
    assert idx.shape[0] == M and idx.min() >= 0 and idx.max() < N_m
    d = np.ascontiguousarray(dims, np.int32)
    p = model_params(kind, dims)
    assert theta.size == p
    G = np.zeros((M, p), np.float32)
    lib().laq_oracle_grads_minibatch(int(kind), _p(theta, C.c_float), _p(X, C.c_float),
                                     _p(y, C.c_int32), M, N_m, ldx, _p(d, C.c_int32), d.size,
                                     float(lam), _p(idx, C.c_int32), idx.shape[1],
                                     _p(G, C.c_float))
    return G


def grad_worker(kind, theta, Xm, ym, dims, lam, N_total):
    """One worker's gradient share: Xm[N_m][ldx], ym[N_m]; N_total = samples of all workers."""
    Xm = _f32(Xm)
    ym = np.ascontiguousarray(ym, np.int32)
    theta = _f32(theta)
    N_m, ldx = Xm.shape
    d = np.ascontiguousarray(dims, np.int32)
    g = np.zeros(model_params(kind, dims), np.float32)
    L = lib()
    pf, pi = C.c_float, C.c_int32
    if kind == 1:
        L.laq_oracle_grad_binlog(_p(theta, pf), _p(Xm, pf), _p(ym, pi), N_m, int(dims[0]), ldx,
                                 int(N_total), float(lam), _p(g, pf), None)
    elif kind == 2:
        L.laq_oracle_grad_softmax(_p(theta, pf), _p(Xm, pf), _p(ym, pi), N_m, int(dims[0]), ldx,
                                  int(dims[1]), int(N_total), float(lam), _p(g, pf), None)
    else:
        L.laq_oracle_grad_mlp(_p(theta, pf), _p(Xm, pf), _p(ym, pi), N_m, ldx, _p(d, pi), d.size,
                              int(N_total), float(lam), _p(g, pf), None)
    return g
