"""ctypes binding of include/laq.h (same names, argument marshalling only)."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = os.path.join(_HERE, "liblaq_hip.so")

OK, EINVAL, ESTATE, EDEVICE, ENONFINITE = 0, 1, 2, 3, 4
MODEL_NONE, MODEL_BINLOG, MODEL_SOFTMAX, MODEL_MLP = 0, 1, 2, 3
MODE_FORCE_UPLOAD = 1
B_EXACT = 32          # laq_create's b for the identity quantizer (LAG / GD)

EXPORTS = ["laq_p_stride", "laq_w_stride", "laq_workspace_bytes", "laq_create", "laq_destroy",
           "laq_reset", "laq_set_mode", "laq_set_model", "laq_model_workspace_bytes",
           "laq_set_data", "laq_tiled_data_bytes", "laq_tile_data", "laq_worker_grads", "laq_minibatch_workspace_bytes",
           "laq_worker_grads_minibatch", "laq_quantize_skip", "laq_quantize_skip_noalloc", "laq_radius_handover",
           "laq_server_step",
           "laq_get_state", "laq_get_counters", "laq_last_error"]


class LaqError(RuntimeError):
    pass


class StateView(C.Structure):
    _fields_ = [("H_dev", C.c_void_p), ("nabla_dev", C.c_void_p), ("Ehat2_dev", C.c_void_p),
                ("t_dev", C.c_void_p), ("dtheta2_dev", C.c_void_p), ("Sq_dev", C.c_void_p),
                ("E2_dev", C.c_void_p), ("lhs_dev", C.c_void_p), ("rhs_dev", C.c_void_p),
                ("uploads_dev", C.c_void_p), ("bits_dev", C.c_void_p), ("status_dev", C.c_void_p),
                ("p_stride", C.c_int64), ("w_stride", C.c_int64)]


def lib_path():
    return _LIB


_lib = None


def lib():
    """Loads the built library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            raise LaqError(f"{_LIB} is missing: build it with `python -m paper_1909_07588_amd.build` "
                           "(or __graft_entry__.build()); there is no CPU fallback")
        L = C.CDLL(_LIB)
        i32, i64, vp, sz, f32 = C.c_int32, C.c_int64, C.c_void_p, C.c_size_t, C.c_float
        L.laq_p_stride.restype = i64
        L.laq_p_stride.argtypes = [i64]
        L.laq_w_stride.restype = i64
        L.laq_w_stride.argtypes = [i64, i32]
        L.laq_workspace_bytes.restype = sz
        L.laq_workspace_bytes.argtypes = [i32, i64, i32, i32]
        L.laq_create.restype = C.c_int
        L.laq_create.argtypes = [C.POINTER(vp), i32, i64, i32, i32, C.POINTER(f32), i32, f32, vp, sz, vp]
        L.laq_destroy.restype = C.c_int
        L.laq_destroy.argtypes = [vp]
        L.laq_reset.restype = C.c_int
        L.laq_reset.argtypes = [vp]
        L.laq_set_mode.restype = C.c_int
        L.laq_set_mode.argtypes = [vp, C.c_uint32]
        L.laq_set_model.restype = C.c_int
        L.laq_set_model.argtypes = [vp, i32, C.POINTER(i32), i32, f32]
        L.laq_model_workspace_bytes.restype = sz
        L.laq_model_workspace_bytes.argtypes = [vp, i64]
        L.laq_set_data.restype = C.c_int
        L.laq_set_data.argtypes = [vp, vp, vp, i64, i64, vp, sz]
        L.laq_tiled_data_bytes.restype = sz
        L.laq_tiled_data_bytes.argtypes = [vp]
        L.laq_tile_data.restype = C.c_int
        L.laq_tile_data.argtypes = [vp, vp, sz]
        L.laq_worker_grads.restype = C.c_int
        L.laq_worker_grads.argtypes = [vp, vp, vp]
        L.laq_minibatch_workspace_bytes.restype = sz
        L.laq_minibatch_workspace_bytes.argtypes = [vp, i64]
        L.laq_worker_grads_minibatch.restype = C.c_int
        L.laq_worker_grads_minibatch.argtypes = [vp, vp, vp, i64, vp, sz, vp]
        L.laq_quantize_skip.restype = C.c_int
        L.laq_quantize_skip.argtypes = [vp, vp, vp, vp, vp]
        L.laq_quantize_skip_noalloc.restype = C.c_int
        L.laq_quantize_skip_noalloc.argtypes = [vp, vp, vp, vp, vp]
        L.laq_radius_handover.restype = C.c_int
        L.laq_radius_handover.argtypes = [vp, vp, vp, C.c_int32]
        L.laq_server_step.restype = C.c_int
        L.laq_server_step.argtypes = [vp, vp, vp, vp, vp]
        L.laq_get_state.restype = C.c_int
        L.laq_get_state.argtypes = [vp, C.POINTER(StateView)]
        L.laq_get_counters.restype = C.c_int
        L.laq_get_counters.argtypes = [vp, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
        L.laq_last_error.restype = C.c_char_p
        L.laq_last_error.argtypes = [vp]
        _lib = L
    return _lib


def p_stride(p):
    return int(lib().laq_p_stride(int(p)))


def w_stride(p, b):
    return int(lib().laq_w_stride(int(p), int(b)))


class Laq:
    """One LAQ context: the C calls of include/laq.h with torch tensors as buffers."""

    def __init__(self, M, p, b, D, xi, t_bar, alpha, device="cuda:0", stream=None):
        import torch
        self.torch = torch
        self.L = lib()
        self.M, self.p, self.b, self.D, self.t_bar = int(M), int(p), int(b), int(D), int(t_bar)
        self.alpha = float(alpha)
        self.device = torch.device(device)
        self.p_stride = p_stride(p)
        self.w_stride = w_stride(p, b)
        xi_arr = np.ascontiguousarray(np.broadcast_to(np.asarray(xi, np.float32), (self.D,)), np.float32)
        nbytes = int(self.L.laq_workspace_bytes(self.M, self.p, self.b, self.D))
        if nbytes == 0:
            raise LaqError("laq_workspace_bytes: invalid sizes")
        self.ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        self._ws_off = (-self.ws.data_ptr()) % 256
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        st = self.L.laq_create(C.byref(h), self.M, self.p, self.b, self.D,
                               xi_arr.ctypes.data_as(C.POINTER(C.c_float)), self.t_bar, self.alpha,
                               C.c_void_p(self.ws.data_ptr() + self._ws_off), nbytes,
                               C.c_void_p(self.stream.cuda_stream))
        if st != OK:
            raise LaqError(f"laq_create failed with status {st}")
        self.h = h
        self._model_ws = None
        self._keep = []
        v = StateView()
        self._chk(self.L.laq_get_state(self.h, C.byref(v)))
        self._view = v

    # -- helpers ------------------------------------------------------------------
    def _chk(self, st):
        if st != OK:
            msg = self.L.laq_last_error(self.h).decode()
            raise LaqError(f"status {st}: {msg}")

    def close(self):
        if getattr(self, "h", None):
            self.L.laq_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ws_tensor(self, ptr, count, dtype):
        """Typed view of a region of the workspace given its device address."""
        torch = self.torch
        off = ptr - self.ws.data_ptr()
        nbytes = count * torch.empty(0, dtype=dtype).element_size()
        return self.ws[off:off + nbytes].view(dtype)

    def state(self):
        """Views (not copies) of the state held in the workspace.  Goes through
        laq_get_state every time: the call tells the library that the state may
        be overwritten, so a radius handed over by laq_worker_grads is dropped."""
        v = StateView()
        self._chk(self.L.laq_get_state(self.h, C.byref(v)))
        self._view = v
        torch = self.torch
        M, D = self.M, self.D
        return dict(
            H=self._ws_tensor(v.H_dev, M * self.p_stride, torch.float32).view(M, self.p_stride),
            nabla=self._ws_tensor(v.nabla_dev, self.p_stride, torch.float32),
            Ehat2=self._ws_tensor(v.Ehat2_dev, M, torch.float64),
            t=self._ws_tensor(v.t_dev, M, torch.int32),
            dtheta2=self._ws_tensor(v.dtheta2_dev, D, torch.float64),
            Sq=self._ws_tensor(v.Sq_dev, M, torch.int64),
            E2=self._ws_tensor(v.E2_dev, M, torch.float64),
            lhs=self._ws_tensor(v.lhs_dev, M, torch.float64),
            rhs=self._ws_tensor(v.rhs_dev, M, torch.float64),
            uploads=self._ws_tensor(v.uploads_dev, M, torch.int64),
            bits=self._ws_tensor(v.bits_dev, 1, torch.int64),
            status=self._ws_tensor(v.status_dev, 1, torch.int32))

    # -- buffers the caller owns ---------------------------------------------------
    def alloc_G(self):
        return self.torch.zeros((self.M, self.p_stride), dtype=self.torch.float32, device=self.device)

    def alloc_messages(self):
        t = self.torch
        return (t.zeros((self.M, self.w_stride), dtype=t.int32, device=self.device),
                t.zeros(self.M, dtype=t.float32, device=self.device),
                t.zeros(self.M, dtype=t.uint8, device=self.device))

    # -- the C calls ---------------------------------------------------------------
    def laq_reset(self):
        self._chk(self.L.laq_reset(self.h))

    def laq_set_mode(self, flags):
        self._chk(self.L.laq_set_mode(self.h, int(flags)))

    def laq_set_model(self, kind, dims, lam):
        d = np.ascontiguousarray(dims, np.int32)
        self._chk(self.L.laq_set_model(self.h, int(kind), d.ctypes.data_as(C.POINTER(C.c_int32)),
                                       d.size, float(lam)))

    def laq_set_data(self, X, y):
        """X[M][N_m][ldx] float32, y[M][N_m] int32, both device tensors (kept alive here)."""
        torch = self.torch
        assert X.dtype == torch.float32 and y.dtype == torch.int32 and X.is_contiguous() and y.is_contiguous()
        M, N_m, ldx = X.shape
        assert M == self.M and tuple(y.shape) == (M, N_m)
        need = int(self.L.laq_model_workspace_bytes(self.h, N_m))
        self._model_ws = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
        off = (-self._model_ws.data_ptr()) % 256
        self._keep = [X, y]
        self._chk(self.L.laq_set_data(self.h, C.c_void_p(X.data_ptr()), C.c_void_p(y.data_ptr()), N_m, ldx,
                                      C.c_void_p(self._model_ws.data_ptr() + off), need))

    def laq_tiled_data_bytes(self):
        return int(self.L.laq_tiled_data_bytes(self.h))

    def laq_tile_data(self):
        """Allocates the tiled copy of the bound X (kept alive here) and hands it to the library."""
        need = self.laq_tiled_data_bytes()
        if need == 0:
            raise LaqError("laq_tile_data: the bound model and data have no kernel that reads tiles")
        self._tiled = self.torch.empty(need + 256, dtype=self.torch.uint8, device=self.device)
        off = (-self._tiled.data_ptr()) % 256
        self._chk(self.L.laq_tile_data(self.h, C.c_void_p(self._tiled.data_ptr() + off), need))

    def laq_worker_grads(self, theta, G):
        self._chk(self.L.laq_worker_grads(self.h, C.c_void_p(theta.data_ptr()), C.c_void_p(G.data_ptr())))

    def laq_worker_grads_minibatch(self, theta, idx, G):
        """idx[M][B] int32 device tensor of sample indices into each worker's shard."""
        torch = self.torch
        assert idx.dtype == torch.int32 and idx.is_contiguous() and idx.shape[0] == self.M
        B = int(idx.shape[1])
        need = int(self.L.laq_minibatch_workspace_bytes(self.h, B))
        ws = getattr(self, "_mb_ws", None)
        if ws is None or ws.numel() < need + 256:
            ws = self._mb_ws = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
        off = (-ws.data_ptr()) % 256
        self._chk(self.L.laq_worker_grads_minibatch(self.h, C.c_void_p(theta.data_ptr()),
                                                    C.c_void_p(idx.data_ptr()), B,
                                                    C.c_void_p(ws.data_ptr() + off), need,
                                                    C.c_void_p(G.data_ptr())))

    def laq_quantize_skip(self, G, codes, R, upload):
        self._chk(self.L.laq_quantize_skip(self.h, C.c_void_p(G.data_ptr()), C.c_void_p(codes.data_ptr()),
                                           C.c_void_p(R.data_ptr()), C.c_void_p(upload.data_ptr())))

    def laq_quantize_skip_noalloc(self, G, codes, R, upload):
        self._chk(self.L.laq_quantize_skip_noalloc(self.h, C.c_void_p(G.data_ptr()), C.c_void_p(codes.data_ptr()),
                                                   C.c_void_p(R.data_ptr()), C.c_void_p(upload.data_ptr())))

    def laq_radius_handover(self, G, rmax):
        """rmax: uint32 (or int32) device tensor [M][count], raw bits of block maxima of |g - h|;
        the caller keeps it alive until the next laq_quantize_skip has run.  rmax = None withdraws
        a hand-over (count = 0)."""
        if rmax is None:
            self._chk(self.L.laq_radius_handover(self.h, None, None, 0))
            return
        assert rmax.dim() == 2 and rmax.shape[0] == self.M and rmax.is_contiguous() and rmax.element_size() == 4
        self._chk(self.L.laq_radius_handover(self.h, C.c_void_p(G.data_ptr()), C.c_void_p(rmax.data_ptr()),
                                             int(rmax.shape[1])))

    def laq_server_step(self, codes, R, upload, theta):
        self._chk(self.L.laq_server_step(self.h, C.c_void_p(codes.data_ptr()), C.c_void_p(R.data_ptr()),
                                         C.c_void_p(upload.data_ptr()), C.c_void_p(theta.data_ptr())))

    def laq_get_counters(self):
        up = (C.c_uint64 * self.M)()
        bits = C.c_uint64(0)
        st = self.L.laq_get_counters(self.h, up, C.byref(bits))
        if st not in (OK, ENONFINITE, EINVAL):
            self._chk(st)
        return np.array(list(up), np.uint64), int(bits.value), st
