"""ctypes binding of the CPU oracle (oracle/cnn_oracle.cpp).  Test infrastructure only."""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None

KIND_INPUT, KIND_CONV, KIND_POOL, KIND_FC = 0, 1, 2, 3
E_SYNTAX, E_SHAPE, E_ARG = -1, -2, -3


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__("oracle: %s failed with code %d" % (what, code))
        self.code = code


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.oracle_num_weights.restype = C.c_size_t
        L.oracle_image_size.restype = C.c_size_t
        L.oracle_op_act.restype = C.c_double
        L.oracle_op_act.argtypes = [C.c_double]
        L.oracle_op_act_deriv_from_output.restype = C.c_double
        L.oracle_op_act_deriv_from_output.argtypes = [C.c_double]
        L.oracle_op_softmax_xent.restype = C.c_double
        L.oracle_op_tanh_sqerr.restype = C.c_double
        L.oracle_set_output_units.argtypes = [C.c_void_p, C.c_int]
        L.oracle_train_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_double, C.c_void_p]
        L.oracle_backward_update.argtypes = [C.c_void_p, C.c_int32, C.c_double, C.c_void_p]
        L.oracle_adopt_argmax_hint.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_double,
                                               C.c_void_p, C.c_void_p]
        L.oracle_train_many.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_double]
        L.oracle_forward_many.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.oracle_set_weights.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        L.oracle_get_weights.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        for name in ("oracle_forward", "oracle_gradients", "oracle_loss", "oracle_get_activation",
                     "oracle_get_delta", "oracle_get_argmax", "oracle_layer_info",
                     "oracle_set_connection_table", "oracle_set_fixed_frontend"):
            getattr(L, name).restype = C.c_int
        L.oracle_destroy.argtypes = [C.c_void_p]
        L.oracle_destroy.restype = None
        _lib = L
    return _lib


def conv_out_size(m_prev, k, s):
    return lib().oracle_conv_out_size(int(m_prev), int(k), int(s))


def set_threads(n):
    return lib().oracle_set_threads(int(n))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


class Oracle:
    """One network held by the oracle.  precision=64 is the truth, 32 only for timing."""

    def __init__(self, arch, precision=64):
        self._h = C.c_void_p()
        rc = lib().oracle_create(arch.encode(), int(precision), C.byref(self._h))
        if rc:
            raise OracleError(rc, "create(%r)" % arch)
        self.arch = arch

    def __del__(self):
        if getattr(self, "_h", None) and self._h.value:
            lib().oracle_destroy(self._h)
            self._h = C.c_void_p()

    def _ck(self, rc, what):
        if rc:
            raise OracleError(rc, what)

    def set_connection_table(self, conv_index, table):
        t = np.ascontiguousarray(table, dtype=np.uint8)
        self._ck(lib().oracle_set_connection_table(self._h, int(conv_index), _p(t, C.c_uint8)),
                 "set_connection_table")

    def set_output_units(self, kind):
        """0: soft-max + cross-entropy (default); 1: scaled tanh + squared error, targets +-1."""
        self._ck(lib().oracle_set_output_units(self._h, int(kind)), "set_output_units")

    def set_fixed_frontend(self, filters, src_channel, n_src_channels):
        f = _f32(filters)
        s = np.ascontiguousarray(src_channel, dtype=np.int32)
        self._ck(lib().oracle_set_fixed_frontend(self._h, int(f.shape[0]), int(f.shape[-1]),
                                                 int(n_src_channels), _p(f, C.c_float),
                                                 _p(s, C.c_int32)), "set_fixed_frontend")

    @property
    def num_weights(self):
        return int(lib().oracle_num_weights(self._h))

    @property
    def num_layers(self):
        return int(lib().oracle_num_layers(self._h))

    @property
    def image_size(self):
        return int(lib().oracle_image_size(self._h))

    def layer_info(self, layer):
        info = np.zeros(8, dtype=np.int32)
        self._ck(lib().oracle_layer_info(self._h, int(layer), _p(info, C.c_int32)), "layer_info")
        return dict(kind=int(info[0]), maps=int(info[1]), h=int(info[2]), w=int(info[3]),
                    K=int(info[4]), S=int(info[5]), Kx=int(info[6]), Sx=int(info[7]))

    def layer_size(self, layer):
        i = self.layer_info(layer)
        return i["maps"] * i["h"] * i["w"]

    def set_weights(self, w):
        w = _f64(w)
        self._ck(lib().oracle_set_weights(self._h, w.ctypes.data, w.size), "set_weights")

    def get_weights(self):
        w = np.empty(self.num_weights, dtype=np.float64)
        self._ck(lib().oracle_get_weights(self._h, w.ctypes.data, w.size), "get_weights")
        return w

    def forward(self, image):
        img = _f32(image).ravel()
        assert img.size == self.image_size
        probs = np.empty(self.layer_size(self.num_layers - 1), dtype=np.float64)
        self._ck(lib().oracle_forward(self._h, _p(img, C.c_float), _p(probs, C.c_double)), "forward")
        return probs

    def train_step(self, image, label, lr):
        img = _f32(image).ravel()
        assert img.size == self.image_size
        loss = C.c_double()
        self._ck(lib().oracle_train_step(self._h, img.ctypes.data, int(label), float(lr),
                                         C.addressof(loss)), "train_step")
        return loss.value

    def adopt_argmax_hint(self, layer, hint, tol):
        """After forward(): take another implementation's pooling winners where the choice is a
        near-tie (gap <= tol * max|input|).  Returns (adopted, rejected)."""
        hint = np.ascontiguousarray(hint, dtype=np.uint8)
        assert hint.size == self.layer_size(layer)
        a, r = C.c_int(), C.c_int()
        self._ck(lib().oracle_adopt_argmax_hint(self._h, int(layer), hint.ctypes.data, float(tol),
                                                C.addressof(a), C.addressof(r)), "adopt_argmax_hint")
        return a.value, r.value

    def backward_update(self, label, lr):
        """After forward(): the backward pass and the SGD update of one on-line step."""
        loss = C.c_double()
        self._ck(lib().oracle_backward_update(self._h, int(label), float(lr), C.addressof(loss)),
                 "backward_update")
        return loss.value

    def train_many(self, images, labels, lr):
        imgs = _f32(images)
        labs = np.ascontiguousarray(labels, dtype=np.int32)
        assert imgs.size == self.image_size * labs.size
        self._ck(lib().oracle_train_many(self._h, imgs.ctypes.data, labs.ctypes.data, labs.size,
                                         float(lr)), "train_many")

    def forward_many(self, images, n):
        imgs = _f32(images)
        assert imgs.size == self.image_size * n
        nc = self.layer_size(self.num_layers - 1)
        probs = np.empty((n, nc), dtype=np.float64)
        self._ck(lib().oracle_forward_many(self._h, imgs.ctypes.data, n, probs.ctypes.data),
                 "forward_many")
        return probs

    def gradients(self, image, label):
        img = _f32(image).ravel()
        g = np.empty(self.num_weights, dtype=np.float64)
        loss = C.c_double()
        self._ck(lib().oracle_gradients(self._h, _p(img, C.c_float), C.c_int32(int(label)),
                                        _p(g, C.c_double), C.byref(loss)), "gradients")
        return g, loss.value

    def loss(self, image, label):
        img = _f32(image).ravel()
        loss = C.c_double()
        self._ck(lib().oracle_loss(self._h, _p(img, C.c_float), C.c_int32(int(label)),
                                   C.byref(loss)), "loss")
        return loss.value

    def activation(self, layer):
        i = self.layer_info(layer)
        a = np.empty((i["maps"], i["h"], i["w"]), dtype=np.float64)
        self._ck(lib().oracle_get_activation(self._h, int(layer), _p(a, C.c_double)), "activation")
        return a

    def delta(self, layer):
        i = self.layer_info(layer)
        a = np.empty((i["maps"], i["h"], i["w"]), dtype=np.float64)
        self._ck(lib().oracle_get_delta(self._h, int(layer), _p(a, C.c_double)), "delta")
        return a

    def argmax(self, layer):
        i = self.layer_info(layer)
        a = np.empty((i["maps"], i["h"], i["w"]), dtype=np.uint8)
        self._ck(lib().oracle_get_argmax(self._h, int(layer), _p(a, C.c_uint8)), "argmax")
        return a


class _Ops:
    """Single-operation entry points (double precision)."""

    @staticmethod
    def _table(table):
        if table is None:
            return None, None
        t = np.ascontiguousarray(table, dtype=np.uint8)
        return t, _p(t, C.c_uint8)

    def conv_forward(self, x, bias, w, mo, ky, kx, sy=0, sx=0, table=None, apply_act=True):
        x = _f64(x)
        mi, hi, wi = x.shape
        w = _f64(w)
        ho, wo = conv_out_size(hi, ky, sy), conv_out_size(wi, kx, sx)
        out = np.empty((mo, ho, wo), dtype=np.float64)
        b = None if bias is None else _f64(bias)
        t, tp = self._table(table)
        rc = lib().oracle_op_conv_forward(_p(x, C.c_double), mi, hi, wi,
                                          None if b is None else _p(b, C.c_double),
                                          _p(w, C.c_double), tp, mo, ky, kx, sy, sx,
                                          int(bool(apply_act)), _p(out, C.c_double))
        if rc:
            raise OracleError(rc, "op_conv_forward")
        return out

    def maxpool_forward(self, x, ky, kx):
        x = _f64(x)
        m, hi, wi = x.shape
        if hi % ky or wi % kx:
            raise OracleError(E_SHAPE, "op_maxpool_forward")
        out = np.empty((m, hi // ky, wi // kx), dtype=np.float64)
        arg = np.empty((m, hi // ky, wi // kx), dtype=np.uint8)
        rc = lib().oracle_op_maxpool_forward(_p(x, C.c_double), m, hi, wi, ky, kx,
                                             _p(out, C.c_double), _p(arg, C.c_uint8))
        if rc:
            raise OracleError(rc, "op_maxpool_forward")
        return out, arg

    def maxpool_backward(self, g_out, arg, hi, wi, ky, kx):
        g_out = _f64(g_out)
        arg = np.ascontiguousarray(arg, dtype=np.uint8)
        m = g_out.shape[0]
        g_in = np.empty((m, hi, wi), dtype=np.float64)
        rc = lib().oracle_op_maxpool_backward(_p(g_out, C.c_double), _p(arg, C.c_uint8), m, hi, wi,
                                              ky, kx, _p(g_in, C.c_double))
        if rc:
            raise OracleError(rc, "op_maxpool_backward")
        return g_in

    def conv_backward(self, delta, w, mi, hi, wi, ky, kx, sy=0, sx=0, table=None, push=False):
        delta = _f64(delta)
        w = _f64(w)
        mo = delta.shape[0]
        g_in = np.empty((mi, hi, wi), dtype=np.float64)
        t, tp = self._table(table)
        rc = lib().oracle_op_conv_backward(_p(delta, C.c_double), _p(w, C.c_double), tp, mo, mi, hi,
                                           wi, ky, kx, sy, sx, int(bool(push)), _p(g_in, C.c_double))
        if rc:
            raise OracleError(rc, "op_conv_backward")
        return g_in

    def conv_weight_grad(self, delta, x, ky, kx, sy=0, sx=0, table=None):
        delta = _f64(delta)
        x = _f64(x)
        mo = delta.shape[0]
        mi, hi, wi = x.shape
        t, tp = self._table(table)
        n_conn = int(t.sum()) if t is not None else mo * mi
        gb = np.empty(mo, dtype=np.float64)
        gw = np.empty((n_conn, ky, kx), dtype=np.float64)
        rc = lib().oracle_op_conv_weight_grad(_p(delta, C.c_double), _p(x, C.c_double), tp, mo, mi,
                                              hi, wi, ky, kx, sy, sx, _p(gb, C.c_double),
                                              _p(gw, C.c_double))
        if rc:
            raise OracleError(rc, "op_conv_weight_grad")
        return gb, gw

    def fc_forward(self, v, bias, w):
        v = _f64(v).ravel()
        w = _f64(w)
        b = _f64(bias)
        a = np.empty(w.shape[0], dtype=np.float64)
        lib().oracle_op_fc_forward(_p(v, C.c_double), v.size, _p(b, C.c_double), _p(w, C.c_double),
                                   w.shape[0], _p(a, C.c_double))
        return a

    def act(self, a):
        return lib().oracle_op_act(float(a))

    def act_deriv_from_output(self, y):
        return lib().oracle_op_act_deriv_from_output(float(y))

    def softmax_xent(self, a, label):
        a = _f64(a)
        p = np.empty_like(a)
        d = np.empty_like(a)
        e = lib().oracle_op_softmax_xent(_p(a, C.c_double), a.size, int(label), _p(p, C.c_double),
                                         _p(d, C.c_double))
        return e, p, d

    def tanh_sqerr(self, a, label):
        a = _f64(a)
        y = np.empty_like(a)
        d = np.empty_like(a)
        e = lib().oracle_op_tanh_sqerr(_p(a, C.c_double), a.size, int(label), _p(y, C.c_double),
                                       _p(d, C.c_double))
        return e, y, d


ops = _Ops()
OUT_SOFTMAX_XENT, OUT_TANH_SQERR = 0, 1
