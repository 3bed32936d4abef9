"""ctypes access to the CPU oracle (test infrastructure only; see gan_oracle.h).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this.
Nothing here computes: it marshals numpy arrays to the C functions.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBS = {np.float64: os.path.join(_HERE, "liboracle_f64.so"), np.float32: os.path.join(_HERE, "liboracle_f32.so")}
MAX_LAYERS = 8


def build(force=False, real=None):
    """Compile gan_oracle.c next to its source: the double-precision oracle, and the same loops in single
    precision (used only to measure how far plain fp32 arithmetic drifts from the fp64 result)."""
    src = os.path.join(_HERE, "gan_oracle.c")
    hdr = os.path.join(_HERE, "gan_oracle.h")
    for dt, path in _LIBS.items():
        if real is not None and dt is not real:
            continue
        if (not force and os.path.exists(path)
                and os.path.getmtime(path) >= max(os.path.getmtime(src), os.path.getmtime(hdr))):
            continue
        cmd = ["gcc", "-O3", "-march=native", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-DORACLE_REAL=" + ("double" if dt is np.float64 else "float"), "-o", path, src, "-lm"]
        subprocess.check_call(cmd)
    return _LIBS[np.float64]


class Config(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("n_models", C.c_int32), ("n_labels", C.c_int32),
        ("cond_g", C.c_int32), ("cond_d", C.c_int32), ("z_dim", C.c_int32),
        ("img_c", C.c_int32), ("img_hw", C.c_int32), ("g_h0", C.c_int32),
        ("n_g", C.c_int32), ("g_ch", C.c_int32 * MAX_LAYERS),
        ("n_d", C.c_int32), ("d_ch", C.c_int32 * MAX_LAYERS),
        ("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("adam_eps", C.c_double),
        ("bn_eps", C.c_double), ("bn_momentum", C.c_double), ("leaky_slope", C.c_double),
        ("d_loss_scale", C.c_double), ("g_loss_scale", C.c_double),
    ]


_loaded = {}
_I = C.POINTER(C.c_int32)


def lib(real=np.float64):
    if real not in _loaded:
        build(real=real)
        _lib = C.CDLL(_LIBS[real])
        creal = C.c_double if real is np.float64 else C.c_float
        _D = C.POINTER(creal)
        _lib.oracle_param_count.restype = C.c_int64
        _lib.oracle_bn_count.restype = C.c_int64
        _lib.oracle_logistic_loss.restype = creal
        _lib.oracle_logistic_loss.argtypes = [_D, C.c_int, C.c_int, creal, _D]
        _lib.oracle_adam.argtypes = [_D, _D, _D, _D, C.c_int64, C.c_int64] + [creal] * 4
        _lib.oracle_bn_train.argtypes = [_D, _D, _D, creal, _D, _D, _D, C.c_int, C.c_int, C.c_int]
        _lib.oracle_bn_eval.argtypes = [_D, _D, _D, creal, _D, _D, _D, C.c_int, C.c_int, C.c_int]
        _lib.oracle_bn_bwd.argtypes = [_D, _D, _D, _D, creal, _D, _D, _D, _D, C.c_int, C.c_int, C.c_int]
        _lib.oracle_bn_running_update.argtypes = [_D, _D, _D, _D, creal, C.c_int, C.c_int64]
        _lib.oracle_leaky_relu.argtypes = [_D, _D, C.c_int64, creal]
        _lib.oracle_leaky_relu_bwd.argtypes = [_D, _D, _D, C.c_int64, creal]
        _lib.oracle_tanh.argtypes = [_D, _D, C.c_int64]
        _lib.oracle_tanh_bwd.argtypes = [_D, _D, _D, C.c_int64]
        conv_args = [_D, _D, _D, _D] + [C.c_int] * 8
        bwd_args = [_D, _D, _D, _D, _D, _D] + [C.c_int] * 8
        _lib.oracle_conv2d.argtypes = conv_args
        _lib.oracle_conv_transpose2d.argtypes = conv_args
        _lib.oracle_conv2d_bwd.argtypes = bwd_args
        _lib.oracle_conv_transpose2d_bwd.argtypes = bwd_args
        _lib.oracle_linear.argtypes = [_D, _D, _D, _D, C.c_int, C.c_int, C.c_int]
        _lib.oracle_linear_bwd.argtypes = [_D, _D, _D, _D, _D, _D, C.c_int, C.c_int, C.c_int]
        _lib.oracle_route.argtypes = [_I, C.c_int, C.c_int, C.c_int, _I, _I, _I]
        _lib.oracle_create.argtypes = [C.POINTER(Config), C.POINTER(C.c_void_p)]
        _lib.oracle_destroy.argtypes = [C.c_void_p]
        _lib.oracle_param_count.argtypes = [C.c_void_p, C.c_int]
        _lib.oracle_bn_count.argtypes = [C.c_void_p, C.c_int]
        _lib.oracle_get_params.argtypes = [C.c_void_p, C.c_int, C.c_int, _D]
        _lib.oracle_set_params.argtypes = [C.c_void_p, C.c_int, C.c_int, _D]
        _lib.oracle_get_grads.argtypes = [C.c_void_p, C.c_int, C.c_int, _D]
        _lib.oracle_get_opt_state.argtypes = [C.c_void_p, C.c_int, C.c_int, _D, _D, C.POINTER(C.c_int64)]
        _lib.oracle_set_opt_state.argtypes = [C.c_void_p, C.c_int, C.c_int, _D, _D, C.c_int64]
        _lib.oracle_set_bn_running.argtypes = [C.c_void_p, C.c_int, C.c_int, _D, _D]
        _lib.oracle_get_bn_running.argtypes = [C.c_void_p, C.c_int, C.c_int, _D, _D]
        _lib.oracle_train_step.argtypes = [C.c_void_p, _I, _D, _D, C.c_int32, C.c_int32]
        _lib.oracle_generate.argtypes = [C.c_void_p, _I, _D, C.c_int32, _D, C.c_int32, C.c_int32]
        _lib.oracle_get_losses.argtypes = [C.c_void_p, _D, _D, _I]
        _F32 = C.POINTER(C.c_float)
        _F64 = C.POINTER(C.c_double)
        _lib.oracle_draw_labels.argtypes = [_F64, C.c_int, _F32, C.c_int, _I]
        _lib.oracle_sample.argtypes = [C.c_void_p, _F64, _F32, _D, C.c_int32, _D, _I, C.c_int32]
        _lib.oracle_anova_f.argtypes = [_I, _F32, C.c_int, C.c_int, C.c_int, C.c_int, _F64]
        _lib.oracle_get_routing.argtypes = [C.c_void_p, _I, _I]
        _lib.oracle_eval_losses.argtypes = [C.c_void_p, C.c_int, _I, _D, _D, C.c_int32, _D, _D]
        _lib.oracle_eval_grads.argtypes = [C.c_void_p, C.c_int, _I, _D, _D, C.c_int32, _D, _D]
        _lib.oracle_set_bf16_emulation.argtypes = [C.c_void_p, C.c_int]
        _lib.oracle_round_bf16.argtypes = [creal]
        _lib.oracle_round_bf16.restype = creal
        _loaded[real] = _lib
    return _loaded[real]


def _d(a):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(C.c_double if a.dtype == np.float64 else C.c_float))


def _i(a):
    return None if a is None else a.ctypes.data_as(_I)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def make_config(spec, n_models, n_labels, hyper=None):
    """spec: dict with cond_g, cond_d, z_dim, img_c, img_hw, g_h0, g_ch, d_ch."""
    h = dict(lr=2e-4, beta1=0.5, beta2=0.999, adam_eps=1e-8, bn_eps=1e-5, bn_momentum=0.1,
             leaky_slope=0.2, d_loss_scale=0.5, g_loss_scale=0.5)
    h.update(hyper or {})
    c = Config()
    c.struct_size = C.sizeof(Config)
    c.n_models, c.n_labels = n_models, n_labels
    c.cond_g, c.cond_d, c.z_dim = spec["cond_g"], spec["cond_d"], spec["z_dim"]
    c.img_c, c.img_hw, c.g_h0 = spec["img_c"], spec["img_hw"], spec["g_h0"]
    c.n_g = len(spec["g_ch"])
    for i, v in enumerate(spec["g_ch"]):
        c.g_ch[i] = v
    c.n_d = len(spec["d_ch"])
    for i, v in enumerate(spec["d_ch"]):
        c.d_ch[i] = v
    for k, v in h.items():
        setattr(c, k, v)
    return c


class Oracle:
    def __init__(self, spec, n_models, n_labels, hyper=None, real=np.float64, emulate_bf16=False):
        """real=np.float64 is the oracle; np.float32 runs the same loops in single precision.
        emulate_bf16: round the tensors a 16-bit-storage implementation stores (see gan_oracle.h); a diagnostic
        reference next to the plain algorithm, never its replacement."""
        self.real = real
        self.L = lib(real)
        self.cfg = make_config(spec, n_models, n_labels, hyper)
        self.h = C.c_void_p()
        rc = self.L.oracle_create(C.byref(self.cfg), C.byref(self.h))
        if rc != 0:
            raise ValueError("oracle_create failed: %d" % rc)
        self.n_models = n_models
        self.img_shape = (spec["img_c"], spec["img_hw"], spec["img_hw"])
        if emulate_bf16:
            assert self.L.oracle_set_bf16_emulation(self.h, 1) == 0

    def close(self):
        if self.h:
            self.L.oracle_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def param_count(self, which):
        return int(self.L.oracle_param_count(self.h, which))

    def bn_count(self, which):
        return int(self.L.oracle_bn_count(self.h, which))

    def get_params(self, which, model):
        out = np.empty(self.param_count(which), self.real)
        assert self.L.oracle_get_params(self.h, which, model, _d(out)) == 0
        return out

    def set_params(self, which, model, src):
        src = np.ascontiguousarray(src, self.real)
        assert src.size == self.param_count(which)
        assert self.L.oracle_set_params(self.h, which, model, _d(src)) == 0

    def get_grads(self, which, model):
        out = np.empty(self.param_count(which), self.real)
        assert self.L.oracle_get_grads(self.h, which, model, _d(out)) == 0
        return out

    def get_opt_state(self, which, model):
        P = self.param_count(which)
        m, v, t = np.empty(P, self.real), np.empty(P, self.real), C.c_int64()
        assert self.L.oracle_get_opt_state(self.h, which, model, _d(m), _d(v), C.byref(t)) == 0
        return m, v, t.value

    def set_opt_state(self, which, model, m, v, t):
        m, v = np.ascontiguousarray(m, self.real), np.ascontiguousarray(v, self.real)
        assert self.L.oracle_set_opt_state(self.h, which, model, _d(m), _d(v), int(t)) == 0

    def set_bn_running(self, which, model, mean, var):
        mean, var = np.ascontiguousarray(mean, self.real), np.ascontiguousarray(var, self.real)
        assert self.L.oracle_set_bn_running(self.h, which, model, _d(mean), _d(var)) == 0

    def get_state(self, model):
        """Everything a step of one model starts from: per network (params, m, v, t, running mean, running var)."""
        return [(self.get_params(w, model),) + self.get_opt_state(w, model) + self.get_bn_running(w, model) for w in (0, 1)]

    def set_state(self, model, state):
        for w, (th, m, v, t, rm, rv) in enumerate(state):
            self.set_params(w, model, th)
            self.set_opt_state(w, model, m, v, t)
            self.set_bn_running(w, model, rm, rv)

    def get_bn_running(self, which, model):
        B = self.bn_count(which)
        m, v = np.empty(B, self.real), np.empty(B, self.real)
        assert self.L.oracle_get_bn_running(self.h, which, model, _d(m), _d(v)) == 0
        return m, v

    def train_step(self, label_ids, noise, real, only_model=-1):
        label_ids = np.ascontiguousarray(label_ids, np.int32)
        noise, real = np.ascontiguousarray(noise, self.real), np.ascontiguousarray(real, self.real)
        n = label_ids.size
        return self.L.oracle_train_step(self.h, _i(label_ids), _d(noise), _d(real), n, only_model)

    def generate(self, label_ids, noise, use_running_stats=0, only_model=-1):
        label_ids = np.ascontiguousarray(label_ids, np.int32)
        noise = np.ascontiguousarray(noise, self.real)
        n = label_ids.size
        out = np.zeros((n,) + self.img_shape, self.real)
        rc = self.L.oracle_generate(self.h, _i(label_ids), _d(noise), n, _d(out), use_running_stats, only_model)
        return rc, out

    def sample(self, prior, u, noise, use_running_stats=1):
        """Mixture samples (Eq. 5): labels drawn from `prior` with the caller's uniforms, then the per-label generators."""
        prior = np.ascontiguousarray(prior, np.float64)
        u = np.ascontiguousarray(u, np.float32)
        noise = np.ascontiguousarray(noise, self.real)
        n = u.size
        out = np.zeros((n,) + self.img_shape, self.real)
        labels = np.empty(n, np.int32)
        rc = self.L.oracle_sample(self.h, prior.ctypes.data_as(C.POINTER(C.c_double)), u.ctypes.data_as(C.POINTER(C.c_float)),
                                  _d(noise), n, _d(out), _i(labels), use_running_stats)
        return rc, out, labels

    def get_losses(self):
        K = self.n_models
        jd, jg, cnt = np.empty(K, self.real), np.empty(K, self.real), np.empty(K, np.int32)
        self.L.oracle_get_losses(self.h, _d(jd), _d(jg), _i(cnt))
        return jd, jg, cnt

    def get_routing(self, n):
        perm, offs = np.empty(n, np.int32), np.empty(self.n_models + 1, np.int32)
        self.L.oracle_get_routing(self.h, _i(perm), _i(offs))
        return perm, offs

    def eval_losses(self, model, label_ids, noise, real):
        label_ids = np.ascontiguousarray(label_ids, np.int32)
        noise, real = np.ascontiguousarray(noise, self.real), np.ascontiguousarray(real, self.real)
        jd, jg = np.empty(1, self.real), np.empty(1, self.real)
        self.L.oracle_eval_losses(self.h, model, _i(label_ids), _d(noise), _d(real), label_ids.size,
                                 _d(jd), _d(jg))
        return float(jd[0]), float(jg[0])

    def eval_grads(self, model, label_ids, noise, real):
        label_ids = np.ascontiguousarray(label_ids, np.int32)
        noise, real = np.ascontiguousarray(noise, self.real), np.ascontiguousarray(real, self.real)
        gD, gG = np.empty(self.param_count(1), self.real), np.empty(self.param_count(0), self.real)
        self.L.oracle_eval_grads(self.h, model, _i(label_ids), _d(noise), _d(real), label_ids.size, _d(gD), _d(gG))
        return gD, gG


# ---- single operations on numpy arrays (NCHW) ------------------------------

def round_bf16(x):
    """The emulation's rounding of one value (via single precision, to nearest even)."""
    return float(lib().oracle_round_bf16(float(x)))


def conv2d(X, W, bias=None, k=4, s=2, p=1):
    X, W, bias = _f64(X), _f64(W), _f64(bias)
    N, Cin, H, Wd = X.shape
    Cout = W.shape[0]
    Y = np.empty((N, Cout, (H + 2 * p - k) // s + 1, (Wd + 2 * p - k) // s + 1))
    lib().oracle_conv2d(_d(X), _d(W), _d(bias), _d(Y), N, Cin, H, Wd, Cout, k, s, p)
    return Y


def conv2d_bwd(X, W, dY, k=4, s=2, p=1, need_dx=True):
    X, W, dY = _f64(X), _f64(W), _f64(dY)
    N, Cin, H, Wd = X.shape
    Cout = W.shape[0]
    dX = np.empty_like(X) if need_dx else None
    dW, db = np.empty_like(W), np.empty(Cout)
    lib().oracle_conv2d_bwd(_d(X), _d(W), _d(dY), _d(dX), _d(dW), _d(db), N, Cin, H, Wd, Cout, k, s, p)
    return dX, dW, db


def conv_transpose2d(X, W, bias=None, k=4, s=2, p=1):
    X, W, bias = _f64(X), _f64(W), _f64(bias)
    N, Cin, H, Wd = X.shape
    Cout = W.shape[1]
    Y = np.empty((N, Cout, (H - 1) * s - 2 * p + k, (Wd - 1) * s - 2 * p + k))
    lib().oracle_conv_transpose2d(_d(X), _d(W), _d(bias), _d(Y), N, Cin, H, Wd, Cout, k, s, p)
    return Y


def conv_transpose2d_bwd(X, W, dY, k=4, s=2, p=1, need_dx=True):
    X, W, dY = _f64(X), _f64(W), _f64(dY)
    N, Cin, H, Wd = X.shape
    Cout = W.shape[1]
    dX = np.empty_like(X) if need_dx else None
    dW, db = np.empty_like(W), np.empty(Cout)
    lib().oracle_conv_transpose2d_bwd(_d(X), _d(W), _d(dY), _d(dX), _d(dW), _d(db), N, Cin, H, Wd, Cout, k, s, p)
    return dX, dW, db


def linear(X, W, bias=None):
    X, W, bias = _f64(X), _f64(W), _f64(bias)
    Y = np.empty((X.shape[0], W.shape[0]))
    lib().oracle_linear(_d(X), _d(W), _d(bias), _d(Y), X.shape[0], X.shape[1], W.shape[0])
    return Y


def linear_bwd(X, W, dY):
    X, W, dY = _f64(X), _f64(W), _f64(dY)
    dX, dW, db = np.empty_like(X), np.empty_like(W), np.empty(W.shape[0])
    lib().oracle_linear_bwd(_d(X), _d(W), _d(dY), _d(dX), _d(dW), _d(db), X.shape[0], X.shape[1], W.shape[0])
    return dX, dW, db


def bn_train(X, gamma, beta, eps):
    X, gamma, beta = _f64(X), _f64(gamma), _f64(beta)
    N, Cn = X.shape[:2]
    HW = int(np.prod(X.shape[2:]))
    Y, mean, var = np.empty_like(X), np.empty(Cn), np.empty(Cn)
    lib().oracle_bn_train(_d(X), _d(gamma), _d(beta), eps, _d(Y), _d(mean), _d(var), N, Cn, HW)
    return Y, mean, var


def bn_eval(X, gamma, beta, eps, mean, var):
    X, gamma, beta, mean, var = _f64(X), _f64(gamma), _f64(beta), _f64(mean), _f64(var)
    N, Cn = X.shape[:2]
    HW = int(np.prod(X.shape[2:]))
    Y = np.empty_like(X)
    lib().oracle_bn_eval(_d(X), _d(gamma), _d(beta), eps, _d(mean), _d(var), _d(Y), N, Cn, HW)
    return Y


def bn_bwd(X, gamma, mean, var, eps, dY):
    X, gamma, mean, var, dY = _f64(X), _f64(gamma), _f64(mean), _f64(var), _f64(dY)
    N, Cn = X.shape[:2]
    HW = int(np.prod(X.shape[2:]))
    dX, dg, db = np.empty_like(X), np.empty(Cn), np.empty(Cn)
    lib().oracle_bn_bwd(_d(X), _d(gamma), _d(mean), _d(var), eps, _d(dY), _d(dX), _d(dg), _d(db), N, Cn, HW)
    return dX, dg, db


def bn_running_update(rmean, rvar, mean, var, momentum, count):
    rmean, rvar = _f64(rmean).copy(), _f64(rvar).copy()
    mean, var = _f64(mean), _f64(var)
    lib().oracle_bn_running_update(_d(rmean), _d(rvar), _d(mean), _d(var), momentum, rmean.size, count)
    return rmean, rvar


def leaky_relu(X, slope):
    X = _f64(X)
    Y = np.empty_like(X)
    lib().oracle_leaky_relu(_d(X), _d(Y), X.size, slope)
    return Y


def leaky_relu_bwd(X, dY, slope):
    X, dY = _f64(X), _f64(dY)
    dX = np.empty_like(X)
    lib().oracle_leaky_relu_bwd(_d(X), _d(dY), _d(dX), X.size, slope)
    return dX


def tanh(X):
    X = _f64(X)
    Y = np.empty_like(X)
    lib().oracle_tanh(_d(X), _d(Y), X.size)
    return Y


def tanh_bwd(Y, dY):
    Y, dY = _f64(Y), _f64(dY)
    dX = np.empty_like(Y)
    lib().oracle_tanh_bwd(_d(Y), _d(dY), _d(dX), Y.size)
    return dX


def logistic_loss(s, sign, scale):
    s = _f64(s)
    ds = np.empty_like(s)
    val = lib().oracle_logistic_loss(_d(s), s.size, sign, scale, _d(ds))
    return val, ds


def adam(theta, m, v, g, t, lr=2e-4, beta1=0.5, beta2=0.999, eps=1e-8):
    theta, m, v, g = _f64(theta).copy(), _f64(m).copy(), _f64(v).copy(), _f64(g)
    lib().oracle_adam(_d(theta), _d(m), _d(v), _d(g), theta.size, t, lr, beta1, beta2, eps)
    return theta, m, v


def route(label_ids, n_models, n_labels):
    label_ids = np.ascontiguousarray(label_ids, np.int32)
    n = label_ids.size
    perm, offs, bad = np.empty(max(n, 1), np.int32), np.empty(n_models + 1, np.int32), C.c_int32()
    lib().oracle_route(_i(label_ids), n, n_models, n_labels, _i(perm), _i(offs), C.byref(bad))
    return perm[:n], offs, bad.value


def draw_labels(prior, u):
    prior = np.ascontiguousarray(prior, np.float64)
    u = np.ascontiguousarray(u, np.float32)
    labels = np.empty(u.size, np.int32)
    rc = lib().oracle_draw_labels(prior.ctypes.data_as(C.POINTER(C.c_double)), prior.size,
                                  u.ctypes.data_as(C.POINTER(C.c_float)), u.size, _i(labels))
    return rc, labels


def anova_f(label_ids, images, n_labels):
    """F-statistic per channel of the per-image mean intensities grouped by label; images [n, C, H, W] float32."""
    label_ids = np.ascontiguousarray(label_ids, np.int32)
    images = np.ascontiguousarray(images, np.float32)
    n, Cc, H, W = images.shape
    F = np.zeros(Cc, np.float64)
    rc = lib().oracle_anova_f(_i(label_ids), images.ctypes.data_as(C.POINTER(C.c_float)), n, n_labels, Cc, H * W,
                              F.ctypes.data_as(C.POINTER(C.c_double)))
    return rc, F


def threads():
    return int(lib().oracle_threads())
