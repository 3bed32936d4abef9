"""ctypes binding of include/gan.h: argument marshalling only, every step runs in the HIP library.

Device buffers are passed as integer addresses (for example torch tensors' data_ptr()).
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
MAX_LAYERS = 8
FP32, BF16 = 0, 1
FAMILY_STRIDED, FAMILY_PAPER = 0, 1

GAN_OK, GAN_E_ARG, GAN_E_SHAPE, GAN_E_OOM, GAN_E_HIP, GAN_E_LABEL, GAN_E_STATE = 0, -1, -2, -3, -4, -5, -6


class GanError(RuntimeError):
    def __init__(self, status, msg=""):
        super().__init__("gan status %d %s" % (status, msg))
        self.status = status


class GanConfig(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("precision", C.c_int32),
        ("n_models", C.c_int32), ("n_labels", C.c_int32),
        ("cond_g", C.c_int32), ("cond_d", C.c_int32), ("z_dim", C.c_int32),
        ("img_c", C.c_int32), ("img_hw", C.c_int32), ("g_h0", C.c_int32),
        ("n_g", C.c_int32), ("g_ch", C.c_int32 * MAX_LAYERS),
        ("n_d", C.c_int32), ("d_ch", C.c_int32 * MAX_LAYERS),
        ("max_total_batch", C.c_int32),
        ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("adam_eps", C.c_float),
        ("bn_eps", C.c_float), ("bn_momentum", C.c_float), ("leaky_slope", C.c_float),
        ("d_loss_scale", C.c_float), ("g_loss_scale", C.c_float),
        ("init_std", C.c_float), ("seed", C.c_uint64),
        ("family", C.c_int32), ("bn_eps_first", C.c_float), ("dropout_p", C.c_float),
    ]


def lib_path():
    return os.path.join(_HERE, "libgan_hip.so")


_lib = None
_VP, _I64P, _FP, _IP = C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_float), C.POINTER(C.c_int32)


def load_library():
    """Load the built library; building is a separate, explicit step (paper_2102_10485_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise GanError(GAN_E_STATE, "HIP library not built: run `python -m paper_2102_10485_amd.build` "
                                    "(there is no CPU fallback)")
    L = C.CDLL(path)
    L.gan_create.argtypes = [C.POINTER(GanConfig), _VP, C.POINTER(_VP)]
    L.gan_destroy.argtypes = [_VP]
    L.gan_train_step.argtypes = [_VP, _VP, _VP, _VP, C.c_int32]
    L.gan_generate.argtypes = [_VP, _VP, _VP, C.c_int32, _VP, C.c_int32]
    L.gan_get_losses.argtypes = [_VP, _FP, _FP, _IP]
    L.gan_param_count.argtypes = [_VP, C.c_int32, _I64P]
    L.gan_bn_count.argtypes = [_VP, C.c_int32, _I64P]
    L.gan_get_params.argtypes = [_VP, C.c_int32, C.c_int32, _FP, C.c_int64]
    L.gan_set_params.argtypes = [_VP, C.c_int32, C.c_int32, _FP, C.c_int64]
    L.gan_get_grads.argtypes = [_VP, C.c_int32, C.c_int32, _FP, C.c_int64]
    L.gan_get_opt_state.argtypes = [_VP, C.c_int32, C.c_int32, _FP, _FP, _I64P]
    L.gan_set_opt_state.argtypes = [_VP, C.c_int32, C.c_int32, _FP, _FP, C.c_int64]
    L.gan_set_bn_running.argtypes = [_VP, C.c_int32, C.c_int32, _FP, _FP, C.c_int64]
    L.gan_get_bn_running.argtypes = [_VP, C.c_int32, C.c_int32, _FP, _FP, C.c_int64]
    L.gan_get_routing.argtypes = [_VP, _IP, _IP]
    L.gan_last_error.argtypes = [_VP]
    L.gan_last_error.restype = C.c_char_p
    L.gan_profile_enable.argtypes = [_VP, C.c_int32]
    L.gan_use_graphs.argtypes = [_VP, C.c_int32]
    L.gan_op_tile_rows.argtypes = [_VP, C.c_int32]
    L.gan_use_second_stream.argtypes = [_VP, C.c_int32]
    L.gan_graph_replays.argtypes = [_VP, C.POINTER(C.c_int64)]
    L.gan_profile_read.argtypes = [_VP, C.c_int32, C.POINTER(C.c_char_p), _I64P, C.POINTER(C.c_double),
                                   C.POINTER(C.c_double), C.POINTER(C.c_double), _IP]
    op = [_VP, _VP, _VP, _VP, _VP, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    L.gan_op_conv_down.argtypes = op
    L.gan_op_conv_up.argtypes = op
    L.gan_op_conv_wgrad.argtypes = op
    L.gan_op_dropout.argtypes = [_VP, _VP, _VP, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_uint64,
                                 C.c_int32, C.c_int32, C.c_int32]
    L.gan_op_w3_to_w4.argtypes = [_VP, _VP, _VP, _VP, C.c_int32, C.c_int32, C.c_int32]
    L.gan_op_dw4_to_dw3.argtypes = [_VP, _VP, _VP, C.c_int32, C.c_int32, C.c_int32]
    L.gan_sample.argtypes = [_VP, C.POINTER(C.c_double), _VP, _VP, C.c_int32, _VP, _VP, C.c_int32]
    L.gan_anova_f.argtypes = [_VP, _VP, _VP, C.c_int32, C.POINTER(C.c_double)]
    L.gan_anova_f_static.argtypes = [_VP, _VP, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _VP, C.POINTER(C.c_double)]
    L.gan_static_last_error.restype = C.c_char_p
    L.gan_probe_mfma.argtypes = [C.c_int32, _VP, C.POINTER(C.c_double)]
    L.gan_probe_copy.argtypes = [C.c_int64, _VP, C.POINTER(C.c_double)]
    _lib = L
    return L


def anova_f_static(label_ids_ptr, images_ptr, n, n_labels, img_c, img_hw, stream=0):
    """gan_anova_f without a context and without device allocations (static scratch array); returns (status, F)."""
    F = np.zeros(max(img_c, 1), np.float64)
    st = load_library().gan_anova_f_static(label_ids_ptr, images_ptr, n, n_labels, img_c, img_hw, stream,
                                           F.ctypes.data_as(C.POINTER(C.c_double)))
    return st, F[:max(img_c, 0)]


def static_last_error():
    return (load_library().gan_static_last_error() or b"").decode()


def probe_mfma(precision, stream=0):
    """TFLOP/s of a register-only MFMA loop in this precision's arithmetic."""
    v = C.c_double()
    st = load_library().gan_probe_mfma(precision, stream, C.byref(v))
    if st != GAN_OK:
        raise GanError(st, "gan_probe_mfma")
    return v.value


def probe_copy(nbytes=1 << 30, stream=0):
    """GB/s (read + written) of a plain device-to-device copy."""
    v = C.c_double()
    st = load_library().gan_probe_copy(nbytes, stream, C.byref(v))
    if st != GAN_OK:
        raise GanError(st, "gan_probe_copy")
    return v.value


def make_config(spec, n_models, n_labels, max_total_batch, precision=FP32, hyper=None, seed=1):
    paper = spec.get("family") == "paper"
    h = dict(lr=2e-4, beta1=0.5, beta2=0.999, adam_eps=1e-8, bn_eps=0.8 if paper else 1e-5, bn_momentum=0.1,
             leaky_slope=0.2, d_loss_scale=0.5, g_loss_scale=0.5, init_std=0.02, bn_eps_first=1e-5,
             dropout_p=0.25 if paper else 0.0)
    h.update(hyper or {})
    c = GanConfig()
    c.struct_size = C.sizeof(GanConfig)
    c.precision = precision
    c.n_models, c.n_labels = n_models, n_labels
    c.cond_g, c.cond_d, c.z_dim = spec["cond_g"], spec["cond_d"], spec["z_dim"]
    c.img_c, c.img_hw, c.g_h0 = spec["img_c"], spec["img_hw"], spec["g_h0"]
    c.n_g = len(spec["g_ch"])
    for i, v in enumerate(spec["g_ch"]):
        c.g_ch[i] = v
    c.n_d = len(spec["d_ch"])
    for i, v in enumerate(spec["d_ch"]):
        c.d_ch[i] = v
    c.max_total_batch = max_total_batch
    c.family = FAMILY_PAPER if paper else FAMILY_STRIDED
    for k, v in h.items():
        setattr(c, k, v)
    c.seed = seed
    return c


def _fp(a):
    return a.ctypes.data_as(_FP)


class Gan:
    """One context = all label models of one configuration on the current device."""

    def __init__(self, cfg, stream=0):
        self.lib = load_library()
        self.cfg = cfg
        self.h = _VP()
        st = self.lib.gan_create(C.byref(cfg), _VP(stream), C.byref(self.h))
        if st != GAN_OK:
            raise GanError(st, "gan_create")
        self.n_models = cfg.n_models

    def close(self):
        if self.h:
            self.lib.gan_destroy(self.h)
            self.h = _VP()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st):
        if st != GAN_OK:
            raise GanError(st, (self.lib.gan_last_error(self.h) or b"").decode())

    def train_step(self, label_ids_ptr, noise_ptr, real_ptr, n):
        self._check(self.lib.gan_train_step(self.h, label_ids_ptr, noise_ptr, real_ptr, n))

    def generate(self, label_ids_ptr, noise_ptr, n, out_ptr, use_running_stats=0):
        self._check(self.lib.gan_generate(self.h, label_ids_ptr, noise_ptr, n, out_ptr, use_running_stats))

    def sample(self, prior, u_ptr, noise_ptr, n, out_ptr, labels_ptr, use_running_stats=1):
        prior = np.ascontiguousarray(prior, np.float64)
        self._check(self.lib.gan_sample(self.h, prior.ctypes.data_as(C.POINTER(C.c_double)), u_ptr, noise_ptr, n, out_ptr,
                                        labels_ptr, use_running_stats))

    def anova_f(self, label_ids_ptr, images_ptr, n, img_c):
        F = np.zeros(img_c, np.float64)
        st = self.lib.gan_anova_f(self.h, label_ids_ptr, images_ptr, n, F.ctypes.data_as(C.POINTER(C.c_double)))
        return st, F

    def get_losses(self, check=True):
        K = self.n_models
        d, g, cnt = np.empty(K, np.float32), np.empty(K, np.float32), np.empty(K, np.int32)
        st = self.lib.gan_get_losses(self.h, _fp(d), _fp(g), cnt.ctypes.data_as(_IP))
        if check:
            self._check(st)
        return (d, g, cnt) if check else (d, g, cnt, st)

    def param_count(self, which):
        n = C.c_int64()
        self._check(self.lib.gan_param_count(self.h, which, C.byref(n)))
        return n.value

    def bn_count(self, which):
        n = C.c_int64()
        self._check(self.lib.gan_bn_count(self.h, which, C.byref(n)))
        return n.value

    def get_params(self, which, model):
        out = np.empty(self.param_count(which), np.float32)
        self._check(self.lib.gan_get_params(self.h, which, model, _fp(out), out.size))
        return out

    def set_params(self, which, model, src):
        src = np.ascontiguousarray(src, np.float32)
        self._check(self.lib.gan_set_params(self.h, which, model, _fp(src), src.size))

    def get_grads(self, which, model):
        out = np.empty(self.param_count(which), np.float32)
        self._check(self.lib.gan_get_grads(self.h, which, model, _fp(out), out.size))
        return out

    def get_opt_state(self, which, model):
        P = self.param_count(which)
        m, v, t = np.empty(P, np.float32), np.empty(P, np.float32), C.c_int64()
        self._check(self.lib.gan_get_opt_state(self.h, which, model, _fp(m), _fp(v), C.byref(t)))
        return m, v, t.value

    def set_opt_state(self, which, model, m, v, t):
        m = None if m is None else np.ascontiguousarray(m, np.float32)
        v = None if v is None else np.ascontiguousarray(v, np.float32)
        self._check(self.lib.gan_set_opt_state(self.h, which, model, None if m is None else _fp(m),
                                               None if v is None else _fp(v), int(t)))

    def set_bn_running(self, which, model, mean, var):
        mean, var = np.ascontiguousarray(mean, np.float32), np.ascontiguousarray(var, np.float32)
        self._check(self.lib.gan_set_bn_running(self.h, which, model, _fp(mean), _fp(var), mean.size))

    def get_bn_running(self, which, model):
        B = self.bn_count(which)
        m, v = np.empty(B, np.float32), np.empty(B, np.float32)
        self._check(self.lib.gan_get_bn_running(self.h, which, model, _fp(m), _fp(v), B))
        return m, v

    def get_routing(self, n):
        perm, offs = np.empty(max(n, 1), np.int32), np.empty(self.n_models + 1, np.int32)
        self._check(self.lib.gan_get_routing(self.h, perm.ctypes.data_as(_IP), offs.ctypes.data_as(_IP)))
        return perm[:n], offs

    def graph_replays(self):
        n = C.c_int64(0)
        self._check(self.lib.gan_graph_replays(self.h, C.byref(n)))
        return int(n.value)

    def use_second_stream(self, on=True):
        self._check(self.lib.gan_use_second_stream(self.h, 1 if on else 0))

    def use_graphs(self, on=True):
        self._check(self.lib.gan_use_graphs(self.h, 1 if on else 0))

    def profile_enable(self, on=True, detail=False, gemm_only=False):
        level = 0 if not on else (2 if detail else (3 if gemm_only else 1))
        self._check(self.lib.gan_profile_enable(self.h, level))

    def profile_read(self, cap=64):
        names = (C.c_char_p * cap)()
        launches = (C.c_int64 * cap)()
        ms, flops, nbytes = (C.c_double * cap)(), (C.c_double * cap)(), (C.c_double * cap)()
        n = C.c_int32()
        self._check(self.lib.gan_profile_read(self.h, cap, names, launches, ms, flops, nbytes, C.byref(n)))
        return {names[i].decode(): dict(launches=launches[i], ms=ms[i], flops=flops[i], bytes=nbytes[i])
                for i in range(n.value)}

    # single operations (device pointers as integers)
    def op_tile_rows(self, rows):
        self._check(self.lib.gan_op_tile_rows(self.h, rows))

    def op_conv_down(self, big, w_down, small_out, offs, n_groups, n_samples, cb, cs, hs):
        self._check(self.lib.gan_op_conv_down(self.h, big, w_down, small_out, offs, n_groups, n_samples, cb, cs, hs))

    def op_conv_up(self, small_in, w_up, big_out, offs, n_groups, n_samples, cb, cs, hs):
        self._check(self.lib.gan_op_conv_up(self.h, small_in, w_up, big_out, offs, n_groups, n_samples, cb, cs, hs))

    def op_conv_wgrad(self, big, small_in, dw, offs, n_groups, n_samples, cb, cs, hs):
        self._check(self.lib.gan_op_conv_wgrad(self.h, big, small_in, dw, offs, n_groups, n_samples, cb, cs, hs))

    def op_dropout(self, x, offs, n_groups, n_samples, ch, h, w, p, seed, step, layer, pass_id):
        self._check(self.lib.gan_op_dropout(self.h, x, offs, n_groups, n_samples, ch, h, w, p, seed, step, layer, pass_id))

    def op_w3_to_w4(self, w3, w4, w4t, n_groups, cb, cs):
        self._check(self.lib.gan_op_w3_to_w4(self.h, w3, w4, w4t, n_groups, cb, cs))

    def op_dw4_to_dw3(self, dw4, dw3, n_groups, cb, cs):
        self._check(self.lib.gan_op_dw4_to_dw3(self.h, dw4, dw3, n_groups, cb, cs))
