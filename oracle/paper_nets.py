"""Oracle for the networks exactly as the paper's Tables 1 and 2 print them (Section 4), trained by the same iteration
(Eq. 3, Eq. 4, Adam): a plain composition of this package's single operations (each pinned on its own) plus nearest
upsampling and dropout.  TEST INFRASTRUCTURE ONLY: slow, fp64, one label model after the other.

    G (Table 1): z -> Linear(z_dim -> C0*s*s) -> ReLU -> reshape [C0, s, s] -> BatchNorm(eps 1e-5)
                 -> Upsample x2 -> Conv k3 s1 p1 (C0 -> g1) -> BatchNorm(eps 0.8) -> LeakyReLU(0.2)
                 -> Upsample x2 -> Conv k3 s1 p1 (g1 -> g2) -> BatchNorm(eps 0.8) -> LeakyReLU(0.2)
                 -> Conv k3 s1 p1 (g2 -> img_c) -> tanh                       (128, 128, 64 in the table; s = img_hw / 4)
    D (Table 2): { Conv k3 s2 p1 -> LeakyReLU(0.2) -> Dropout(0.25) [-> BatchNorm(eps 0.8), not after the first] } x 4
                 -> flatten -> Linear -> logit                                 (16, 32, 64, 128 in the table)

Readings (the tables do not say):
  * the distributed scheme uses these unconditional networks, one pair per label (Section 4);
  * BatchNorm's 0.8 is taken as the epsilon the tables call it; momentum 0.1; biased variance normalises, the
    unbiased one goes into the running statistics;
  * a layer directly followed by BatchNorm has no bias (it would cancel); the others have one;
  * D returns a logit and the sigmoid of Table 2 lives in the cost (Table 4 prints "None" for the same layer);
  * dropout is active in all three discriminator passes of an iteration (real, fake, fake through the updated D),
    each with its own mask; kept values are scaled by 1 / (1 - p).

The dropout mask must be reproducible bit for bit by any other implementation, so it comes from a counter-based
generator, Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
SC'11), written here from its definition:
    counter = (q low, q high, layer + 256 * pass, iteration of the model), q = element index // 4
    key     = (seed low, seed high xor model index)
    element index = ((n * C + c) * H + y) * W + x with n the sample's position among the model's samples (stable order)
    u = (output word number (element index % 4) >> 8) * 2^-24 ;  keep the element iff u >= p
(all four output words of a counter are used: four consecutive elements share one evaluation of the generator).
"""
import numpy as np

import oracle as O

_M0, _M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_W0, _W1 = np.uint32(0x9E3779B9), np.uint32(0xBB67AE85)
_LO32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten rounds of Philox-4x32 on arrays of counters (broadcast); returns the four output words."""
    c0, c1, c2, c3 = (np.asarray(x, np.uint32) for x in (c0, c1, c2, c3))
    k0, k1 = np.asarray(k0, np.uint32), np.asarray(k1, np.uint32)
    with np.errstate(over="ignore"):
        for r in range(10):
            if r > 0:                                   # the key is bumped by the Weyl constants between rounds
                k0, k1 = (k0 + _W0).astype(np.uint32), (k1 + _W1).astype(np.uint32)
            p0, p1 = _M0 * c0.astype(np.uint64), _M1 * c2.astype(np.uint64)
            hi0, lo0 = (p0 >> np.uint64(32)).astype(np.uint32), (p0 & _LO32).astype(np.uint32)
            hi1, lo1 = (p1 >> np.uint64(32)).astype(np.uint32), (p1 & _LO32).astype(np.uint32)
            c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return c0, c1, c2, c3


def dropout_keep(shape, p, seed, model, step, layer, pass_id):
    """Boolean keep-mask of an [n, C, H, W] tensor of one model (definition in the module header)."""
    total = int(np.prod(shape))
    q = np.arange((total + 3) // 4, dtype=np.uint64)                    # one counter per four consecutive elements
    lo, hi = (q & _LO32).astype(np.uint32), (q >> np.uint64(32)).astype(np.uint32)
    k0 = np.uint32(seed & 0xFFFFFFFF)
    k1 = np.uint32(((seed >> 32) & 0xFFFFFFFF) ^ model)
    words = philox4x32_10(lo, hi, np.uint32(layer + 256 * pass_id), np.uint32(step), k0, k1)
    w = np.stack(words, axis=1).reshape(-1)[:total]                      # element i: word i % 4 of counter i // 4
    u = (w >> np.uint32(8)).astype(np.float64) * (1.0 / 16777216.0)
    return (u >= p).reshape(shape)


def upsample2(x):
    """Nearest-neighbour upsampling by 2 of [n, C, H, W]: out[2y + a, 2x + b] = in[y, x]."""
    return np.repeat(np.repeat(x, 2, axis=2), 2, axis=3)


def upsample2_bwd(dy):
    """Adjoint of upsample2: every input pixel collects its four copies."""
    n, c, h2, w2 = dy.shape
    return dy.reshape(n, c, h2 // 2, 2, w2 // 2, 2).sum(axis=(3, 5))


HYPER = dict(lr=2e-4, beta1=0.5, beta2=0.999, adam_eps=1e-8, bn_eps_first=1e-5, bn_eps=0.8, bn_momentum=0.1,
             slope=0.2, drop=0.25, d_scale=0.5, g_scale=0.5)


def g_shapes(img_c, img_hw, z_dim, g_ch):
    c0, g1, g2 = g_ch
    s = img_hw // 4
    return [("fc.w", (c0 * s * s, z_dim)), ("fc.b", (c0 * s * s,)), ("bn0.gamma", (c0,)), ("bn0.beta", (c0,)),
            ("conv1.w", (g1, c0, 3, 3)), ("bn1.gamma", (g1,)), ("bn1.beta", (g1,)),
            ("conv2.w", (g2, g1, 3, 3)), ("bn2.gamma", (g2,)), ("bn2.beta", (g2,)),
            ("conv3.w", (img_c, g2, 3, 3)), ("conv3.b", (img_c,))]


def d_shapes(img_c, img_hw, d_ch):
    out, cin, h = [], img_c, img_hw
    for j, c in enumerate(d_ch, 1):
        out += [("conv%d.w" % j, (c, cin, 3, 3)), ("conv%d.b" % j, (c,))]
        if j > 1:
            out += [("bn%d.gamma" % j, (c,)), ("bn%d.beta" % j, (c,))]
        cin, h = c, (h + 2 - 3) // 2 + 1
    out += [("fc.w", (1, cin * h * h)), ("fc.b", (1,))]
    return out


def init_params(shapes, rng, std=0.02):
    """Weights N(0, std^2), biases and beta 0, gamma 1."""
    p = {}
    for name, shp in shapes:
        if name.endswith(".w"):
            p[name] = rng.normal(0.0, std, shp)
        elif name.endswith("gamma"):
            p[name] = np.ones(shp)
        else:
            p[name] = np.zeros(shp)
    return p


class PaperNets:
    """K independent pairs of the paper-literal networks; `train_step` is one iteration for every label present."""

    def __init__(self, img_c, img_hw, n_models, z_dim=100, g_ch=(128, 128, 64), d_ch=(16, 32, 64, 128), hyper=None,
                 seed=0):
        assert img_hw % 4 == 0
        self.img_c, self.img_hw, self.K, self.z_dim = img_c, img_hw, n_models, z_dim
        self.g_ch, self.d_ch = tuple(g_ch), tuple(d_ch)
        self.h = dict(HYPER, **(hyper or {}))
        self.seed = seed
        self.gs, self.ds = g_shapes(img_c, img_hw, z_dim, g_ch), d_shapes(img_c, img_hw, d_ch)
        self.G = [None] * n_models
        self.D = [None] * n_models
        self.opt = [[{}, {}] for _ in range(n_models)]                 # per model, per net: name -> (m, v)
        self.t = np.zeros((n_models, 2), np.int64)
        self.step = np.zeros(n_models, np.int64)                       # iterations this model has run
        self.run = [[{}, {}] for _ in range(n_models)]                 # running (mean, var) per BatchNorm
        self.jd, self.jg = np.zeros(n_models), np.zeros(n_models)
        self.counts = np.zeros(n_models, np.int32)
        self.grads = [[None, None] for _ in range(n_models)]

    def set_params(self, which, model, params):
        tgt = {k: np.array(v, np.float64) for k, v in params.items()}
        assert [k for k, _ in (self.gs if which == 0 else self.ds)] == list(tgt)
        (self.G if which == 0 else self.D)[model] = tgt

    # ---- generator ---------------------------------------------------------------------------------------
    def g_forward(self, p, z, running=None, update=None):
        h, k = self.h, {}
        n = z.shape[0]
        c0 = self.g_ch[0]
        s = self.img_hw // 4
        k["z"] = z
        k["a0"] = O.linear(z, p["fc.w"], p["fc.b"])
        k["x0"] = O.leaky_relu(k["a0"], 0.0).reshape(n, c0, s, s)
        cur = self._bn(k, "0", k["x0"], p["bn0.gamma"], p["bn0.beta"], h["bn_eps_first"], running, update)
        for j in (1, 2):
            k["u%d" % j] = upsample2(cur)
            k["c%d" % j] = O.conv2d(k["u%d" % j], p["conv%d.w" % j], None, 3, 1, 1)
            k["b%d" % j] = self._bn(k, str(j), k["c%d" % j], p["bn%d.gamma" % j], p["bn%d.beta" % j], h["bn_eps"],
                                    running, update)
            cur = k["h%d" % j] = O.leaky_relu(k["b%d" % j], h["slope"])
        k["out"] = O.tanh(O.conv2d(cur, p["conv3.w"], p["conv3.b"], 3, 1, 1))
        return k["out"], k

    def g_backward(self, p, k, dout):
        h, g = self.h, {}
        d = O.tanh_bwd(k["out"], dout)
        d, g["conv3.w"], g["conv3.b"] = O.conv2d_bwd(k["h2"], p["conv3.w"], d, 3, 1, 1)
        for j in (2, 1):
            d = O.leaky_relu_bwd(k["b%d" % j], d, h["slope"])
            d, g["bn%d.gamma" % j], g["bn%d.beta" % j] = O.bn_bwd(k["c%d" % j], p["bn%d.gamma" % j], k["mean" + str(j)],
                                                                  k["var" + str(j)], h["bn_eps"], d)
            d, g["conv%d.w" % j], _ = O.conv2d_bwd(k["u%d" % j], p["conv%d.w" % j], d, 3, 1, 1)
            d = upsample2_bwd(d)
        d, g["bn0.gamma"], g["bn0.beta"] = O.bn_bwd(k["x0"], p["bn0.gamma"], k["mean0"], k["var0"], h["bn_eps_first"], d)
        d = O.leaky_relu_bwd(k["a0"], d.reshape(k["a0"].shape), 0.0)
        _, g["fc.w"], g["fc.b"] = O.linear_bwd(k["z"], p["fc.w"], d)
        return {name: g[name] for name, _ in self.gs}

    def _bn(self, k, tag, x, gamma, beta, eps, running, update):
        """Training-mode BatchNorm; `running` (dict) is updated in place when `update` is set."""
        y, mean, var = O.bn_train(x, gamma, beta, eps)
        k["mean" + tag], k["var" + tag] = mean, var
        if update is not None and running is not None:
            rm, rv = running.get(tag, (np.zeros_like(mean), np.ones_like(var)))
            running[tag] = O.bn_running_update(rm, rv, mean, var, self.h["bn_momentum"], x.size // x.shape[1])
        return y

    # ---- discriminator -----------------------------------------------------------------------------------
    def d_forward(self, p, x, model, step, pass_id, running=None, update=None, train=True):
        h, k = self.h, {"x": x}
        cur = x
        keep_scale = 1.0 / (1.0 - h["drop"])
        for j in range(1, len(self.d_ch) + 1):
            k["in%d" % j] = cur
            k["c%d" % j] = O.conv2d(cur, p["conv%d.w" % j], p["conv%d.b" % j], 3, 2, 1)
            a = O.leaky_relu(k["c%d" % j], h["slope"])
            if train:
                k["m%d" % j] = dropout_keep(a.shape, h["drop"], self.seed, model, step, j, pass_id) * keep_scale
                a = a * k["m%d" % j]
            else:
                k["m%d" % j] = np.ones_like(a)
            k["d%d" % j] = a
            cur = a if j == 1 else self._bn(k, str(j), a, p["bn%d.gamma" % j], p["bn%d.beta" % j], h["bn_eps"], running,
                                            update)
        k["flat"] = np.ascontiguousarray(cur.reshape(cur.shape[0], -1))
        k["shape"] = cur.shape
        return O.linear(k["flat"], p["fc.w"], p["fc.b"])[:, 0], k

    def d_backward(self, p, k, ds, need_dx=False):
        h, g = self.h, {}
        d, g["fc.w"], g["fc.b"] = O.linear_bwd(k["flat"], p["fc.w"], ds[:, None])
        d = d.reshape(k["shape"])
        for j in range(len(self.d_ch), 0, -1):
            if j > 1:
                d, g["bn%d.gamma" % j], g["bn%d.beta" % j] = O.bn_bwd(k["d%d" % j], p["bn%d.gamma" % j],
                                                                      k["mean" + str(j)], k["var" + str(j)], h["bn_eps"], d)
            d = O.leaky_relu_bwd(k["c%d" % j], d * k["m%d" % j], h["slope"])
            d, g["conv%d.w" % j], g["conv%d.b" % j] = O.conv2d_bwd(k["in%d" % j], p["conv%d.w" % j], d, 3, 2, 1,
                                                                   need_dx=(j > 1 or need_dx))
        return {name: g[name] for name, _ in self.ds}, d

    # ---- the iteration -----------------------------------------------------------------------------------
    def costs_and_grads(self, model, z, x, step, update_running=False):
        """J_D, dJ_D/dtheta_D, J_G (through the given D, not an updated one), dJ_G/dtheta_G for one model's batch."""
        pG, pD, h = self.G[model], self.D[model], self.h
        run = self.run[model] if update_running else [None, None]
        upd = True if update_running else None
        fake, kg = self.g_forward(pG, z, run[0], upd)
        sr, kr = self.d_forward(pD, x, model, step, 0, run[1], upd)
        sf, kf = self.d_forward(pD, fake, model, step, 1, run[1], upd)
        jr, dsr = O.logistic_loss(sr, -1, h["d_scale"])
        jf, dsf = O.logistic_loss(sf, +1, h["d_scale"])
        gr, _ = self.d_backward(pD, kr, dsr)
        gf, _ = self.d_backward(pD, kf, dsf)
        gD = {n_: gr[n_] + gf[n_] for n_ in gr}
        return jr + jf, gD, (fake, kg)

    def g_cost_and_grads(self, model, fake_kg, step, update_running=False):
        pG, pD, h = self.G[model], self.D[model], self.h
        run = self.run[model] if update_running else [None, None]
        upd = True if update_running else None
        fake, kg = fake_kg
        s2, k2 = self.d_forward(pD, fake, model, step, 2, run[1], upd)
        jg, ds2 = O.logistic_loss(s2, -1, h["g_scale"])
        _, dfake = self.d_backward(pD, k2, ds2, need_dx=True)
        return jg, self.g_backward(pG, kg, dfake)

    def _adam(self, model, which, params, grads):
        h = self.h
        self.t[model, which] += 1
        for name in params:
            m, v = self.opt[model][which].get(name, (np.zeros_like(params[name]), np.zeros_like(params[name])))
            th, m, v = O.adam(params[name].ravel(), m.ravel(), v.ravel(), grads[name].ravel(), int(self.t[model, which]),
                              h["lr"], h["beta1"], h["beta2"], h["adam_eps"])
            params[name] = th.reshape(params[name].shape)
            self.opt[model][which][name] = (m.reshape(params[name].shape), v.reshape(params[name].shape))

    def train_step(self, label_ids, noise, real):
        """One iteration: D update from (real, fake), then G update through the updated D on the same fake batch."""
        label_ids = np.asarray(label_ids)
        mdl = label_ids if self.K > 1 else np.zeros_like(label_ids)
        for l in range(self.K):
            idx = np.flatnonzero(mdl == l)                              # increasing: the stable order
            self.counts[l] = idx.size
            if idx.size == 0:
                self.jd[l] = self.jg[l] = 0.0
                continue
            self.step[l] += 1
            z = np.ascontiguousarray(noise[idx], np.float64)
            x = np.ascontiguousarray(real[idx], np.float64)
            self.jd[l], gD, fake_kg = self.costs_and_grads(l, z, x, int(self.step[l]), update_running=True)
            self._adam(l, 1, self.D[l], gD)
            self.jg[l], gG = self.g_cost_and_grads(l, fake_kg, int(self.step[l]), update_running=True)
            self._adam(l, 0, self.G[l], gG)
            self.grads[l] = [gG, gD]
