"""Seeded synthetic workloads: architecture descriptors, initial parameters, labels, images, noise.

This module holds none of the method's arithmetic.  It describes the five
workloads (shapes and class counts of the paper's four datasets, Section 3),
draws every random number the method consumes (initial parameters, z
minibatches, stand-in images) with numpy, and hands identical arrays to
whichever implementation is asked to run a step.

The paper's datasets are not available; the images below only have their
shapes and class counts and stand in for them.
"""
import numpy as np

BASE_SEED = 210210485

# z_dim 100 everywhere (the paper's generator tables: input 100, or 110 = 100 + 10 when conditioned)
SPECS = {
    # 28x28x1, ten classes: conditional pair(s)
    "mnist": dict(cond_g=10, cond_d=10, z_dim=100, img_c=1, img_hw=28, g_h0=7, g_ch=[128, 64], d_ch=[64, 128]),
    # 32x32x3, hundred classes: unconditional generator, label maps on the discriminator input
    "cifar": dict(cond_g=0, cond_d=100, z_dim=100, img_c=3, img_hw=32, g_h0=4, g_ch=[512, 256, 128],
                  d_ch=[128, 256, 512]),
    # 64x64x3, one GPU's share of a thousand classes: plain DCGAN widths
    "imagenet": dict(cond_g=0, cond_d=0, z_dim=100, img_c=3, img_hw=64, g_h0=4, g_ch=[512, 256, 128, 64],
                     d_ch=[64, 128, 256, 512]),
    # small nets for unit tests (channel counts that still span MFMA tiles)
    "tiny": dict(cond_g=4, cond_d=4, z_dim=12, img_c=1, img_hw=8, g_h0=2, g_ch=[64, 64], d_ch=[64, 128]),
    "tiny3": dict(cond_g=0, cond_d=3, z_dim=20, img_c=3, img_hw=16, g_h0=2, g_ch=[128, 64, 64], d_ch=[64, 128, 64]),
    # one conditional pair over twenty labels (the paper's single-pair DC-CGAN at test size)
    "tiny20": dict(cond_g=20, cond_d=20, z_dim=12, img_c=3, img_hw=16, g_h0=2, g_ch=[128, 64, 64], d_ch=[64, 128, 64]),
    "tiny0": dict(cond_g=0, cond_d=0, z_dim=20, img_c=3, img_hw=16, g_h0=2, g_ch=[128, 64, 128], d_ch=[128, 64, 64]),
    "micro": dict(cond_g=2, cond_d=2, z_dim=3, img_c=1, img_hw=4, g_h0=1, g_ch=[3, 2], d_ch=[2, 3]),
    # the networks exactly as the paper's Tables 1 and 2 print them (Upsample + Conv k3 generator; Conv k3 s2 +
    # LeakyReLU + Dropout + BatchNorm discriminator with 16/32/64/128 channels), unconditional, one pair per label
    "paper32": dict(family="paper", cond_g=0, cond_d=0, z_dim=100, img_c=3, img_hw=32, g_h0=8, g_ch=[128, 128, 64],
                    d_ch=[16, 32, 64, 128]),
    "paper16": dict(family="paper", cond_g=0, cond_d=0, z_dim=24, img_c=3, img_hw=16, g_h0=4, g_ch=[64, 128, 64],
                    d_ch=[16, 32, 72]),
    # the same family at shapes that reach the other paths of its image-side kernels: one image channel, a side that
    # is not a multiple of the 8-pixel patches, 128 feature channels in front of the image; and four image channels
    "paper28": dict(family="paper", cond_g=0, cond_d=0, z_dim=16, img_c=1, img_hw=28, g_h0=7, g_ch=[128, 64, 128],
                    d_ch=[16, 32]),
    "paper16c4": dict(family="paper", cond_g=0, cond_d=0, z_dim=16, img_c=4, img_hw=16, g_h0=4, g_ch=[64, 64, 64],
                      d_ch=[16, 32]),
}

# name -> (spec, n_models, n_labels, per-label batch, precision)
CONFIGS = {
    0: dict(spec="mnist", n_models=1, n_labels=10, batch=64, precision="fp32", steps=5),
    1: dict(spec="mnist", n_models=10, n_labels=10, batch=128, precision="fp32", steps=200),
    2: dict(spec="cifar", n_models=100, n_labels=100, batch=64, precision="bf16", steps=3),
    3: dict(spec="imagenet", n_models=8, n_labels=8, batch=128, precision="bf16", steps=3),
    4: dict(spec="cifar", n_models=100, n_labels=100, batch="zipf", precision="bf16", steps=3),
}


def param_tensors(spec, which):
    """Tensors of one network in the documented flat order: list of (name, shape, kind).

    kind is 'w' (weight, N(0, 0.02)), 'b' (bias, 0), 'gamma' (1) or 'beta' (0).
    Layers followed by BatchNorm have no bias.
    """
    out = []
    if spec.get("family") == "paper":
        return _paper_tensors(spec, which)
    if which == 0:
        g_ch, h0 = spec["g_ch"], spec["g_h0"]
        out.append(("fc.w", (g_ch[0] * h0 * h0, spec["z_dim"] + spec["cond_g"]), "w"))
        out.append(("bn0.gamma", (g_ch[0],), "gamma"))
        out.append(("bn0.beta", (g_ch[0],), "beta"))
        for i in range(1, len(g_ch) + 1):
            cin = g_ch[i - 1]
            cout = g_ch[i] if i < len(g_ch) else spec["img_c"]
            out.append(("ct%d.w" % i, (cin, cout, 4, 4), "w"))
            if i < len(g_ch):
                out.append(("bn%d.gamma" % i, (cout,), "gamma"))
                out.append(("bn%d.beta" % i, (cout,), "beta"))
            else:
                out.append(("ct%d.b" % i, (cout,), "b"))
    else:
        d_ch = spec["d_ch"]
        h = spec["img_hw"]
        for j, cout in enumerate(d_ch):
            cin = spec["img_c"] + spec["cond_d"] if j == 0 else d_ch[j - 1]
            out.append(("c%d.w" % (j + 1), (cout, cin, 4, 4), "w"))
            if j == 0:
                out.append(("c1.b", (cout,), "b"))
            else:
                out.append(("bn%d.gamma" % (j + 1), (cout,), "gamma"))
                out.append(("bn%d.beta" % (j + 1), (cout,), "beta"))
            h //= 2
        out.append(("fc.w", (1, d_ch[-1] * h * h), "w"))
        out.append(("fc.b", (1,), "b"))
    return out


def _paper_tensors(spec, which):
    """The networks of the paper's Tables 1 and 2 (every conv of D and the two ends of G carry a bias; a layer
    directly followed by BatchNorm does not)."""
    out = []
    if which == 0:
        g_ch, h0 = spec["g_ch"], spec["g_h0"]
        out += [("fc.w", (g_ch[0] * h0 * h0, spec["z_dim"]), "w"), ("fc.b", (g_ch[0] * h0 * h0,), "b"),
                ("bn0.gamma", (g_ch[0],), "gamma"), ("bn0.beta", (g_ch[0],), "beta")]
        for i in range(1, len(g_ch)):
            out += [("conv%d.w" % i, (g_ch[i], g_ch[i - 1], 3, 3), "w"), ("bn%d.gamma" % i, (g_ch[i],), "gamma"),
                    ("bn%d.beta" % i, (g_ch[i],), "beta")]
        n = len(g_ch)
        out += [("conv%d.w" % n, (spec["img_c"], g_ch[-1], 3, 3), "w"), ("conv%d.b" % n, (spec["img_c"],), "b")]
    else:
        cin, h = spec["img_c"], spec["img_hw"]
        for j, c in enumerate(spec["d_ch"], 1):
            out += [("conv%d.w" % j, (c, cin, 3, 3), "w"), ("conv%d.b" % j, (c,), "b")]
            if j > 1:
                out += [("bn%d.gamma" % j, (c,), "gamma"), ("bn%d.beta" % j, (c,), "beta")]
            cin, h = c, h // 2
        out += [("fc.w", (1, cin * h * h), "w"), ("fc.b", (1,), "b")]
    return out


def param_count(spec, which):
    return int(sum(int(np.prod(s)) for _, s, _ in param_tensors(spec, which)))


def param_slices(spec, which):
    """name -> (slice into the flat vector, shape)."""
    out, o = {}, 0
    for name, shape, _ in param_tensors(spec, which):
        n = int(np.prod(shape))
        out[name] = (slice(o, o + n), shape)
        o += n
    return out


def init_params(spec, which, rng, std=0.02):
    parts = []
    for _, shape, kind in param_tensors(spec, which):
        n = int(np.prod(shape))
        if kind == "w":
            parts.append(rng.normal(0.0, std, n))
        elif kind == "gamma":
            parts.append(np.ones(n))
        else:
            parts.append(np.zeros(n))
    return np.concatenate(parts).astype(np.float32)


def blob_images(labels, rng, hw=28, n_labels=10):
    """One bright Gaussian blob per image, centre on a circle indexed by the label (28x28x1 stand-in)."""
    labels = np.asarray(labels)
    n = labels.size
    ang = 2.0 * np.pi * labels / float(n_labels)
    cy = hw / 2.0 + (hw * 2.0 / 7.0) * np.cos(ang) + rng.normal(0.0, 1.0, n)
    cx = hw / 2.0 + (hw * 2.0 / 7.0) * np.sin(ang) + rng.normal(0.0, 1.0, n)
    yy, xx = np.meshgrid(np.arange(hw), np.arange(hw), indexing="ij")
    r2 = (yy[None] - cy[:, None, None]) ** 2 + (xx[None] - cx[:, None, None]) ** 2
    img = np.exp(-r2 / (2.0 * 3.0 ** 2))
    return (2.0 * img - 1.0)[:, None, :, :].astype(np.float32)


def field_images(labels, rng, hw=32, channels=3, sigma=2.0, n_labels=100, offset_seed=BASE_SEED):
    """Smooth random fields: low-passed white noise plus a per-(label, channel) offset, squashed to (-1, 1)."""
    labels = np.asarray(labels)
    n = labels.size
    off_rng = np.random.default_rng(offset_seed + 7919)
    offsets = off_rng.uniform(-0.5, 0.5, (n_labels, channels))
    f = np.fft.fftfreq(hw)
    g = np.exp(-2.0 * (np.pi * sigma) ** 2 * (f[:, None] ** 2 + f[None, :] ** 2))   # Gaussian low-pass, periodic
    white = rng.normal(0.0, 1.0, (n, channels, hw, hw))
    sm = np.fft.ifft2(np.fft.fft2(white) * g[None, None]).real
    sm /= np.sqrt(np.sum(g ** 2) / (hw * hw))                                       # back to unit variance
    sm += offsets[labels][:, :, None, None]
    return np.tanh(sm).astype(np.float32)


def zipf_batches(n_models, total, lo=8, hi=256, s=1.1):
    """Rank-size batch sizes b_r = clip(round(C r^-s), lo, hi) with C chosen so that they sum to `total`."""
    r = np.arange(1, n_models + 1, dtype=np.float64)

    def sizes(c):
        return np.clip(np.round(c * r ** (-s)), lo, hi).astype(np.int64)

    a, b = 1.0, 1e7
    for _ in range(200):
        mid = 0.5 * (a + b)
        if sizes(mid).sum() < total:
            a = mid
        else:
            b = mid
    out = sizes(b)
    # absorb any rounding remainder in the largest unclipped entries
    i = 0
    while out.sum() != total and i < 10 * n_models:
        j = i % n_models
        d = int(np.sign(total - out.sum()))
        if lo <= out[j] + d <= hi:
            out[j] += d
        i += 1
    return out


class Workload:
    """Everything one configuration needs, drawn from fixed sub-streams of one seed."""

    def __init__(self, config_id, n_models=None, batch=None, spec=None, n_labels=None, seed=None):
        cfg = dict(CONFIGS[config_id]) if config_id in CONFIGS else {}
        self.config_id = config_id
        self.spec_name = spec or cfg["spec"]
        self.spec = SPECS[self.spec_name]
        self.n_models = n_models if n_models is not None else cfg["n_models"]
        self.n_labels = n_labels if n_labels is not None else (cfg.get("n_labels") if n_models is None else
                                                               max(self.n_models, 1))
        if self.n_models > 1:
            self.n_labels = self.n_models
        batch = batch if batch is not None else cfg["batch"]
        self.precision = cfg.get("precision", "fp32")
        self.seed = seed if seed is not None else BASE_SEED + (config_id if isinstance(config_id, int) else 99)
        root = np.random.default_rng(self.seed)
        self.rng_params, self.rng_labels, self.rng_images, self.rng_noise = root.spawn(4)
        if isinstance(batch, str):
            sizes = zipf_batches(self.n_models, 64 * self.n_models)
            self.batch_sizes = sizes[self.rng_labels.permutation(self.n_models)]
        elif self.n_models == 1:
            self.batch_sizes = np.array([batch])
        else:
            self.batch_sizes = np.full(self.n_models, batch, dtype=np.int64)
        self.n = int(self.batch_sizes.sum())

    def params(self, which, model):
        """Initial parameters of one model; reproducible per (which, model)."""
        rng = np.random.default_rng([self.seed, 11 + which, model])
        return init_params(self.spec, which, rng)

    def labels(self, single_label=None):
        """Flat label vector of one step: a seeded shuffle of the per-label groups."""
        if self.n_models == 1:
            if single_label is not None:
                return np.full(self.n, single_label, np.int32)
            return self.rng_labels.integers(0, self.n_labels, self.n).astype(np.int32)
        lab = np.repeat(np.arange(self.n_models), self.batch_sizes).astype(np.int32)
        return lab[self.rng_labels.permutation(self.n)]

    def images(self, labels):
        s = self.spec
        if s["img_c"] == 1:
            return blob_images(labels, self.rng_images, hw=s["img_hw"], n_labels=max(self.n_labels, 1))
        sigma = 2.0 * s["img_hw"] / 32.0
        return field_images(labels, self.rng_images, hw=s["img_hw"], channels=s["img_c"], sigma=sigma,
                            n_labels=max(self.n_labels, 1), offset_seed=self.seed)

    def noise(self, n=None):
        return self.rng_noise.normal(0.0, 1.0, (n or self.n, self.spec["z_dim"])).astype(np.float32)
