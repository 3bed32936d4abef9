"""Pins of the oracle for the networks as printed in the paper's Tables 1 and 2 (oracle/paper_nets.py): the published
known-answer vectors of the dropout generator, the adjoint and closed forms of the upsampling, the identity that
maps Upsample x2 + Conv k3 p1 onto a k4 s2 p1 transposed convolution, finite differences of both costs through the
whole pair, Adam's closed-form first step, and the independence of the label models (Eq. 5).  CPU only.
"""
import numpy as np
import pytest

import oracle as O
from oracle import paper_nets as P


def test_philox_known_answers():
    """Philox-4x32-10 known-answer vectors published with the generator (Salmon et al., SC'11, test vector file)."""
    kat = [((0, 0, 0, 0), (0, 0), (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)),
           ((0xffffffff,) * 4, (0xffffffff,) * 2, (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)),
           ((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0),
            (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1))]
    for ctr, key, want in kat:
        got = tuple(int(w) for w in P.philox4x32_10(*ctr, *key))
        assert got == want
    # vectorised call == element by element
    c0 = np.arange(5, dtype=np.uint32)
    many = P.philox4x32_10(c0, 7, 9, 11, 13, 17)
    for i in range(5):
        one = P.philox4x32_10(i, 7, 9, 11, 13, 17)
        assert all(int(many[w][i]) == int(one[w]) for w in range(4))


def test_dropout_mask_properties():
    shape = (6, 8, 16, 16)
    a = P.dropout_keep(shape, 0.25, seed=5, model=1, step=3, layer=2, pass_id=0)
    assert a.dtype == bool and a.shape == shape
    assert np.array_equal(a, P.dropout_keep(shape, 0.25, 5, 1, 3, 2, 0))               # a pure function of its arguments
    assert abs(a.mean() - 0.75) < 0.02                                                  # 12288 draws: sigma = 0.004
    for other in (P.dropout_keep(shape, 0.25, 5, 1, 3, 2, 1), P.dropout_keep(shape, 0.25, 5, 1, 4, 2, 0),
                  P.dropout_keep(shape, 0.25, 5, 2, 3, 2, 0), P.dropout_keep(shape, 0.25, 6, 1, 3, 2, 0),
                  P.dropout_keep(shape, 0.25, 5, 1, 3, 3, 0)):
        assert 0.55 < (a == other).mean() < 0.70                                        # independent masks agree in 62.5 %
    assert P.dropout_keep(shape, 0.0, 5, 1, 3, 2, 0).all()
    # the mask of a sample does not depend on how many samples follow it
    assert np.array_equal(a[:2], P.dropout_keep((2,) + shape[1:], 0.25, 5, 1, 3, 2, 0))
    # element i takes output word i % 4 of counter i // 4: the four words of a counter are four different draws (the
    # decisions inside a group of four are as independent as across groups), a length that is not a multiple of four
    # just stops early, and the elements 4..7 are the four words of counter 1
    flat = a.reshape(-1)
    g = flat.reshape(-1, 4)
    for u, v in ((0, 1), (1, 2), (2, 3), (0, 3)):
        assert 0.55 < (g[:, u] == g[:, v]).mean() < 0.70
    assert np.array_equal(flat[:13], P.dropout_keep((13, 1, 1, 1), 0.25, 5, 1, 3, 2, 0).reshape(-1))
    words = P.philox4x32_10(1, 0, 2, 3, 5, 1)                                           # counter (1, 0, layer, step), key (seed, model)
    assert [bool((int(w) >> 8) >= 4194304) for w in words] == [bool(b) for b in flat[4:8]]


def test_upsample_and_its_adjoint():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(2, 3, 4, 5))
    u = P.upsample2(x)
    assert u.shape == (2, 3, 8, 10)
    for a in (0, 1):
        for b in (0, 1):
            assert np.array_equal(u[:, :, a::2, b::2], x)
    y = rng.normal(size=u.shape)
    assert abs(np.sum(u * y) - np.sum(x * P.upsample2_bwd(y))) < 1e-12 * np.sum(np.abs(u * y))


def test_upsample_conv3_is_a_transposed_convolution_with_summed_taps():
    """Upsample x2 followed by Conv k3 s1 p1 equals ConvTranspose k4 s2 p1 with W4 = A W3 A^T per channel pair."""
    rng = np.random.default_rng(1)
    x = rng.normal(size=(2, 3, 5, 5))
    w3 = rng.normal(size=(4, 3, 3, 3))                                                   # [cout][cin][ky][kx]
    ref = O.conv2d(P.upsample2(x), w3, None, 3, 1, 1)
    A = np.array([[0, 0, 1], [0, 1, 1], [1, 1, 0], [1, 0, 0]], float)
    w4 = np.einsum("ak,oikl,bl->ioab", A, w3, A)                                         # [cin][cout][4][4]
    got = O.conv_transpose2d(x, w4, None, 4, 2, 1)
    assert np.max(np.abs(got - ref)) < 1e-12 * np.max(np.abs(ref))


def small_nets(K=1, seed=0):
    nets = P.PaperNets(img_c=2, img_hw=8, n_models=K, z_dim=5, g_ch=(4, 4, 3), d_ch=(2, 3, 4, 5), seed=11)
    rng = np.random.default_rng(seed)
    for l in range(K):
        nets.set_params(0, l, P.init_params(nets.gs, rng, std=0.3))
        pd = P.init_params(nets.ds, rng, std=0.3)
        for k in pd:                                          # biases and BatchNorm parameters away from their defaults
            if not k.endswith(".w"):
                pd[k] = pd[k] + rng.normal(0, 0.2, pd[k].shape)
        nets.set_params(1, l, pd)
    return nets


def test_shapes_of_the_printed_tables():
    """Table 1: 100 -> 8192 = 128 * 8 * 8, convolutions 128 -> 128 -> 64 -> 3; Table 2: 3 -> 16 -> 32 -> 64 -> 128."""
    gs = dict(P.g_shapes(3, 32, 100, (128, 128, 64)))
    assert gs["fc.w"] == (8192, 100) and gs["conv1.w"] == (128, 128, 3, 3) and gs["conv2.w"] == (64, 128, 3, 3)
    assert gs["conv3.w"] == (3, 64, 3, 3)
    ds = dict(P.d_shapes(3, 64, (16, 32, 64, 128)))
    assert ds["fc.w"] == (1, 2048)                            # the 2048 inputs Table 2 prints belong to 64 x 64 images
    assert dict(P.d_shapes(3, 32, (16, 32, 64, 128)))["fc.w"] == (1, 512)
    nets = small_nets()
    rng = np.random.default_rng(2)
    out, _ = nets.g_forward(nets.G[0], rng.normal(size=(3, 5)))
    assert out.shape == (3, 2, 8, 8) and np.all(np.abs(out) < 1)
    s, _ = nets.d_forward(nets.D[0], out, 0, 1, 0)
    assert s.shape == (3,)


def test_costs_at_zero_logits():
    """With D's last layer zeroed every logit is 0: J_D = 2 * (1/2) ln 2, J_G = (1/2) ln 2 (Eq. 3, Eq. 4)."""
    nets = small_nets()
    nets.D[0]["fc.w"][:] = 0
    nets.D[0]["fc.b"][:] = 0
    rng = np.random.default_rng(3)
    z, x = rng.normal(size=(6, 5)), np.tanh(rng.normal(size=(6, 2, 8, 8)))
    jd, _, fk = nets.costs_and_grads(0, z, x, 1)
    jg, _ = nets.g_cost_and_grads(0, fk, 1)
    assert abs(jd - np.log(2)) < 1e-12 and abs(jg - 0.5 * np.log(2)) < 1e-12


@pytest.mark.parametrize("which", [0, 1])
def test_gradients_by_finite_differences(which):
    """dJ_D/dtheta_D and dJ_G/dtheta_G through the whole pair (dropout masks fixed by (step, pass), BatchNorm in
    training mode with the printed epsilons) against central differences in fp64."""
    nets = small_nets()
    rng = np.random.default_rng(4)
    z, x = rng.normal(size=(7, 5)), np.tanh(rng.normal(size=(7, 2, 8, 8)))

    def cost():
        jd, gD, fk = nets.costs_and_grads(0, z, x, 2)
        if which == 1:
            return jd, gD
        jg, gG = nets.g_cost_and_grads(0, fk, 2)
        return jg, gG

    _, grads = cost()
    params = nets.G[0] if which == 0 else nets.D[0]
    h = 1e-6
    checked = 0
    for name, g in grads.items():
        flat = params[name].reshape(-1)
        for i in rng.choice(flat.size, size=min(4, flat.size), replace=False):
            old = flat[i]
            flat[i] = old + h
            jp, _ = cost()
            flat[i] = old - h
            jm, _ = cost()
            flat[i] = old
            fd = (jp - jm) / (2 * h)
            assert abs(fd - g.reshape(-1)[i]) <= 2e-6 * max(1.0, abs(fd)) + 1e-8, (name, int(i), fd, g.reshape(-1)[i])
            checked += 1
    assert checked >= 30


def test_first_adam_step_moves_every_parameter_by_lr():
    nets = small_nets()
    rng = np.random.default_rng(5)
    z, x = rng.normal(size=(9, 5)), np.tanh(rng.normal(size=(9, 2, 8, 8)))
    before = [{k: v.copy() for k, v in nets.G[0].items()}, {k: v.copy() for k, v in nets.D[0].items()}]
    nets.train_step(np.zeros(9, np.int32), z, x)
    for which, params in ((0, nets.G[0]), (1, nets.D[0])):
        for name, v in params.items():
            g = nets.grads[0][which][name]
            big = np.abs(g) > 1e-4                                # |g| >> adam_eps: the step is lr * sign(g) exactly
            step = v - before[which][name]
            assert np.allclose(step[big], -2e-4 * np.sign(g[big]), rtol=1e-3, atol=0)
            assert np.all(step[g == 0] == 0)
    assert nets.jd[0] > 0 and nets.jg[0] > 0 and nets.counts[0] == 9


def test_label_models_are_independent():
    """Eq. 5: the pairs never exchange anything -- two models in one call equal each model stepped on its own."""
    rng = np.random.default_rng(6)
    lab = rng.integers(0, 2, 12).astype(np.int32)
    z, x = rng.normal(size=(12, 5)), np.tanh(rng.normal(size=(12, 2, 8, 8)))
    both = small_nets(K=2)
    both.train_step(lab, z, x)
    for l in (0, 1):
        solo = small_nets(K=2)
        sel = np.flatnonzero(lab == l)
        solo.train_step(lab[sel], z[sel], x[sel])
        for which, a, b in ((0, both.G[l], solo.G[l]), (1, both.D[l], solo.D[l])):
            for name in a:
                assert np.array_equal(a[name], b[name])
        assert both.jd[l] == solo.jd[l] and both.jg[l] == solo.jg[l]
        other = 1 - l
        assert solo.counts[other] == 0 and solo.t[other].sum() == 0


def test_discriminator_block_order_and_dropout_scaling():
    """Table 2's block is Conv -> LeakyReLU -> Dropout -> BatchNorm: kept values are scaled by 1 / (1 - p), dropped
    ones are exactly zero before the normalisation, and the normalised output has the BatchNorm moments."""
    nets = small_nets()
    rng = np.random.default_rng(7)
    x = np.tanh(rng.normal(size=(16, 2, 8, 8)))
    p = nets.D[0]
    _, k = nets.d_forward(p, x, 0, 1, 0)
    a1 = O.leaky_relu(O.conv2d(x, p["conv1.w"], p["conv1.b"], 3, 2, 1), 0.2)
    keep = P.dropout_keep(a1.shape, 0.25, nets.seed, 0, 1, 1, 0)
    assert np.all(k["d1"][~keep] == 0) and np.allclose(k["d1"][keep], a1[keep] / 0.75, rtol=1e-14, atol=0)
    assert np.array_equal(k["in2"], k["d1"])                            # no BatchNorm after the first block
    for j in (2, 3, 4):
        d = k["d%d" % j]
        keep = P.dropout_keep(d.shape, 0.25, nets.seed, 0, 1, j, 0)
        assert np.all(d[~keep] == 0)
        y = k["in%d" % (j + 1)] if j < 4 else k["flat"].reshape(k["shape"])
        xhat = (y - p["bn%d.beta" % j][None, :, None, None]) / p["bn%d.gamma" % j][None, :, None, None]
        var = d.var(axis=(0, 2, 3))
        assert np.allclose(xhat.mean(axis=(0, 2, 3)), 0, atol=1e-12)
        assert np.allclose(xhat.var(axis=(0, 2, 3)), var / (var + 0.8), rtol=1e-10)        # epsilon = 0.8 as printed
    # evaluation mode: no dropout
    _, ke = nets.d_forward(p, x, 0, 1, 0, train=False)
    assert np.array_equal(ke["d1"], a1)


def test_generator_block_order():
    """Table 1: Linear -> ReLU -> BatchNorm(1e-5) -> [Upsample -> Conv -> BatchNorm(0.8) -> LeakyReLU] x 2 -> Conv -> tanh."""
    nets = small_nets()
    rng = np.random.default_rng(8)
    z = rng.normal(size=(10, 5))
    p = nets.G[0]
    out, k = nets.g_forward(p, z)
    a0 = z @ p["fc.w"].T + p["fc.b"]
    assert np.allclose(k["x0"].reshape(10, -1), np.maximum(a0, 0), atol=1e-13)
    v0 = k["x0"].var(axis=(0, 2, 3))
    y0 = k["u1"][:, :, ::2, ::2]                                         # the BatchNorm output, read back through the upsampling
    assert np.allclose(y0.var(axis=(0, 2, 3)), v0 / (v0 + 1e-5), rtol=1e-9)
    for j in (1, 2):
        v = k["c%d" % j].var(axis=(0, 2, 3))
        assert np.allclose(k["b%d" % j].var(axis=(0, 2, 3)), v / (v + 0.8), rtol=1e-10)
        assert np.array_equal(k["h%d" % j], np.where(k["b%d" % j] > 0, k["b%d" % j], 0.2 * k["b%d" % j]))
    assert k["u2"].shape[2] == 2 * k["h1"].shape[2] and out.shape[2] == k["h2"].shape[2]
