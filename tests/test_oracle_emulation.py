"""Pins for the oracle's bf16-storage emulation switch (a diagnostic reference next to the plain algorithm).

What fixes it from outside: the format's definition for the rounding function; the switch-off identity; the
generator's and the discriminator's forward passes rebuilt here from the oracle's (separately pinned) single
operations with the rounding written out at every point the header lists, which must agree to the last bits -- a
rounding that is missing, misplaced or doubled anywhere in those passes breaks the equality; representability of
what is stored; and the distance to the plain result staying within the format's error.
"""
import numpy as np

import oracle as O
from paper_2102_10485_amd import synth


def bf16(a):
    """The format's definition on arrays: round to single, then keep the top 16 bits, to nearest, ties to even."""
    f = np.ascontiguousarray(a, np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(a))


def representable(a):
    a = np.asarray(a, np.float64)
    return np.array_equal(bf16(a), a)


def make(spec_name, n_models, n_labels, seed=5, std=0.02, emulate=True):
    spec = synth.SPECS[spec_name]
    orc = O.Oracle(spec, n_models, n_labels, emulate_bf16=emulate)
    rng = np.random.default_rng(seed)
    for l in range(n_models):
        for which in (0, 1):
            orc.set_params(which, l, synth.init_params(spec, which, rng, std=std))
    return spec, orc


def batch(spec, labels, seed=9):
    rng = np.random.default_rng(seed)
    n = len(labels)
    return (np.asarray(labels, np.int32), rng.normal(size=(n, spec["z_dim"])),
            np.tanh(rng.normal(size=(n, spec["img_c"], spec["img_hw"], spec["img_hw"]))))


def test_rounding_function_follows_the_format():
    rng = np.random.default_rng(0)
    vals = np.concatenate([rng.normal(size=2000) * 10.0 ** rng.integers(-20, 20, 2000),
                           [0.0, -0.0, 1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 1.0 + 2.0 ** -8 + 2.0 ** -30,
                            1.0 + 2.0 ** -8 - 2.0 ** -30, 65280.0, 3.3895313892515355e38, 1e-40, np.inf, -np.inf]])
    got = np.array([O.round_bf16(v) for v in vals])
    np.testing.assert_array_equal(got, bf16(vals))
    # ties go to the even mantissa; just above / below a tie goes to the nearer neighbour
    assert O.round_bf16(1.0 + 2.0 ** -8) == 1.0 and O.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert O.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert np.isnan(O.round_bf16(float("nan")))


def test_switch_off_is_the_plain_algorithm_bit_for_bit():
    spec, a = make("tiny", 2, 2, emulate=False)
    _, b = make("tiny", 2, 2, emulate=True)
    assert b.L.oracle_set_bf16_emulation(b.h, 0) == 0
    lab, z, x = batch(spec, [0, 1, 1, 0, 1, 0, 0])
    for _ in range(2):
        a.train_step(lab, z, x)
        b.train_step(lab, z, x)
    for l in range(2):
        for which in (0, 1):
            np.testing.assert_array_equal(a.get_params(which, l), b.get_params(which, l))
    np.testing.assert_array_equal(a.get_losses()[0], b.get_losses()[0])


def _g_forward_by_hand(spec, th, lab, z, eps=1e-5):
    """G's forward pass from the single operations, rounding where a 16-bit-storage implementation stores."""
    sl = synth.param_slices(spec, 0)
    n = len(lab)
    onehot = np.zeros((n, spec["cond_g"]))
    if spec["cond_g"]:
        onehot[np.arange(n), lab] = 1.0
    cur = bf16(np.concatenate([z, onehot], axis=1))
    w = th[sl["fc.w"][0]].reshape(sl["fc.w"][1])
    pre = O.linear(cur, bf16(w)).reshape(n, spec["g_ch"][0], spec["g_h0"], spec["g_h0"])
    _, mean, var = O.bn_train(pre, th[sl["bn0.gamma"][0]], th[sl["bn0.beta"][0]], eps)      # statistics before rounding
    cur = bf16(np.maximum(O.bn_eval(bf16(pre), th[sl["bn0.gamma"][0]], th[sl["bn0.beta"][0]], eps, mean, var), 0.0))
    ng = len(spec["g_ch"])
    for i in range(1, ng + 1):
        w = th[sl["ct%d.w" % i][0]].reshape(sl["ct%d.w" % i][1])
        if i < ng:
            pre = O.conv_transpose2d(cur, bf16(w))
            ga, be = th[sl["bn%d.gamma" % i][0]], th[sl["bn%d.beta" % i][0]]
            _, mean, var = O.bn_train(pre, ga, be, eps)
            cur = bf16(np.maximum(O.bn_eval(bf16(pre), ga, be, eps, mean, var), 0.0))
        else:
            cur = bf16(np.tanh(O.conv_transpose2d(cur, bf16(w), th[sl["ct%d.b" % i][0]])))   # the bias is not rounded
    return cur


def _d_logits_by_hand(spec, th, lab, img, eps=1e-5, slope=0.2):
    sl = synth.param_slices(spec, 1)
    n, C, H = len(lab), spec["img_c"], spec["img_hw"]
    w1 = th[sl["c1.w"][0]].reshape(sl["c1.w"][1])
    out = O.conv2d(bf16(img), bf16(w1[:, :C]))                      # image channels: per-element rounded weights
    Ho = H // 2
    for r in range(n):
        if spec["cond_d"] == 0:
            break
        wl = w1[:, C + lab[r]]                                      # [cout, 4, 4] taps of this sample's label plane
        for oy in range(Ho):
            for ox in range(Ho):
                ky = [k for k in range(4) if 0 <= 2 * oy - 1 + k < H]
                kx = [k for k in range(4) if 0 <= 2 * ox - 1 + k < H]
                out[r, :, oy, ox] += bf16(wl[:, ky][:, :, kx].sum(axis=(1, 2)))   # one rounded sum per position
    out += bf16(th[sl["c1.b"][0]])[None, :, None, None]
    cur = bf16(np.where(out > 0, out, slope * out))
    for j in range(2, len(spec["d_ch"]) + 1):
        w = th[sl["c%d.w" % j][0]].reshape(sl["c%d.w" % j][1])
        pre = O.conv2d(cur, bf16(w))
        ga, be = th[sl["bn%d.gamma" % j][0]], th[sl["bn%d.beta" % j][0]]
        _, mean, var = O.bn_train(pre, ga, be, eps)
        u = O.bn_eval(bf16(pre), ga, be, eps, mean, var)
        cur = bf16(np.where(u > 0, u, slope * u))
    wf = th[sl["fc.w"][0]]                                          # the final linear layer: unrounded weights
    return cur.reshape(n, -1) @ wf + th[sl["fc.b"][0]][0]


def _softplus(u):
    return np.maximum(u, 0) + np.log1p(np.exp(-np.abs(u)))


def test_forward_passes_round_exactly_where_the_header_says():
    for name, nlab in (("micro", 2), ("tiny", 4)):
        spec, orc = make(name, 1, nlab, std=0.3)
        lab, z, x = batch(spec, [0, 1, 1, 0, 1, 0, 1], seed=3)
        thG, thD = orc.get_params(0, 0), orc.get_params(1, 0)
        rc, fake = orc.generate(lab, z)
        want = _g_forward_by_hand(spec, thG, lab, z)
        np.testing.assert_allclose(fake, want, rtol=0, atol=1e-12)
        assert representable(fake)
        # both costs at the current parameters: D on (real, fake) and on fake alone
        jd, jg = orc.eval_losses(0, lab, z, x)
        s_real = _d_logits_by_hand(spec, thD, lab, x)
        s_fake = _d_logits_by_hand(spec, thD, lab, want)
        np.testing.assert_allclose(jd, 0.5 * _softplus(-s_real).mean() + 0.5 * _softplus(s_fake).mean(), rtol=1e-12)
        np.testing.assert_allclose(jg, 0.5 * _softplus(-s_fake).mean(), rtol=1e-12)
        # a plain oracle on the same inputs is NOT equal: the roundings are really there
        _, plain = make(name, 1, nlab, std=0.3, emulate=False)
        assert abs(plain.eval_losses(0, lab, z, x)[0] - jd) > 1e-7
        assert not representable(plain.generate(lab, z)[1])


def test_emulated_step_stays_within_the_formats_error_of_the_plain_step():
    spec, emu = make("tiny3", 2, 2)
    _, ref = make("tiny3", 2, 2, emulate=False)
    lab, z, x = batch(spec, [0, 1, 1, 0, 1, 0, 0, 1, 1, 1, 0, 1], seed=4)
    emu.train_step(lab, z, x)
    ref.train_step(lab, z, x)
    for a, b in zip(emu.get_losses()[:2], ref.get_losses()[:2]):
        assert np.all(np.abs(a - b) <= 2e-2 * np.abs(b)) and np.any(a != b)
    for l in range(2):
        for which in (0, 1):
            ge, gr = emu.get_grads(which, l), ref.get_grads(which, l)
            # (at initialisation the real and the fake half of Eq. 3 nearly cancel, which amplifies the storage rounding
            # to 5-15 % of the small gradient: the reason the 16-bit path is compared with this emulation, not only
            # with the plain result)
            assert ge @ gr / (np.linalg.norm(ge) * np.linalg.norm(gr)) > 0.98
            assert not representable(ge)               # parameter gradients are left unrounded
            # the master parameters and Adam stay in full precision: the update is Adam's on the emulated gradient
            m, v, t = emu.get_opt_state(which, l)
            np.testing.assert_allclose(m, 0.5 * ge, rtol=1e-12)
            np.testing.assert_allclose(v, 0.001 * ge * ge, rtol=1e-9)
            assert t == 1
