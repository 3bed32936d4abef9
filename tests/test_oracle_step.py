"""Pins for the oracle's whole training iteration (Section 2: Eq. 3, Eq. 4, Adam; Eq. 5 independence)."""
import math

import numpy as np
import pytest

import oracle as O
from paper_2102_10485_amd import synth


def make(spec_name, n_models, n_labels, seed=5, hyper=None, std=0.02):
    spec = synth.SPECS[spec_name]
    orc = O.Oracle(spec, n_models, n_labels, hyper)
    rng = np.random.default_rng(seed)
    for l in range(n_models):
        for which in (0, 1):
            assert orc.param_count(which) == synth.param_count(spec, which)
            orc.set_params(which, l, synth.init_params(spec, which, rng, std=std))
    return spec, orc


def batch(spec, labels, seed=9):
    rng = np.random.default_rng(seed)
    n = len(labels)
    noise = rng.normal(size=(n, spec["z_dim"]))
    real = np.tanh(rng.normal(size=(n, spec["img_c"], spec["img_hw"], spec["img_hw"])))
    return np.asarray(labels, np.int32), noise, real


def test_first_step_losses_near_log2():
    # with near-zero weights every logit is ~0, so J_D ~ log 2 and -J_G ~ (1/2) log 2
    spec, orc = make("tiny", 1, 4, std=1e-4)
    lab, z, x = batch(spec, [0, 1, 2, 3, 1, 2, 0, 3])
    assert orc.train_step(lab, z, x) == 0
    jd, jg, cnt = orc.get_losses()
    assert cnt[0] == 8
    assert abs(jd[0] - math.log(2.0)) < 1e-5
    assert abs(jg[0] - 0.5 * math.log(2.0)) < 2e-3      # D has already taken one Adam step of size lr


def test_whole_cost_gradients_by_finite_differences():
    spec, orc = make("micro", 1, 2, std=0.5)
    lab, z, x = batch(spec, [0, 1, 1, 0, 1])
    gD, gG = orc.eval_grads(0, lab, z, x)
    h = 1e-5
    rng = np.random.default_rng(0)
    for which, g in ((1, gD), (0, gG)):
        th = orc.get_params(which, 0)
        for j in rng.choice(th.size, size=min(th.size, 40), replace=False):
            tp, tm = th.copy(), th.copy()
            tp[j] += h
            tm[j] -= h
            orc.set_params(which, 0, tp)
            lp = orc.eval_losses(0, lab, z, x)[0 if which == 1 else 1]
            orc.set_params(which, 0, tm)
            lm = orc.eval_losses(0, lab, z, x)[0 if which == 1 else 1]
            fd = (lp - lm) / (2 * h)
            assert abs(fd - g[j]) < 1e-6 * max(1.0, abs(fd)) + 1e-9, (which, j, fd, g[j])
        orc.set_params(which, 0, th)
        # directional derivative along a random direction V: <g, V> = d/dt J(theta + tV)
        V = rng.normal(size=th.size)
        orc.set_params(which, 0, th + h * V)
        lp = orc.eval_losses(0, lab, z, x)[0 if which == 1 else 1]
        orc.set_params(which, 0, th - h * V)
        lm = orc.eval_losses(0, lab, z, x)[0 if which == 1 else 1]
        orc.set_params(which, 0, th)
        assert abs((lp - lm) / (2 * h) - g @ V) < 1e-6 * max(1.0, abs(g @ V))


def test_step_applies_adam_to_those_gradients():
    spec, orc = make("micro", 1, 2, std=0.5)
    lab, z, x = batch(spec, [0, 1, 1, 0, 1])
    gD, _ = orc.eval_grads(0, lab, z, x)
    thD0, thG0 = orc.get_params(1, 0), orc.get_params(0, 0)
    orc.train_step(lab, z, x)
    np.testing.assert_allclose(orc.get_grads(1, 0), gD, rtol=1e-13, atol=1e-15)
    thD1, thG1 = orc.get_params(1, 0), orc.get_params(0, 0)
    np.testing.assert_allclose(thD1, thD0 - 2e-4 * gD / (np.abs(gD) + 1e-8), rtol=1e-12, atol=1e-15)
    # G's gradient is taken through the UPDATED discriminator: compare with a second context at (thG0, thD1)
    _, orc2 = make("micro", 1, 2, std=0.5)
    orc2.set_params(1, 0, thD1)
    orc2.set_params(0, 0, thG0)
    _, gG2 = orc2.eval_grads(0, lab, z, x)
    np.testing.assert_allclose(orc.get_grads(0, 0), gG2, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(thG1, thG0 - 2e-4 * gG2 / (np.abs(gG2) + 1e-8), rtol=1e-12, atol=1e-15)
    _, _, tD = orc.get_opt_state(1, 0)
    _, _, tG = orc.get_opt_state(0, 0)
    assert tD == 1 and tG == 1


def test_models_are_independent_bitwise():
    # Eq. 5: the K label models never interact, so K models stepped together equal K separate single runs
    K = 3
    spec = synth.SPECS["tiny"]
    hyper = None
    rng = np.random.default_rng(77)
    lab = np.array([2, 0, 1, 1, 2, 0, 0, 2, 1, 2, 2, 0], np.int32)
    n = lab.size
    pg = [synth.init_params(spec, 0, rng) for _ in range(K)]
    pd = [synth.init_params(spec, 1, rng) for _ in range(K)]
    steps = [batch(spec, lab, seed=100 + s) for s in range(3)]
    big = O.Oracle(spec, K, K, hyper)
    for l in range(K):
        big.set_params(0, l, pg[l])
        big.set_params(1, l, pd[l])
    for lab_, z, x in steps:
        assert big.train_step(lab_, z, x) == 0
    perm, offs = big.get_routing(n)
    assert list(offs) == [0, 4, 7, 12]
    for l in range(K):
        # a one-model context that sees only label l's samples, conditioned on the same one-hot
        one = O.Oracle(spec, 1, K, hyper)
        one.set_params(0, 0, pg[l])
        one.set_params(1, 0, pd[l])
        sel = np.flatnonzero(lab == l)
        assert list(perm[offs[l]:offs[l + 1]]) == list(sel)
        for lab_, z, x in steps:
            one.train_step(lab_[sel], z[sel], x[sel])
        for which in (0, 1):
            assert np.array_equal(one.get_params(which, 0), big.get_params(which, l))
        assert one.get_losses()[0][0] == big.get_losses()[0][l]
        for which in (0, 1):
            a, b = one.get_bn_running(which, 0), big.get_bn_running(which, l)
            assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_empty_model_is_untouched_and_only_model():
    spec, orc = make("tiny", 3, 3)
    lab, z, x = batch(spec, [0, 2, 2, 0, 0, 2])
    before = [orc.get_params(w, 1) for w in (0, 1)]
    assert orc.train_step(lab, z, x) == 0
    jd, jg, cnt = orc.get_losses()
    assert list(cnt) == [3, 0, 3] and jd[1] == 0 and jg[1] == 0
    for w in (0, 1):
        assert np.array_equal(before[w], orc.get_params(w, 1))
        assert orc.get_opt_state(w, 1)[2] == 0 and orc.get_opt_state(w, 0)[2] == 1
    # only_model: same result for that model, the others not stepped
    spec, a = make("tiny", 3, 3)
    a.train_step(lab, z, x, only_model=2)
    assert np.array_equal(a.get_params(0, 2), orc.get_params(0, 2))
    assert a.get_opt_state(0, 0)[2] == 0
    # out-of-range labels are dropped and reported
    lab2 = lab.copy()
    lab2[1] = 7
    assert a.train_step(lab2, z, x) == -5


def test_generate_matches_training_forward_and_running_stats():
    spec, orc = make("tiny", 2, 2)
    lab, z, x = batch(spec, [0, 1, 1, 0, 0, 1, 1, 0])
    rc, img = orc.generate(lab, z)
    assert rc == 0 and img.shape == (8, 1, 8, 8) and np.all(np.abs(img) < 1)
    # generation is per model: generating model 1's rows alone gives the same images
    sel = np.flatnonzero(lab == 1)
    _, img1 = orc.generate(lab[sel], z[sel])
    np.testing.assert_array_equal(img[sel], img1)
    orc.train_step(lab, z, x)
    rm, rv = orc.get_bn_running(0, 0)
    assert not np.allclose(rm, 0) and not np.allclose(rv, 1)
    rc, img_run = orc.generate(lab, z, use_running_stats=1)
    assert rc == 0 and not np.allclose(img_run, orc.generate(lab, z)[1])


def test_whole_step_against_autograd_library():
    """The same two networks, costs and optimiser assembled from an independent library's CPU operators
    (used as black boxes, double precision), three iterations, mixed labels in one conditional pair."""
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    spec, orc = make("tiny", 1, 4, std=0.2)
    sl_g, sl_d = synth.param_slices(spec, 0), synth.param_slices(spec, 1)

    def tensors(flat, slices):
        return {k: torch.tensor(flat[s].reshape(shape), dtype=torch.float64, requires_grad=True)
                for k, (s, shape) in slices.items()}

    pg, pd = tensors(orc.get_params(0, 0), sl_g), tensors(orc.get_params(1, 0), sl_d)
    og = torch.optim.Adam(list(pg.values()), lr=2e-4, betas=(0.5, 0.999), eps=1e-8)
    od = torch.optim.Adam(list(pd.values()), lr=2e-4, betas=(0.5, 0.999), eps=1e-8)
    n_g, n_d = len(spec["g_ch"]), len(spec["d_ch"])

    def bn(x, g, b):
        return F.batch_norm(x, None, None, g, b, training=True, eps=1e-5)

    def G(z, onehot):
        h = F.linear(torch.cat([z, onehot], 1), pg["fc.w"]).view(-1, spec["g_ch"][0], spec["g_h0"], spec["g_h0"])
        h = F.relu(bn(h, pg["bn0.gamma"], pg["bn0.beta"]))
        for i in range(1, n_g + 1):
            if i < n_g:
                h = F.conv_transpose2d(h, pg["ct%d.w" % i], None, stride=2, padding=1)
                h = F.relu(bn(h, pg["bn%d.gamma" % i], pg["bn%d.beta" % i]))
            else:
                h = torch.tanh(F.conv_transpose2d(h, pg["ct%d.w" % i], pg["ct%d.b" % i], stride=2, padding=1))
        return h

    def D(x, onehot):
        maps = onehot[:, :, None, None].expand(-1, -1, x.shape[2], x.shape[3])
        h = F.leaky_relu(F.conv2d(torch.cat([x, maps], 1), pd["c1.w"], pd["c1.b"], stride=2, padding=1), 0.2)
        for j in range(2, n_d + 1):
            h = F.conv2d(h, pd["c%d.w" % j], None, stride=2, padding=1)
            h = F.leaky_relu(bn(h, pd["bn%d.gamma" % j], pd["bn%d.beta" % j]), 0.2)
        return F.linear(h.flatten(1), pd["fc.w"], pd["fc.b"])[:, 0]

    for step in range(3):
        lab, z, x = batch(spec, [0, 3, 1, 2, 2, 1, 0, 3, 3, 0], seed=40 + step)
        orc.train_step(lab, z, x)
        zt, xt = torch.tensor(z), torch.tensor(x)
        oh = F.one_hot(torch.tensor(lab, dtype=torch.long), 4).double()
        fake = G(zt, oh)
        od.zero_grad()
        jd = 0.5 * F.softplus(-D(xt, oh)).mean() + 0.5 * F.softplus(D(fake.detach(), oh)).mean()
        jd.backward()
        od.step()
        og.zero_grad()
        jg = 0.5 * F.softplus(-D(fake, oh)).mean()
        jg.backward()
        og.step()
        ojd, ojg, _ = orc.get_losses()
        assert abs(ojd[0] - jd.item()) < 1e-10 and abs(ojg[0] - jg.item()) < 1e-10
    for which, p, sl in ((0, pg, sl_g), (1, pd, sl_d)):
        flat = orc.get_params(which, 0)
        for k, (s, shape) in sl.items():
            np.testing.assert_allclose(flat[s].reshape(shape), p[k].detach().numpy(), rtol=1e-7, atol=1e-9, err_msg=k)


def test_single_precision_build_runs_the_same_algorithm():
    """The oracle's loops compiled with a 32-bit real agree with the 64-bit oracle to rounding on the first
    iteration (same algorithm), and the printed drift of later iterations documents how quickly rounding is
    amplified by the iteration itself (the reason the fp32 parity bound widens from the second iteration on)."""
    spec = synth.SPECS["tiny"]
    a, b = O.Oracle(spec, 1, 4), O.Oracle(spec, 1, 4, real=np.float32)
    rng = np.random.default_rng(8)
    for which in (0, 1):
        p = synth.init_params(spec, which, rng)
        a.set_params(which, 0, p)
        b.set_params(which, 0, p)
    drift = []
    for s in range(4):
        lab, z, x = batch(spec, [0, 3, 1, 2, 2, 1, 0, 3] * 4, seed=60 + s)
        z, x = z.astype(np.float32), x.astype(np.float32)
        a.train_step(lab, z, x)
        b.train_step(lab, z, x)
        e = max(np.linalg.norm(b.get_params(w, 0) - a.get_params(w, 0)) / np.linalg.norm(a.get_params(w, 0)) for w in (0, 1))
        drift.append(e)
    assert drift[0] < 1e-5
    assert abs(b.get_losses()[0][0] - a.get_losses()[0][0]) < 1e-2
    print("single-precision drift per iteration:", drift)
