"""Parity of the two rows next to the training step against the oracle (GPU): mixture sampling (Eq. 5: class draws
from the prior, then the per-label generators) and the one-way ANOVA F-statistic per channel (Section 4).

Class draws are integers decided in double on both sides: compared bit for bit.  Images: 1e-4 (fp32 storage) / 2e-2
(bf16 storage) relative L2 on the image scale.  F: all arithmetic is double on both sides and only the summation
order differs: 1e-9 relative."""
import numpy as np
import pytest

import oracle as O
from paper_2102_10485_amd import binding, synth
from tests import gpu_util as U
from tests.test_gpu_step import Pair, batch, TOL

pytestmark = pytest.mark.gpu


def _gpu_sample(p, prior, u, z, running=1):
    torch = U.torch_mod()
    n = len(u)
    shape = (n, p.spec["img_c"], p.spec["img_hw"], p.spec["img_hw"])
    out = torch.zeros(shape, dtype=torch.float32, device="cuda")
    labels = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    du, dz = torch.from_numpy(np.ascontiguousarray(u, np.float32)).cuda(), torch.from_numpy(np.ascontiguousarray(z, np.float32)).cuda()
    p.gpu.sample(prior, du.data_ptr(), dz.data_ptr(), n, out.data_ptr(), labels.data_ptr(), running)
    torch.cuda.synchronize()
    return out.cpu().numpy(), labels.cpu().numpy()


@pytest.mark.parametrize("prec", [binding.FP32, binding.BF16])
def test_sample_small(prec):
    """Three tiny models with identical parameters on both sides (no training step in between: after one, single
    elements of the two parameter sets legitimately differ by 2 lr, which the near-cancelling running-statistics
    output would amplify; generation with trained statistics is covered in test_gpu_step.test_generate)."""
    p = Pair("tiny3", 3, 3, 64, prec)
    rng = np.random.default_rng(8)
    n = 50
    u = rng.random(n).astype(np.float32)
    u[:4] = [0.0, 0.25, 0.75, 0.99999994]                     # on the cumulative values of the prior below, and the ends
    zz = rng.normal(size=(n, p.spec["z_dim"])).astype(np.float32)
    prior = [0.25, 0.5, 0.25]
    for running in (1, 0):
        img, labels = _gpu_sample(p, prior, u, zz, running)
        rc, ref, ref_labels = p.orc.sample(prior, u, zz.astype(np.float64), use_running_stats=running)
        assert rc == 0
        np.testing.assert_array_equal(labels, ref_labels)
        assert U.rel_l2(img, ref, floor=0.1 * np.sqrt(ref.size)) <= TOL[prec]
    # a prior with empty classes, unnormalised
    img, labels = _gpu_sample(p, [0.0, 0.0, 5.0], u, zz)
    assert np.all(labels == 2)
    # bad priors are refused on the host
    with pytest.raises(binding.GanError):
        _gpu_sample(p, [0.0, 0.0, 0.0], u, zz)
    with pytest.raises(binding.GanError):
        _gpu_sample(p, [0.5, -0.5, 1.0], u, zz)
    p.close()


def test_sample_config2_full_size_bf16():
    """6400 draws over 100 labels with a rank-Zipf prior: every label bit-exact; images of two labels against the
    oracle (with the running statistics every image depends on its own noise row only)."""
    w = synth.Workload(2)
    models = [0, 99]
    p = Pair("cifar", 100, 100, w.n, binding.BF16, seed=w.seed, oracle_models=models)
    rng = np.random.default_rng(9)
    prior = 1.0 / np.arange(1, 101) ** 1.1
    u = rng.random(w.n).astype(np.float32)
    z = rng.normal(size=(w.n, p.spec["z_dim"])).astype(np.float32)
    img, labels = _gpu_sample(p, prior, u, z)
    rc, want = O.draw_labels(prior, u)
    assert rc == 0
    np.testing.assert_array_equal(labels, want)
    assert np.bincount(labels, minlength=100)[0] > np.bincount(labels, minlength=100)[99]
    for k in models:
        rows = np.where(labels == k)[0]
        assert rows.size > 0
        rc, ref = p.orc.generate(np.full(rows.size, k, np.int32), z[rows].astype(np.float64), use_running_stats=1, only_model=k)
        assert U.rel_l2(img[rows], ref, floor=0.1 * np.sqrt(ref.size)) <= TOL[binding.BF16]
    p.close()


def _gpu_anova(gan, lab, img):
    torch = U.torch_mod()
    dl = torch.from_numpy(np.ascontiguousarray(lab, np.int32)).cuda()
    di = torch.from_numpy(np.ascontiguousarray(img, np.float32)).cuda()
    return gan.anova_f(dl.data_ptr(), di.data_ptr(), len(lab), img.shape[1])


@pytest.mark.parametrize("config", [1, 2, 4])
def test_anova_f_of_the_workloads(config):
    torch = U.torch_mod()
    w = synth.Workload(config)
    gan = binding.Gan(binding.make_config(w.spec, w.n_models, w.n_labels, w.n, binding.FP32), torch.cuda.current_stream().cuda_stream)
    lab = w.labels()
    img = w.images(lab)
    st, F = _gpu_anova(gan, lab, img)
    rc, ref = O.anova_f(lab, img, w.n_labels)
    assert st == 0 and rc == 0
    np.testing.assert_allclose(F, ref, rtol=1e-9)
    assert np.all(F > 10.0)
    gan.close()


def test_anova_f_edge_cases():
    torch = U.torch_mod()
    spec = synth.SPECS["tiny0"]                                 # unconditional networks: any number of labels
    C_, H_ = spec["img_c"], spec["img_hw"]
    gan = binding.Gan(binding.make_config(spec, 1, 5, 300, binding.FP32), torch.cuda.current_stream().cuda_stream)
    rng = np.random.default_rng(12)
    n = 257                                                     # ragged against the 256-thread reductions
    lab = rng.integers(0, 5, n).astype(np.int32)
    img = (rng.normal(size=(n, C_, H_, H_)) * 0.3 + 0.05 * lab[:, None, None, None]).astype(np.float32)
    st, F = _gpu_anova(gan, lab, img)
    rc, ref = O.anova_f(lab, img, 5)
    assert st == 0
    np.testing.assert_allclose(F, ref, rtol=1e-9)
    # labels outside the range are ignored; a class may be empty
    lab2 = lab.copy()
    lab2[lab2 == 3] = 9
    lab2[:3] = -1
    st, F2 = _gpu_anova(gan, lab2, img)
    rc, ref2 = O.anova_f(lab2, img, 5)
    assert st == 0 and rc == 0
    np.testing.assert_allclose(F2, ref2, rtol=1e-9)
    # one class only: no statistic
    st, F3 = _gpu_anova(gan, np.zeros(n, np.int32), img)
    assert st == binding.GAN_E_STATE and np.all(F3 == 0)
    # the worked example of the oracle's pins: F = 13
    vals = np.array([1, 2, 3, 2, 3, 4, 5, 6, 7], np.float32)
    ex = np.broadcast_to(vals[:, None, None, None], (9, C_, H_, H_)).copy()
    st, F4 = _gpu_anova(gan, np.array([0, 0, 0, 1, 1, 1, 2, 2, 2], np.int32), ex)
    assert st == 0
    np.testing.assert_allclose(F4, [13.0] * C_, rtol=1e-12)
    gan.close()
