"""The entry point that allocates nothing (gan_anova_f_static: intermediate results in a static device array) against
the existing one (gan_anova_f: buffers from hipMalloc) and the oracle, on two calls in a row, the second smaller, so
that what the first call left in the shared array cannot leak into the second."""
import numpy as np
import pytest

import oracle as O
from paper_2102_10485_amd import binding, synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_matches_the_allocating_one():
    torch = U.torch_mod()
    w = synth.Workload(2)                                      # 6400 images of 100 labels, 32x32x3
    spec = w.spec
    C_, H_ = spec["img_c"], spec["img_hw"]
    stream = torch.cuda.current_stream().cuda_stream
    gan = binding.Gan(binding.make_config(spec, w.n_models, w.n_labels, w.n, binding.FP32), stream)
    lab = w.labels()
    img = w.images(lab)
    rng = np.random.default_rng(4)
    keep = np.sort(rng.choice(w.n, 1237, replace=False))       # second call: fewer images, fewer labels present
    keep = keep[lab[keep] < 37]
    for labels, images, n_labels in ((lab, img, w.n_labels), (lab[keep], img[keep], 37)):
        dl = torch.from_numpy(np.ascontiguousarray(labels, np.int32)).cuda()
        di = torch.from_numpy(np.ascontiguousarray(images, np.float32)).cuda()
        n = len(labels)
        st, F = binding.anova_f_static(dl.data_ptr(), di.data_ptr(), n, n_labels, C_, H_, stream)
        assert st == binding.GAN_OK, binding.static_last_error()
        # the existing entry point takes the label range from its context: labels beyond n_labels do not occur here
        st2, F2 = gan.anova_f(dl.data_ptr(), di.data_ptr(), n, C_)
        assert st2 == binding.GAN_OK
        np.testing.assert_array_equal(F, F2)                   # same kernels, same order of every sum
        rc, ref = O.anova_f(labels, images, n_labels)
        assert rc == 0
        np.testing.assert_allclose(F, ref, rtol=1e-9)
    # sizes beyond the static array are refused before anything is launched
    st, F = binding.anova_f_static(dl.data_ptr(), di.data_ptr(), 65537, 10, C_, H_, stream)
    assert st == binding.GAN_E_SHAPE and "MAX_IMAGES" in binding.static_last_error() and np.all(F == 0)
    st, F = binding.anova_f_static(dl.data_ptr(), di.data_ptr(), 10, 1025, C_, H_, stream)
    assert st == binding.GAN_E_SHAPE and "MAX_LABELS" in binding.static_last_error()
    st, F = binding.anova_f_static(dl.data_ptr(), di.data_ptr(), 10, 10, 5, H_, stream)
    assert st == binding.GAN_E_ARG
    gan.close()
