"""The routing kernel (GPU) where its tables do not all live in LDS: a batch too large for the label copy, and more
models than the count table has room for.  The expected result is the definition itself, written out with numpy: a
stable partition of the flat batch by model (Eq. 5: pair k sees the samples of label k, in their order)."""
import numpy as np
import pytest

from paper_2102_10485_amd import binding, synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _step_and_routing(spec_name, n_models, n_labels, lab, seed):
    torch = U.torch_mod()
    spec = synth.SPECS[spec_name]
    n = len(lab)
    g = binding.Gan(binding.make_config(spec, n_models, n_labels, n, binding.BF16), torch.cuda.current_stream().cuda_stream)
    rng = np.random.default_rng(seed)
    z = rng.normal(size=(n, spec["z_dim"])).astype(np.float32)
    x = np.tanh(rng.normal(size=(n, spec["img_c"], spec["img_hw"], spec["img_hw"]))).astype(np.float32)
    dl, dz, dx = (torch.from_numpy(a).cuda() for a in (lab, z, x))
    g.train_step(dl.data_ptr(), dz.data_ptr(), dx.data_ptr(), n)
    jd, jg, cnt = g.get_losses()
    perm, offs = g.get_routing(n)
    g.close()
    return perm, offs, cnt, jd, jg


def _expected(lab, n_models):
    model = np.zeros_like(lab) if n_models == 1 else lab
    counts = np.bincount(model, minlength=n_models)
    return np.argsort(model, kind="stable").astype(np.int32), np.concatenate([[0], np.cumsum(counts)]).astype(np.int32), counts


def test_one_pair_with_a_batch_larger_than_the_label_copy():
    rng = np.random.default_rng(1)
    lab = rng.integers(0, 4, 40000).astype(np.int32)                  # 160 kB of labels: read from global memory
    perm, offs, cnt, jd, jg = _step_and_routing("tiny", 1, 4, lab, 2)
    eperm, eoffs, ecnt = _expected(lab, 1)
    assert np.array_equal(perm, eperm) and np.array_equal(offs, eoffs) and np.array_equal(cnt, ecnt)
    assert np.all(np.isfinite(jd)) and np.all(np.isfinite(jg))


def test_more_models_than_the_count_table_has_room_for():
    L = 130                                                            # 256 x 130 counts: kept in global memory
    rng = np.random.default_rng(3)
    lab = rng.integers(0, L, 1000).astype(np.int32)
    lab[lab == 7] = 8                                                  # one model without samples
    perm, offs, cnt, jd, jg = _step_and_routing("tiny0", L, L, lab, 4)
    eperm, eoffs, ecnt = _expected(lab, L)
    assert ecnt[7] == 0 and ecnt.min() == 0
    assert np.array_equal(perm, eperm) and np.array_equal(offs, eoffs) and np.array_equal(cnt, ecnt)
    assert np.all(np.isfinite(jd)) and np.all(np.isfinite(jg)) and jd[7] == 0 and jg[7] == 0
