"""Behaviour of the C ABI around the training step (GPU): unsupported shapes are refused with a status, never by
ending the process; generating between a step and its queries leaves the step's routing and counts alone; the
checkpoint calls restore a context exactly."""
import numpy as np
import pytest

from paper_2102_10485_amd import binding, synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _ctx(spec_name="tiny", K=4, n=64, prec=binding.FP32):
    torch = U.torch_mod()
    return binding.Gan(binding.make_config(synth.SPECS[spec_name], K, K, n, prec), torch.cuda.current_stream().cuda_stream)


def test_single_operations_refuse_shapes_the_kernels_do_not_support():
    torch = U.torch_mod()
    g = _ctx()
    buf = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    offs = torch.tensor([0, 4], dtype=torch.int32, device="cuda")
    p, o = buf.data_ptr(), offs.data_ptr()
    for fn, args in ((g.lib.gan_op_conv_down, (64, 32, 4)),       # 32 output channels: below the 64-wide tiles
                     (g.lib.gan_op_conv_up, (32, 64, 4)),
                     (g.lib.gan_op_conv_down, (64, 96, 4)),       # not a multiple of 64
                     (g.lib.gan_op_conv_up, (100, 64, 4)),
                     (g.lib.gan_op_conv_wgrad, (64, 4, 4)),
                     (g.lib.gan_op_conv_wgrad, (60, 64, 4))):
        st = fn(g.h, p, p, p, o, 1, 4, *args)
        assert st == binding.GAN_E_SHAPE, (fn.__name__, args, st)
        assert g.lib.gan_last_error(g.h)
    # an operand of 2 GiB or more is beyond the kernels' 32-bit offsets
    assert g.lib.gan_op_conv_down(g.h, p, p, p, o, 1, 40000, 512, 512, 8) == binding.GAN_E_SHAPE
    # null pointers and negative sizes are argument errors
    assert g.lib.gan_op_conv_down(g.h, 0, p, p, o, 1, 4, 64, 64, 4) == binding.GAN_E_ARG
    assert g.lib.gan_op_conv_down(g.h, p, p, p, o, 1, -1, 64, 64, 4) == binding.GAN_E_ARG
    # a tile height the kernels do not have
    assert g.lib.gan_op_tile_rows(g.h, 96) == binding.GAN_E_ARG
    # and the context still works afterwards, with every tile height there is
    for rows in (64, 128, 256, 0):
        g.op_tile_rows(rows)
        g.op_conv_down(p, p, p, o, 1, 4, 64, 64, 4)
    g.close()


def test_generate_between_a_step_and_its_queries_changes_nothing_they_return():
    torch = U.torch_mod()
    g = _ctx()
    spec = synth.SPECS["tiny"]
    rng = np.random.default_rng(3)
    n = 50
    lab = rng.integers(0, 4, n).astype(np.int32)
    z = rng.normal(size=(n, spec["z_dim"])).astype(np.float32)
    x = np.tanh(rng.normal(size=(n, 1, 8, 8))).astype(np.float32)
    dl, dz, dx = (torch.from_numpy(a).cuda() for a in (lab, z, x))
    g.train_step(dl.data_ptr(), dz.data_ptr(), dx.data_ptr(), n)
    jd, jg, cnt = g.get_losses()
    perm, offs = g.get_routing(n)
    perm, offs = perm.copy(), offs.copy()
    # a generation call with other labels and another size in between
    lab2 = np.array([3, 3, 1, 3, 3, 3, 1], np.int32)
    d2, z2 = torch.from_numpy(lab2).cuda(), torch.from_numpy(z[:7].copy()).cuda()
    out = torch.zeros((7, 1, 8, 8), dtype=torch.float32, device="cuda")
    g.generate(d2.data_ptr(), z2.data_ptr(), 7, out.data_ptr(), 0)
    jd2, jg2, cnt2 = g.get_losses()
    perm2, offs2 = g.get_routing(n)
    assert np.array_equal(cnt, cnt2) and np.array_equal(cnt, np.bincount(lab, minlength=4))
    assert np.array_equal(jd, jd2) and np.array_equal(jg, jg2)
    assert np.array_equal(perm, perm2) and np.array_equal(offs, offs2)
    g.close()


@pytest.mark.parametrize("prec", [binding.FP32, binding.BF16])
def test_checkpoint_calls_restore_a_context_bit_for_bit(prec):
    """Parameters, Adam moments and step counts, BatchNorm running statistics read from one context and loaded into a
    fresh one: the next step is bit-identical in both."""
    torch = U.torch_mod()
    spec = synth.SPECS["tiny"]
    rng = np.random.default_rng(9)
    a, b = _ctx(prec=prec), _ctx(prec=prec)
    batches = []
    for s in range(3):
        n = [40, 64, 33][s]
        batches.append((rng.integers(0, 4, n).astype(np.int32), rng.normal(size=(n, spec["z_dim"])).astype(np.float32),
                        np.tanh(rng.normal(size=(n, 1, 8, 8))).astype(np.float32)))

    def step(g, bt):
        t = [torch.from_numpy(v).cuda() for v in bt]
        g.train_step(t[0].data_ptr(), t[1].data_ptr(), t[2].data_ptr(), len(bt[0]))
        torch.cuda.synchronize()

    step(a, batches[0])
    step(a, batches[1])
    for l in range(4):
        for w in (0, 1):
            b.set_params(w, l, a.get_params(w, l))
            m, v, t = a.get_opt_state(w, l)
            b.set_opt_state(w, l, m, v, t)
            b.set_bn_running(w, l, *a.get_bn_running(w, l))
    step(a, batches[2])
    step(b, batches[2])
    for l in range(4):
        for w in (0, 1):
            assert np.array_equal(a.get_params(w, l), b.get_params(w, l))
            for u, v_ in zip(a.get_opt_state(w, l), b.get_opt_state(w, l)):
                assert np.array_equal(u, v_)
            for u, v_ in zip(a.get_bn_running(w, l), b.get_bn_running(w, l)):
                assert np.array_equal(u, v_)
    assert np.array_equal(a.get_losses()[0], b.get_losses()[0])
    a.close()
    b.close()
