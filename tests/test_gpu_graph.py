"""The optional ways to run a step -- replayed as a HIP graph, with the weight gradients and weight updates on a
second stream, or both -- against plain launches on one stream (the default): same kernels, so every step must equal
the plain result bit for bit.  Four contexts take the same steps from the same parameters: replaying
(gan_use_graphs), second stream (gan_use_second_stream), both, neither.  The inputs live in the same device buffers throughout and are overwritten before every step (labels
too: the routing is rebuilt on the device inside the replay); between the steps the program does its own eager work
-- host queries, a generate call on the replaying context, torch kernels -- and synchronises."""
import numpy as np
import pytest

from paper_2102_10485_amd import binding, synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("spec_name,precision", [("tiny3", "fp32"), ("tiny3", "bf16"), ("paper16", "bf16")])
def test_replays_equal_plain_launches(spec_name, precision):
    torch = U.torch_mod()
    spec = synth.SPECS[spec_name]
    K, n = 3, 40
    prec = binding.BF16 if precision == "bf16" else binding.FP32
    rng = np.random.default_rng(77)
    st = torch.cuda.current_stream().cuda_stream
    ctxs = [binding.Gan(binding.make_config(spec, K, K, n, prec, seed=5), st) for _ in range(4)]
    ctxs[0].use_graphs(True)
    ctxs[1].use_second_stream(True)
    ctxs[2].use_second_stream(True)
    ctxs[2].use_graphs(True)
    plain = ctxs[3]
    for l in range(K):
        for which in (0, 1):
            p = synth.init_params(spec, which, np.random.default_rng([9, which, l]))
            for g in ctxs:
                g.set_params(which, l, p)
    hw, ch = spec["img_hw"], spec["img_c"]
    d_lab = torch.zeros(n, dtype=torch.int32, device="cuda")
    d_z = torch.zeros(n, spec["z_dim"], dtype=torch.float32, device="cuda")
    d_x = torch.zeros(n, ch, hw, hw, dtype=torch.float32, device="cuda")
    junk = torch.zeros(1 << 20, device="cuda")
    d_img = torch.zeros(n, ch, hw, hw, dtype=torch.float32, device="cuda")
    for step in range(7):
        lab = rng.integers(0, K, n).astype(np.int32)
        if step == 3:
            lab[lab == 1] = 2                                   # a model without samples in this step
        d_lab.copy_(torch.from_numpy(lab))
        d_z.copy_(torch.from_numpy(rng.normal(size=(n, spec["z_dim"])).astype(np.float32)))
        d_x.copy_(torch.from_numpy(np.tanh(rng.normal(size=(n, ch, hw, hw))).astype(np.float32)))
        for g in ctxs:
            g.train_step(d_lab.data_ptr(), d_z.data_ptr(), d_x.data_ptr(), n)
        torch.cuda.synchronize()
        b = plain.get_losses()
        for k, g in enumerate(ctxs[:3]):
            for u, v in zip(g.get_losses(), b):
                assert np.array_equal(u, v), (step, k, u, v)
            for l in range(K):
                for which in (0, 1):
                    assert np.array_equal(g.get_params(which, l), plain.get_params(which, l)), (step, k, l, which)
                    ma, va, ta = g.get_opt_state(which, l)
                    mb, vb, tb = plain.get_opt_state(which, l)
                    assert ta == tb and np.array_equal(ma, mb) and np.array_equal(va, vb), (step, k, l, which)
        assert np.array_equal(ctxs[0].get_routing(n)[0], np.argsort(lab, kind="stable"))
        # eager work between the replays
        junk.add_(1.0).mul_(0.5)
        ctxs[0].generate(d_lab.data_ptr(), d_z.data_ptr(), n, d_img.data_ptr())
        assert bool(torch.isfinite(d_img).all())
        if step == 4:
            # new parameters for one model: the storage-type copies are rebuilt outside the replayed part
            p = synth.init_params(spec, 0, np.random.default_rng([10, 0, 0]))
            for g in ctxs:
                g.set_params(0, 0, p)
        torch.cuda.synchronize()
    # the first call ran as plain launches, the second was captured: six replays; none where replays are off
    assert [g.graph_replays() for g in ctxs] == [6, 0, 6, 0]
    for g in ctxs:
        g.close()
