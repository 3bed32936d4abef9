"""The training step of the networks exactly as the paper's Tables 1 and 2 print them (GAN_FAMILY_PAPER) against
oracle/paper_nets.py on identical seeded inputs (GPU): G = linear + ReLU + BN(1e-5), two Upsample + Conv k3 + BN(0.8) +
LeakyReLU blocks, Conv k3 + tanh; D = Conv k3 s2 + LeakyReLU + Dropout(0.25) [+ BN(0.8)] blocks with 16/32/64/128
channels, linear.  Every step starts from the oracle's state (loaded through the checkpoint calls), as in
tests/test_gpu_step.py; the dropout masks of both sides come from the same counter-based generator, so a single
wrong mask bit would show as an O(1) error of a cost.

bf16 storage has no emulating oracle for these networks: costs, parameters and updates are held to the stated 2e-2
against the fp64 result and Adam's arithmetic to fp32 rounding; its gradients are reported, not bounded.
"""
import numpy as np
import pytest

import oracle as O
from oracle import paper_nets as PN
from paper_2102_10485_amd import binding, synth
from tests import gpu_util as U
from tests import parity as P

pytestmark = pytest.mark.gpu


def flat(d, shapes):
    return np.concatenate([np.asarray(d[name], np.float64).ravel() for name, _ in shapes])


def unflat(v, shapes):
    out, o = {}, 0
    for name, shp in shapes:
        n = int(np.prod(shp))
        out[name] = np.asarray(v[o:o + n], np.float64).reshape(shp)
        o += n
    return out


class PaperPair:
    def __init__(self, spec_name, K, max_n, prec, seed=5):
        torch = U.torch_mod()
        self.torch, self.spec, self.K, self.prec = torch, synth.SPECS[spec_name], K, prec
        s = self.spec
        self.gpu = binding.Gan(binding.make_config(s, K, K, max_n, prec, seed=seed), torch.cuda.current_stream().cuda_stream)
        self.orc = PN.PaperNets(s["img_c"], s["img_hw"], K, z_dim=s["z_dim"], g_ch=s["g_ch"], d_ch=s["d_ch"], seed=seed)
        self.shapes = [self.orc.gs, self.orc.ds]
        for w in (0, 1):
            assert [(n, tuple(sh)) for n, sh in self.shapes[w]] == [(n, tuple(sh)) for n, sh, _ in synth.param_tensors(s, w)]
            assert self.gpu.param_count(w) == synth.param_count(s, w)
        for l in range(K):
            rng = np.random.default_rng([seed, l])
            for w in (0, 1):
                p = synth.init_params(s, w, rng)
                self.orc.set_params(w, l, unflat(p, self.shapes[w]))
        self.bn_tags = [["0"] + [str(i) for i in range(1, len(s["g_ch"]))], [str(j) for j in range(2, len(s["d_ch"]) + 1)]]
        self.before = {}

    def _oracle_state(self, l):
        """(params, m, v, t, running mean, running var) per network, rounded to what fp32 holds, written back."""
        o, out = self.orc, []
        nets = [o.G[l], o.D[l]]
        for w in (0, 1):
            r32 = lambda a: np.asarray(a, np.float32).astype(np.float64)
            for name, _ in self.shapes[w]:
                nets[w][name] = r32(nets[w][name])
                if name in o.opt[l][w]:
                    m, v = o.opt[l][w][name]
                    o.opt[l][w][name] = (r32(m), r32(v))
            zeros = {name: np.zeros(shp) for name, shp in self.shapes[w]}
            m = flat({n_: o.opt[l][w].get(n_, (zeros[n_], zeros[n_]))[0] for n_ in zeros}, self.shapes[w])
            v = flat({n_: o.opt[l][w].get(n_, (zeros[n_], zeros[n_]))[1] for n_ in zeros}, self.shapes[w])
            rm, rv = [], []
            for tag in self.bn_tags[w]:
                ch = self._bn_channels(w, tag)
                mean, var = o.run[l][w].get(tag, (np.zeros(ch), np.ones(ch)))
                o.run[l][w][tag] = (r32(mean), r32(var))
                rm.append(o.run[l][w][tag][0]); rv.append(o.run[l][w][tag][1])
            out.append((flat(nets[w], self.shapes[w]), m, v, int(o.t[l, w]), np.concatenate(rm), np.concatenate(rv)))
        return out

    def _bn_channels(self, w, tag):
        s = self.spec
        return s["g_ch"][int(tag)] if w == 0 else s["d_ch"][int(tag) - 1]

    def step(self, lab, z, x):
        t = self.torch
        for l in range(self.K):
            st = self._oracle_state(l)
            for w, (th, m, v, tt, rm, rv) in enumerate(st):
                self.gpu.set_params(w, l, th)
                self.gpu.set_opt_state(w, l, m, v, tt)
                self.gpu.set_bn_running(w, l, rm, rv)
            self.before[l] = dict(params=[st[0][0], st[1][0]], m=[st[0][1], st[1][1]], v=[st[0][2], st[1][2]], t=[st[0][3], st[1][3]])
        self.keep = tuple(t.from_numpy(np.ascontiguousarray(a)).cuda() for a in (lab.astype(np.int32), z, x))
        self.gpu.train_step(self.keep[0].data_ptr(), self.keep[1].data_ptr(), self.keep[2].data_ptr(), len(lab))
        self.orc.train_step(lab, z.astype(np.float64), x.astype(np.float64))

    def oracle_snapshot(self, l):
        o = self.orc
        out = dict(jd=float(o.jd[l]), jg=float(o.jg[l]), params=[], grads=[], m=[], v=[], t=[], bn=[])
        nets = [o.G[l], o.D[l]]
        for w in (0, 1):
            out["params"].append(flat(nets[w], self.shapes[w]))
            out["grads"].append(flat(o.grads[l][w], self.shapes[w]))
            out["m"].append(flat({n_: o.opt[l][w][n_][0] for n_, _ in self.shapes[w]}, self.shapes[w]))
            out["v"].append(flat({n_: o.opt[l][w][n_][1] for n_, _ in self.shapes[w]}, self.shapes[w]))
            out["t"].append(int(o.t[l, w]))
            out["bn"].append((np.concatenate([o.run[l][w][tag][0] for tag in self.bn_tags[w]]),
                              np.concatenate([o.run[l][w][tag][1] for tag in self.bn_tags[w]])))
        return out

    def compare(self, what):
        cnt = self.gpu.get_losses()[2]
        assert np.array_equal(cnt, self.orc.counts)
        bounds = P.FP32_VS_PLAIN if self.prec == binding.FP32 else P.BF16_VS_PLAIN
        fails, report = [], []
        for l in range(self.K):
            if cnt[l] == 0:
                continue
            f, rows = P.compare_step(self.spec, self.before[l], P.snapshot(self.gpu, l), self.oracle_snapshot(l), bounds,
                                     "%s model %d" % (what, l), adam=O.adam)
            fails += f
            report += rows
        print(P.format_rows(report))
        assert not fails, fails

    def close(self):
        self.gpu.close()


def batch(spec, labels, seed):
    rng = np.random.default_rng(seed)
    n = len(labels)
    z = rng.normal(size=(n, spec["z_dim"])).astype(np.float32)
    x = np.tanh(rng.normal(size=(n, spec["img_c"], spec["img_hw"], spec["img_hw"]))).astype(np.float32)
    return np.asarray(labels, np.int32), z, x


@pytest.mark.parametrize("prec", [binding.FP32, binding.BF16])
def test_paper_networks_small(prec):
    """Channel counts that need padding everywhere (16, 32, 72), three ragged models, three iterations, one model
    left without samples in the second."""
    p = PaperPair("paper16", 3, 48, prec)
    rng = np.random.default_rng(1)
    for s, n in enumerate([31, 48, 40]):
        lab = rng.integers(0, 3, n)
        if s == 1:
            lab[lab == 2] = 0
        p.step(*batch(p.spec, lab, 300 + s))
        p.compare("step %d" % s)
    p.close()


@pytest.mark.parametrize("prec", [binding.FP32, binding.BF16])
def test_paper_networks_at_the_printed_widths(prec):
    """32x32x3 with the widths the tables print (G 128/128/64, D 16/32/64/128), three ragged label models, three
    iterations."""
    p = PaperPair("paper32", 3, 32, prec)
    rng = np.random.default_rng(2)
    for s, n in enumerate([26, 32, 19]):
        lab = np.concatenate([np.zeros(3, np.int64), rng.integers(0, 3, n - 3)])     # every model present, ragged
        p.step(*batch(p.spec, lab, 400 + s))
        p.compare("step %d" % s)
    p.close()


@pytest.mark.parametrize("prec", [binding.FP32, binding.BF16])
@pytest.mark.parametrize("spec_name", ["paper28", "paper16c4"])
def test_paper_networks_other_image_shapes(prec, spec_name):
    """One image channel on a 28 x 28 image behind 128 feature channels (patches that hang over the border, the wider
    instantiation of the image-side kernels), and four image channels (two row tiles of (tap, channel) in the weight
    gradient of the last convolution); two ragged models, two iterations."""
    p = PaperPair(spec_name, 2, 24, prec)
    rng = np.random.default_rng(3)
    for s, n in enumerate([19, 24]):
        lab = np.concatenate([np.arange(2), rng.integers(0, 2, n - 2)])
        p.step(*batch(p.spec, lab, 500 + s))
        p.compare("step %d" % s)
    p.close()
