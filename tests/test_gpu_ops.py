"""Per-kernel parity of the grouped implicit-GEMM engine against the oracle's direct loops (GPU).

Sizes span several 128-row tiles, a ragged tail, an empty group, and groups with different weights.
"""
import numpy as np
import pytest

import oracle as O
from paper_2102_10485_amd import binding, synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctxs():
    torch = U.torch_mod()
    torch.cuda.init()
    out = {}
    for prec in (binding.FP32, binding.BF16):
        cfg = binding.make_config(synth.SPECS["tiny"], 1, 4, 8, prec)
        out[prec] = binding.Gan(cfg, torch.cuda.current_stream().cuda_stream)
    yield out
    for g in out.values():
        g.close()


CASES = [
    # cb, cs, hs, group sizes
    (64, 128, 4, [5, 0, 19, 8]),
    (128, 64, 8, [3, 7]),
    (64, 64, 7, [9, 2, 4]),
    (256, 128, 2, [70, 1]),
    (128, 256, 4, [20, 5]),
    (64, 512, 2, [130]),
    (256, 512, 4, [33, 40]),       # 256-wide output tiles in both directions, several M-tiles per model
    (128, 128, 16, [3]),           # one sample is a whole 256-row tile
    (64, 128, 4, [1, 1, 2]),       # models with a single sample
    (64, 256, 8, [5, 0, 3]),       # down: 256-wide tiles of four samples each, ragged tails
    (256, 64, 8, [2, 7]),          # up: the same, per output phase
    (64, 256, 16, [2, 1]),         # down: one sample per 256-row tile
    (256, 64, 16, [1, 2]),         # up: one sample per tile
]


def tolerance(prec):
    return 2e-5 if prec == binding.FP32 else 1e-2


@pytest.mark.parametrize("tile_rows", [0, 64, 128, 256])
@pytest.mark.parametrize("prec", [binding.FP32, binding.BF16])
@pytest.mark.parametrize("cb,cs,hs,groups", CASES)
def test_conv_down_up_wgrad(ctxs, prec, cb, cs, hs, groups, tile_rows):
    """tile_rows: the forward-type kernel's tile height (0: as a training step would choose for this size, which is
    the smallest tile at these sizes); with 256 the width follows the output channels (64, 128 or 256 columns), so the
    cases together run every tile instantiation."""
    torch = U.torch_mod()
    g = ctxs[prec]
    g.op_tile_rows(tile_rows)
    bf = prec == binding.BF16
    rng = np.random.default_rng(cb * 1000 + cs + hs)
    n = int(sum(groups))
    offs = np.concatenate([[0], np.cumsum(groups)]).astype(np.int32)
    G = len(groups)
    W = U.round_to(rng.normal(0, 0.05, (G, cs, cb, 4, 4)), bf)          # [cs][cb][ky][kx] per group
    big = U.round_to(rng.normal(0, 1, (n, cb, 2 * hs, 2 * hs)), bf)     # NCHW for the oracle
    small = U.round_to(rng.normal(0, 1, (n, cs, hs, hs)), bf)
    w_up = np.ascontiguousarray(W.transpose(0, 3, 4, 2, 1)).reshape(G, 16, cb, cs)
    w_down = np.ascontiguousarray(W.transpose(0, 3, 4, 1, 2)).reshape(G, 16, cs, cb)
    d_offs = U.dev(offs)
    d_big = U.dev(U.pack(big.transpose(0, 2, 3, 1), bf))
    d_small = U.dev(U.pack(small.transpose(0, 2, 3, 1), bf))
    d_wup, d_wdown = U.dev(U.pack(w_up, bf)), U.dev(U.pack(w_down, bf))
    tol = tolerance(prec)

    # down: conv forward
    out = torch.zeros(n * hs * hs * cs, dtype=torch.int16 if bf else torch.float32, device="cuda")
    g.op_conv_down(d_big.data_ptr(), d_wdown.data_ptr(), out.data_ptr(), d_offs.data_ptr(), G, n, cb, cs, hs)
    got = U.unpack(out, bf, (n, hs, hs, cs)).transpose(0, 3, 1, 2)
    ref = np.concatenate([O.conv2d(big[offs[i]:offs[i + 1]], W[i], None) for i in range(G) if groups[i]])
    assert np.max(np.abs(got - ref)) <= tol * np.max(np.abs(ref)), "down"

    # up: transposed conv forward
    out = torch.zeros(n * 4 * hs * hs * cb, dtype=torch.int16 if bf else torch.float32, device="cuda")
    g.op_conv_up(d_small.data_ptr(), d_wup.data_ptr(), out.data_ptr(), d_offs.data_ptr(), G, n, cb, cs, hs)
    got = U.unpack(out, bf, (n, 2 * hs, 2 * hs, cb)).transpose(0, 3, 1, 2)
    ref = np.concatenate([O.conv_transpose2d(small[offs[i]:offs[i + 1]], W[i], None) for i in range(G) if groups[i]])
    assert np.max(np.abs(got - ref)) <= tol * np.max(np.abs(ref)), "up"

    # wgrad (fp32 output in both modes)
    dw = torch.full((G * 16 * cb * cs,), 7.0, dtype=torch.float32, device="cuda")
    g.op_conv_wgrad(d_big.data_ptr(), d_small.data_ptr(), dw.data_ptr(), d_offs.data_ptr(), G, n, cb, cs, hs)
    got = dw.cpu().numpy().reshape(G, 4, 4, cb, cs)
    for i in range(G):
        if groups[i] == 0:
            assert np.all(got[i] == 0)
            continue
        _, dW, _ = O.conv2d_bwd(big[offs[i]:offs[i + 1]], W[i], small[offs[i]:offs[i + 1]], need_dx=False)
        ref = dW.transpose(2, 3, 1, 0)                                   # [cs][cb][ky][kx] -> [ky][kx][cb][cs]
        assert np.max(np.abs(got[i] - ref)) <= 2e-5 * np.max(np.abs(ref)) * (50 if bf else 1), "wgrad group %d" % i


@pytest.mark.gpu
def test_probes_report_plausible_ceilings():
    """The register-only MFMA loop and the plain copy return rates of the right order for this chip."""
    U.torch_mod().cuda.set_device(0)
    bf = binding.probe_mfma(binding.BF16)
    fp = binding.probe_mfma(binding.FP32)
    cp = binding.probe_copy(1 << 28)
    assert 500.0 < bf < 2600.0          # published dense bf16 peak: 2.5 PFLOP/s
    assert 30.0 < fp < 170.0            # published fp32 matrix peak: 157.3 TFLOP/s
    assert 1000.0 < cp < 8200.0         # published HBM peak: 8 TB/s


@pytest.mark.parametrize("prec", [binding.FP32, binding.BF16])
@pytest.mark.parametrize("cin,cout,hs,groups", [(128, 128, 8, [3, 0, 2]), (128, 64, 16, [2, 1])])
def test_upsample_conv3_runs_on_the_transposed_convolution_engine(ctxs, prec, cin, cout, hs, groups):
    """The generator blocks the paper prints (Table 1: Upsample x2, then Conv k3 s1 p1) on the grouped k4 s2 p1
    transposed-convolution kernel with the summed taps W4 = A W3 A^T; reference: the oracle's literal upsampling
    followed by its 3 x 3 convolution."""
    from oracle import paper_nets as P
    torch = U.torch_mod()
    g = ctxs[prec]
    g.op_tile_rows(0)
    bf = prec == binding.BF16
    rng = np.random.default_rng(cin + cout + hs)
    n = int(sum(groups))
    offs = np.concatenate([[0], np.cumsum(groups)]).astype(np.int32)
    G = len(groups)
    w3 = rng.normal(0, 0.05, (G, cout, cin, 3, 3))                       # [cout][cin][ky][kx] per group
    A = np.array([[0, 0, 1], [0, 1, 1], [1, 1, 0], [1, 0, 0]], float)
    w4 = U.round_to(np.einsum("ak,goikl,bl->gabio", A, w3, A), bf)       # [group][ky4][kx4][cin][cout], storage rounding
    small = U.round_to(rng.normal(0, 1, (n, cin, hs, hs)), bf)
    w_up = np.ascontiguousarray(w4.transpose(0, 1, 2, 4, 3)).reshape(G, 16, cout, cin)   # the kernel's [tap][cb][cs]
    d_offs = U.dev(offs)
    d_small = U.dev(U.pack(small.transpose(0, 2, 3, 1), bf))
    d_w = U.dev(U.pack(w_up, bf))
    out = torch.zeros(n * 4 * hs * hs * cout, dtype=torch.int16 if bf else torch.float32, device="cuda")
    g.op_conv_up(d_small.data_ptr(), d_w.data_ptr(), out.data_ptr(), d_offs.data_ptr(), G, n, cout, cin, hs)
    got = U.unpack(out, bf, (n, 2 * hs, 2 * hs, cout)).transpose(0, 3, 1, 2)
    # the summed taps are rounded to the storage type before the multiplication: the reference uses the same
    # rounded W4 through the pinned identity, and the literal form with the unrounded W3 bounds the difference
    ref4 = np.concatenate([O.conv_transpose2d(small[offs[i]:offs[i + 1]], w4[i].transpose(2, 3, 0, 1), None)
                           for i in range(G) if groups[i]])
    lit = np.concatenate([O.conv2d(P.upsample2(small[offs[i]:offs[i + 1]]), w3[i], None, 3, 1, 1)
                          for i in range(G) if groups[i]])
    tol = tolerance(prec)
    assert np.max(np.abs(got - ref4)) <= tol * np.max(np.abs(ref4))
    assert np.max(np.abs(got - lit)) <= (2e-5 if not bf else 2e-2) * np.max(np.abs(lit))
