"""Comparison of one training iteration taken by two implementations from the SAME state (no GPU needed here).

A "snapshot" is what an implementation holds for one label model after a step:
    dict(jd, jg, params=[G, D], grads=[G, D], m=[G, D], v=[G, D], t=[G, D], bn=[(mean, var), (mean, var)])
(flat arrays in the documented parameter order).  `before` is the state both started from (params, m, v, t).

What is compared, and why these quantities:
  * the two costs (Eq. 3, Eq. 4), relative;
  * the gradients, per tensor and per network: Adam's first moment after the step is beta1 m + (1 - beta1) g with the
    same m on both sides, so g, m and v are linear in the backward pass and carry its error undistorted;
  * the update theta_after - theta_before, relative to the reference's update -- NOT theta against |theta|: one
    Adam step moves a parameter by about lr = 2e-4 against an initial scale of 2e-2, so a path that never updated, or
    updated with the wrong sign, sits within 1e-2 .. 2e-2 of the reference in |theta| but is 1.0 or 2.0 away in the
    update;
  * Adam's arithmetic on its own: the oracle's Adam applied to the implementation's OWN gradient from the common state
    must reproduce its moments and its update to fp32 rounding -- a skipped, mis-signed or mis-scaled update fails
    here whatever the gradient's accuracy;
  * the parameters themselves against |theta| (the stated contract), the step counts, the BatchNorm running statistics.

The one discontinuity of the iteration is the (Leaky)ReLU derivative at zero: a pre-activation within rounding of
zero gets slope 1 on one side and 0.2 (or 0) on the other, which changes the gradient of that layer's output channel
by a percent or so (one of the few thousand terms of its sums changes by up to a factor five); BatchNorm's backward
pass spreads the changed element over its channel's batch sums and the data gradients spread that over every tensor
upstream, diffusely, by 1e-4 .. 3e-3 depending on batch size and width.  It happens to a few of a hundred
label-model steps.  Gradient comparisons in fp32 storage therefore set aside at most ONE output channel per tensor,
which must still be within 10 % (a channel computed wrongly is off by its whole size), and bound the rest at 5e-3;
in bf16 storage the bounds are wide enough to absorb it and nothing is set aside.

Bounds (`Bounds`): `cost`, `theta` are the stated tolerances (1e-4 in fp32 storage, 2e-2 in bf16 storage against the
plain fp64 result).  `grad` bounds the relative L2 error of a network's gradient, `grad_tensor` that of one tensor
and of one filter tap of a convolution weight.  The update is
ill-conditioned where a gradient element is within the backward pass's error of zero: Adam turns g into about
-lr sign(g), so such an element may land on either side, an error of up to 2 lr on it.  With a relative gradient
error e, about e of the elements are that close to zero (density of a bell-shaped distribution at its centre times
the width 2 e sigma), which puts the relative L2 error of the update near sqrt(e) .. 2 sqrt(e): `update` =
min(3 sqrt(grad), 0.5).  A missing update (1.0) and a mis-signed one (2.0) are outside it whatever the gradient
bound, and a single filter tap left out of a weight gradient is an error of 1.0 on that tap's slice.

bf16 storage.  Rounding a stored value is discontinuous: where the fp32 sum behind it lies within its own rounding
error of a bf16 boundary, two correct implementations that add in different orders store values one bf16 unit
(0.4-0.8 %) apart, a few dozen such values per label model and step at these sizes.  BatchNorm's backward pass
subtracts the batch mean of the gradient, which at (and near) initialisation removes most of it -- D's logits are
nearly equal, so the cost's gradient is nearly constant over the batch -- and what is left carries those few
discrete differences amplified: the oracle's bf16-storage emulation run with single-precision sums is 1e-3 .. 2e-2
(D) and 2e-2 .. 6e-2 (G, which sits behind D's update) away from the same emulation with double-precision sums, on
the very gradients compared here, while its costs agree to 1e-5 .. 4e-4.  No tolerance tighter than that distance
means anything for a whole step in bf16 storage, so the bound on the gradients is that distance, measured in the
same test on the same inputs and state (`emulation_bounds`), times 3 for the spread between two realisations of the
same process (it varies by 2.4 between the models of one batch); tight checks of the bf16 kernels are the single
operation tests (tests/test_gpu_ops.py), where nothing feeds a rounding difference back.
"""
import numpy as np

from paper_2102_10485_amd import synth


class Bounds:
    """Any bound left None is reported but not asserted."""

    def __init__(self, cost=None, theta=None, grad=None, grad_tensor=None, bn=None, update=None, set_aside=None):
        self.cost, self.theta, self.grad, self.set_aside = cost, theta, grad, set_aside
        self.grad_tensor = grad_tensor if grad_tensor is not None else (4.0 * grad if grad is not None else None)
        self.update = update if update is not None else (min(3.0 * np.sqrt(grad), 0.5) if grad is not None else None)
        self.bn = bn if bn is not None else (5.0 * cost if cost is not None else None)


# fp32 storage against the fp64 oracle: the stated 1e-4 on everything linear in the passes.
FP32_VS_PLAIN = Bounds(cost=1e-4, theta=1e-4, grad=5e-3, set_aside=0.1)
# bf16 storage against the plain fp64 oracle: the stated 2e-2 on costs and parameters; a missing or mis-signed update
# is caught here too; the gradients are reported (the storage rounding moves them by 5-15 % at initialisation).
BF16_VS_PLAIN = Bounds(cost=2e-2, theta=2e-2, update=0.7)


def fp32_bounds(pairs, spread=3.0):
    """Bounds for an fp32-storage implementation against the fp64 oracle.  Costs, parameters and running statistics:
    the stated 1e-4.  Gradients: 1e-4 where single precision can hold it; BatchNorm's backward pass removes the
    batch mean of a nearly constant gradient, and behind D's update G's gradient also sees every element of theta_D
    that Adam's sign-like step put on the other side, so from the second step on two correct single-precision
    implementations are further apart than that.  pairs: (snapshot of the oracle's loops compiled in single
    precision, fp64 snapshot) of the same step from the same state for every model checked; their largest distance
    times 3 (spread between two realisations) is the bound when it exceeds the floor.  The floor, 5e-3, is one
    activation-derivative decision taken the other way (see the module text): besides the one output channel that is
    set aside, the BatchNorm backward pass spreads the changed element over its channel's batch and the data gradients
    spread that over every tensor upstream, diffusely -- measured 1.2e-4 on G's gradient with one such decision in D's
    first layer at 40 samples per model, 2.6e-3 with one in a 64-channel generator block at 10 samples per model, 1e-6
    without.  Anything wrong in a kernel (a tap, a sign, a scale of a percent) is far above it."""
    d_grad = max(rel_l2(a["grads"][w], b["grads"][w]) for a, b in pairs for w in (0, 1))
    # The parameters follow the gradient through Adam's sign-like first steps: where the single-precision build of the
    # oracle itself takes such a decision the other way, its parameters leave the 1e-4 too (every element whose
    # gradient changed sign moves by 2 lr), and the same spread applies.
    d_theta = max(rel_l2(a["params"][w], b["params"][w]) for a, b in pairs for w in (0, 1))
    return Bounds(cost=1e-4, theta=max(1e-4, spread * d_theta), grad=max(5e-3, spread * d_grad), set_aside=0.1)


def emulation_bounds(pairs, spread=3.0):
    """Bounds for a bf16-storage implementation against the emulation with double-precision sums, from the distance
    of the emulation with single-precision sums to it.  pairs: (emu32 snapshot, emu64 snapshot) of the same step
    for every label model checked -- the differences are a few discrete events per model, so the largest distance
    over the models is the scale, and one event's worth (5e-3 on a gradient, 1e-3 on a cost) is the floor."""
    d_cost = max(abs(a[k] - b[k]) / abs(b[k]) for a, b in pairs for k in ("jd", "jg"))
    d_grad = max(rel_l2(a["grads"][w], b["grads"][w]) for a, b in pairs for w in (0, 1))
    grad = max(5e-3, spread * d_grad)
    return Bounds(cost=max(1e-3, spread * d_cost), grad=grad, grad_tensor=2.0 * grad, bn=5e-3)


def rel_l2(a, b, floor=0.0):
    a, b = np.asarray(a, np.float64).ravel(), np.asarray(b, np.float64).ravel()
    den = max(np.linalg.norm(b), floor)
    return np.linalg.norm(a - b) / den if den > 0 else np.linalg.norm(a - b)


def _channels(name, shape):
    """(number of output channels, axis) of a parameter tensor in the documented order."""
    if len(shape) == 4 and name.startswith("ct"):
        return shape[1], 1                                  # transposed convolution: [Cin][Cout][4][4]
    return shape[0], 0


def channel_errors(got, ref, name, shape):
    """Squared error and squared reference norm per output channel."""
    nch, axis = _channels(name, shape)
    a = np.moveaxis(np.asarray(got, np.float64).reshape(shape), axis, 0).reshape(nch, -1)
    b = np.moveaxis(np.asarray(ref, np.float64).reshape(shape), axis, 0).reshape(nch, -1)
    return ((a - b) ** 2).sum(axis=1), (b ** 2).sum(axis=1)


def compare_step(spec, before, got, ref, bounds, tag="", adam=None):
    """Returns (failures, rows): failures is a list of tuples naming what exceeded its bound; rows is the full table
    (quantity, error, bound) for reporting.  before: dict(params, m, v, t) both sides started from.  adam: the
    oracle's Adam as a function (theta, m, v, g, t) -> (theta, m, v), or None to skip the self-consistency check."""
    rows, fails = [], []

    def check(name, err, bound):
        rows.append((tag, name, float(err), float(bound) if bound is not None else float("inf")))
        if not np.isfinite(err) or (bound is not None and not (err <= bound)):
            fails.append((tag, name, float(err), bound))

    for name in ("jd", "jg"):
        check(name, abs(got[name] - ref[name]) / abs(ref[name]), bounds.cost)
    for which, net in ((0, "G"), (1, "D")):
        if got["t"][which] != ref["t"][which]:
            fails.append((tag, net + ".t", got["t"][which], ref["t"][which]))
        g_ref, g_got = ref["grads"][which], got["grads"][which]
        # per tensor (one output channel set aside, see above); a tensor whose gradient is tiny next to the network's
        # (a cancelled sum: the last bias and BatchNorm shift of D add gradients of opposite sign over the real and the
        # fake half) is measured against 1e-2 of the network's gradient norm spread evenly over its elements
        gn2 = float(g_ref @ g_ref) / g_ref.size
        net_e2, net_r2, set_aside = 0.0, 0.0, 0.0
        for tname, (sl, shape) in synth.param_slices(spec, which).items():
            n = int(np.prod(shape))
            e2, r2 = channel_errors(g_got[sl], g_ref[sl], tname, shape)
            worst = int(np.argmax(e2))
            set_aside = max(set_aside, np.sqrt(e2[worst] / max(r2[worst], r2.mean(), 1e-4 * gn2 * n / e2.size)))
            keep = np.ones(e2.size, bool)
            if e2.size > 1 and bounds.set_aside is not None:      # only where the bounds are tight enough to need it
                keep[worst] = False
            den2 = max(r2[keep].sum(), 1e-4 * gn2 * n)
            check("%s.grad[%s]" % (net, tname), np.sqrt(e2[keep].sum() / den2), bounds.grad_tensor)
            net_e2 += e2[keep].sum(); net_r2 += r2[keep].sum()
            if len(shape) == 4:                     # convolution weight: every filter tap on its own
                nch, axis = _channels(tname, shape)
                nt = shape[2] * shape[3]
                a = np.moveaxis(g_got[sl].reshape(shape), axis, 0)[keep].reshape(-1, nt)
                b = np.moveaxis(g_ref[sl].reshape(shape), axis, 0)[keep].reshape(-1, nt)
                tap = max(np.linalg.norm(a[:, t] - b[:, t]) / max(np.linalg.norm(b[:, t]), np.sqrt(1e-4 * gn2 * n / nt))
                          for t in range(nt))
                check("%s.grad[%s]/tap" % (net, tname), tap, bounds.grad_tensor)
        check(net + ".grad", np.sqrt(net_e2 / net_r2), bounds.grad)
        check(net + ".grad/set-aside channel", set_aside, bounds.set_aside)
        th0 = before["params"][which]
        if adam is not None:
            # Adam on the implementation's own gradient, from the common state
            th_e, m_e, v_e = adam(th0, before["m"][which], before["v"][which], g_got, before["t"][which] + 1)
            check(net + ".adam.m", rel_l2(got["m"][which], m_e), 1e-5)
            check(net + ".adam.v", rel_l2(got["v"][which], v_e), 1e-4)     # 1 - 0.999f is 1.3e-5 away from 0.001
            check(net + ".adam.update", rel_l2(got["params"][which] - th0, th_e - th0), 1e-3)
        d_got, d_ref = got["params"][which] - th0, ref["params"][which] - th0
        check(net + ".update", rel_l2(d_got, d_ref), bounds.update)
        check(net + ".theta", rel_l2(got["params"][which], ref["params"][which]), bounds.theta)
        (gm, gv), (rm, rv) = got["bn"][which], ref["bn"][which]
        check(net + ".bn_mean", rel_l2(gm, rm, floor=1e-2 * np.sqrt(max(rm.size, 1))), bounds.bn)
        check(net + ".bn_var", rel_l2(gv, rv), bounds.bn)
    return fails, rows


def snapshot(impl, model):
    """impl: anything with get_losses / get_params / get_grads / get_opt_state / get_bn_running (the HIP binding and
    the oracle wrapper both have them)."""
    jd, jg = impl.get_losses()[:2]
    out = dict(jd=float(jd[model]), jg=float(jg[model]), params=[], grads=[], m=[], v=[], t=[], bn=[])
    for which in (0, 1):
        out["params"].append(np.asarray(impl.get_params(which, model), np.float64))
        out["grads"].append(np.asarray(impl.get_grads(which, model), np.float64))
        m, v, t = impl.get_opt_state(which, model)
        out["m"].append(np.asarray(m, np.float64)); out["v"].append(np.asarray(v, np.float64)); out["t"].append(int(t))
        mean, var = impl.get_bn_running(which, model)
        out["bn"].append((np.asarray(mean, np.float64), np.asarray(var, np.float64)))
    return out


def format_rows(rows, only_worst=True):
    worst = {}
    for tag, name, err, bound in rows:
        key = name.split("[")[0] if only_worst else name
        if key not in worst or err / bound > worst[key][0] / worst[key][1]:
            worst[key] = (err, bound, tag)
    return "\n".join("  %-14s worst %.2e (bound %.1e) %s" % (k, e, b, t) for k, (e, b, t) in sorted(worst.items()))
