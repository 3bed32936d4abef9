"""Writes the stored oracle results for the full-size workloads (calls only `oracle/` and the input generators).

    python tests/golden/make_golden.py [config ...]

For each configuration the CPU oracle is stepped, free-running, on the same seeded inputs the GPU test will use, for
the stated subset of label models (the models are independent, Eq. 5 of the paper, so a subset is exact for its
members).  Four variants of the oracle run side by side:
    f64  the oracle                                   (what fp32 and bf16 storage are held to by the stated tolerances)
    f32  its loops compiled in single precision       (how far a correct fp32 implementation is from f64 at that step)
    e64  its bf16-storage emulation, fp64 sums        (the reference that rounds what a bf16-storage path rounds)
    e32  the same emulation with single-precision sums (how far a correct bf16-storage implementation is from e64)
Stored per configuration and variant: the two costs of every step; after the first step (taken from the seeded initial
state, so every implementation starts it from identical values) every gradient tensor and every parameter tensor
sampled at fixed seeded positions (up to SAMPLES per tensor); the sampled parameters again after the steps in `snaps`.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle as O  # noqa: E402
from paper_2102_10485_amd import synth  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))

# config -> (models checked, steps, parameter snapshots after these steps; the first step is always one of them)
PLAN = {
    0: dict(models=[0], steps=5, snaps=[1, 5]),
    1: dict(models=[0, 9], steps=50, snaps=[1, 5, 50]),
    2: dict(models=[0, 49, 99], steps=3, snaps=[1, 3]),
    3: dict(models=[0, 7], steps=3, snaps=[1, 3]),
    4: dict(models="zipf", steps=3, snaps=[1, 3]),
}
SAMPLES = 2048
VARIANTS = {"f64": dict(real=np.float64), "f32": dict(real=np.float32),
            "e64": dict(real=np.float64, emulate_bf16=True), "e32": dict(real=np.float32, emulate_bf16=True)}


def sample_positions(spec, which):
    """Fixed positions inside every tensor of a network: name -> indices into the flat parameter vector."""
    out = {}
    for name, (sl, shape) in synth.param_slices(spec, which).items():
        n = int(np.prod(shape))
        rng = np.random.default_rng([which, n, len(name)])
        idx = np.sort(rng.choice(n, size=min(n, SAMPLES), replace=False)) + sl.start
        out[name] = idx
    return out


def pick_models(work, plan):
    if plan["models"] != "zipf":
        return list(plan["models"])
    b = work.batch_sizes
    order = np.argsort(b, kind="stable")
    return [int(order[-1]), int(order[len(order) // 2]), int(order[0])]      # largest, a median, the smallest


def run(config):
    plan = PLAN[config]
    work = synth.Workload(config)
    models = pick_models(work, plan)
    orcs = {tag: O.Oracle(work.spec, work.n_models, work.n_labels, **kw) for tag, kw in VARIANTS.items()}
    for l in models:
        for which in (0, 1):
            p = work.params(which, l)
            for o in orcs.values():
                o.set_params(which, l, p)
    pos = {which: sample_positions(work.spec, which) for which in (0, 1)}
    out = {"models": np.array(models), "batch_sizes": work.batch_sizes}
    lab = work.labels(single_label=3) if work.n_models == 1 else work.labels()
    t0 = time.time()
    for step in range(1, plan["steps"] + 1):
        z, x = work.noise(), work.images(lab)
        for tag, o in orcs.items():
            for l in models:
                o.train_step(lab, z, x, only_model=l)
            jd, jg, cnt = o.get_losses()
            out["%s_jd_%d" % (tag, step)] = np.array([jd[l] for l in models], np.float64)
            out["%s_jg_%d" % (tag, step)] = np.array([jg[l] for l in models], np.float64)
            for l in models:
                for which in (0, 1):
                    if step == 1:
                        g = o.get_grads(which, l)
                        for name, idx in pos[which].items():
                            out["%s_g_%d_%d_%s" % (tag, l, which, name)] = g[idx].astype(np.float64)
                    if step in plan["snaps"]:
                        th = o.get_params(which, l)
                        for name, idx in pos[which].items():
                            out["%s_p_%d_%d_%d_%s" % (tag, step, l, which, name)] = th[idx].astype(np.float64)
        d = {k: max(abs(out["%s_%s_%d" % (a, c, step)] - out["%s_%s_%d" % (b, c, step)]).max() /
                    abs(out["%s_%s_%d" % (b, c, step)]).min() for c in ("jd", "jg"))
             for k, (a, b) in dict(f32=("f32", "f64"), e32=("e32", "e64"), e64=("e64", "f64")).items()}
        print("config %d step %d done (%.0f s)  cost distance f32-f64 %.2e  e32-e64 %.2e  e64-f64 %.2e"
              % (config, step, time.time() - t0, d["f32"], d["e32"], d["e64"]), flush=True)
    np.savez_compressed(os.path.join(HERE, "config%d.npz" % config), **out)


if __name__ == "__main__":
    for c in ([int(a) for a in sys.argv[1:]] or sorted(PLAN)):
        run(c)
