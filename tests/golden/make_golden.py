"""Writes the stored oracle results for the full-size workloads (calls only `oracle/` and the input generators).

    python tests/golden/make_golden.py [config ...]

For each configuration the CPU oracle is stepped on the same seeded inputs the GPU test will use, for the stated
subset of label models (the models are independent, Eq. 5 of the paper, so a subset is exact for its members).
Stored per configuration: the two costs of every step, and, after the last step, every parameter tensor sampled
at fixed seeded positions (up to 4096 per tensor).  The same is stored from the oracle's loops compiled in single
precision: its distance from the fp64 result measures how strongly the iteration amplifies rounding at that point.
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

# config -> (models checked, steps, param snapshots after these steps)
PLAN = {
    0: dict(models=[0], steps=5, snaps=[1, 5], single=True),
    1: dict(models=[0, 9], steps=50, snaps=[1, 5, 50], single=True),
    2: dict(models=[0, 49, 99], steps=3, snaps=[3], single=True),
    3: dict(models=[0, 7], steps=3, snaps=[3], single=True),
    4: dict(models="zipf", steps=3, snaps=[3], single=True),
}
SAMPLES = 4096


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
    reals = [np.float64] + ([np.float32] if plan["single"] else [])
    orcs = {r: O.Oracle(work.spec, work.n_models, work.n_labels, real=r) for r in reals}
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
        for r, o in orcs.items():
            tag = "f64" if r is np.float64 else "f32"
            for l in models:
                o.train_step(lab, z, x, only_model=l)
            jd, jg, cnt = o.get_losses()
            out["%s_jd_%d" % (tag, step)] = np.array([jd[l] for l in models], np.float64)
            out["%s_jg_%d" % (tag, step)] = np.array([jg[l] for l in models], np.float64)
            if step in plan["snaps"]:
                for l in models:
                    for which in (0, 1):
                        th = o.get_params(which, l)
                        for name, idx in pos[which].items():
                            out["%s_p_%d_%d_%d_%s" % (tag, step, l, which, name)] = th[idx].astype(np.float64)
        print("config %d step %d done (%.0f s)" % (config, step, time.time() - t0), flush=True)
    np.savez_compressed(os.path.join(HERE, "config%d.npz" % config), **out)


if __name__ == "__main__":
    for c in ([int(a) for a in sys.argv[1:]] or sorted(PLAN)):
        run(c)
