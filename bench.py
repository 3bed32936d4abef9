"""Benchmark of the grouped per-label DC-CGAN training step on one MI355X.

A step is one pass of the whole hot path over one synthetic batch: route by label, G forward, D forward on real
and fake, the discriminator cost and backward, Adam on D, D again on the fake batch, the generator cost, backward
through D and G, Adam on G -- for every label model at once.  Inputs are resident in HBM before the timed region.
Prints one JSON line.
"""
import argparse
import json
import sys
import time

import numpy as np

PEAK = {"mfma_bf16": 2500.0, "mfma_fp32": 157.3, "hbm": 8000.0}   # TFLOP/s, TFLOP/s, GB/s (published MI355X figures)

# HBM bytes per launch from hardware counters (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, KiB per dispatch, averaged over the
# launches of a kernel instantiation in `bench.py --steps 3 --warmup 1 --no-profile --copy-probe`, config 2 bf16), scaled by what
# the same counters read for the 1 GiB elementwise probe (fetch x 2.0, write x 1.0).  Valid only for the kernel sources they
# were taken with: `sources` is the digest of csrc/ at that time, and the roofline reports null traffic when it differs.
MEASURED_TRAFFIC = {
    "sources": "1272be6df4352ca9",
    "workload": "config 2 bf16",
    "fetch_scale": 2.000, "write_scale": 1.000,
    "kib_per_launch": {
        "gemm_dense<128x128>": (103311, 108800),
        "gemm_up<256x256>": (453060, 275200),
        "gemm_up<256x128>": (159017, 435200),
        "gemm_dense+lrelu<256x128>": (154519, 614758),
        "gemm_down<256x256>": (498161, 209600),
        "wgrad<256x256>": (410476, 512076),
        "gemm_up+actbwd<256x128>": (584743, 614400),
        "wgrad<64x128>": (460879, 25605),
        "gemm_dense<256x128>": (103311, 409886),
        "wgrad<256x128>": (52079, 410066),
    },
}


def sources_digest():
    import glob
    import hashlib
    import os
    h = hashlib.sha256()
    root = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2102_10485_amd", "csrc")
    for f in sorted(glob.glob(os.path.join(root, "*.hip")) + glob.glob(os.path.join(root, "*.h"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(kernel, workload):
    m = MEASURED_TRAFFIC
    if m["sources"] != sources_digest() or m["workload"] != workload or kernel not in m["kib_per_launch"]:
        return None
    fetch, write = m["kib_per_launch"][kernel]
    return 1024.0 * (fetch * m["fetch_scale"] + write * m["write_scale"])


DESCR = {
    0: "config 0: one conditional pair, 28x28x1, batch 64, fp32",
    1: "config 1: 10 label models, 28x28x1, batch 128 per label",
    2: "config 2: 100 label models, 32x32x3, batch 64 per label",
    3: "config 3: 8 label models (one GPU's share of 1000), 64x64x3, batch 128 per label",
    4: "config 4: 100 label models, 32x32x3, rank-Zipf batch sizes in [16, 256], 6400 images",
}


def cpu_baseline(work, min_seconds=10.0, max_models=16):
    """The oracle as it stands, on the host cores, for one step of a bounded sample of the same workload."""
    import oracle as O
    spec = work.spec
    orc = O.Oracle(spec, work.n_models, work.n_labels)
    lab = work.labels(single_label=3) if work.n_models == 1 else work.labels()
    x = work.images(lab)
    z = work.noise()
    models = []
    t0 = time.perf_counter()
    images = 0
    for l in range(min(max_models, work.n_models)):       # whole label models until the sample is >= ~10 s of work
        orc.train_step(lab, z, x, only_model=l)
        images += int(orc.get_losses()[2][l])
        models.append(l)
        if time.perf_counter() - t0 >= min_seconds:
            break
    dt = time.perf_counter() - t0
    orc.close()
    return {"value": images / dt, "unit": "images/s", "cores": O.threads(), "kind": "oracle",
            "sample": "1 step of %d of %d label models (%d images) in %.1f s, fp64 direct loops"
                      % (len(models), work.n_models, images, dt)}


def other_rows(args, torch, binding, work, gan, prec, prec_name, d_lab, d_real, d_noise, n):
    """The two rows next to the training step, timed the same way (inputs resident, warm-up, K timed calls)."""
    rng = np.random.default_rng(work.seed + 77)
    descr = DESCR[args.config] + (", %s" % prec_name)
    if args.row == "sample":
        # a few training steps first so that the running statistics are those of a trained-ish model
        for i in range(2):
            gan.train_step(d_lab.data_ptr(), d_noise[i].data_ptr(), d_real.data_ptr(), n)
        prior = np.bincount(work.labels(), minlength=work.n_labels).astype(np.float64)      # the class frequencies of the workload
        d_u = torch.from_numpy(rng.random(n).astype(np.float32)).cuda()
        out = torch.empty((n, work.spec["img_c"], work.spec["img_hw"], work.spec["img_hw"]), dtype=torch.float32, device="cuda")
        labels = torch.empty(n, dtype=torch.int32, device="cuda")

        def call(i):
            gan.sample(prior, d_u.data_ptr(), d_noise[i % 2].data_ptr(), n, out.data_ptr(), labels.data_ptr(), 1)
        metric, unit = "mixture samples/sec (class draw + per-label generators, running statistics)", "images/s"
    else:
        def call(i):
            st, F = gan.anova_f(d_lab.data_ptr(), d_real.data_ptr(), n, work.spec["img_c"])
            assert st == 0 and np.all(np.isfinite(F))
        metric, unit = "images/sec through the per-channel ANOVA F-statistic (device reductions + host finish)", "images/s"
    for i in range(args.warmup):
        call(i)
    torch.cuda.synchronize()
    if args.row == "sample" and not args.no_profile:
        gan.profile_enable(True, gemm_only=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        call(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out_j = {"metric": metric, "value": n * args.steps / dt, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
             "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
             "dtype": prec_name if args.row == "sample" else "f64", "data": "synthetic",
             "config": {"workload": descr + ", row: " + args.row, "images_per_step": n}}
    if args.row == "sample" and not args.no_profile:
        prof = gan.profile_read()
        gan.profile_enable(False)
        dom = max((k for k in prof if k != MFMA_BUSY), key=lambda k: prof[k]["ms"])
        r = prof[dom]
        peak = PEAK["mfma_bf16"] if prec_name == "bf16" else PEAK["mfma_fp32"]
        tf = r["flops"] / (r["ms"] * 1e9)
        out_j["roofline"] = {"kernel": dom, "bound": "mfma", "achieved": tf, "peak": peak, "unit": "TFLOP/s", "frac": tf / peak,
                             "traffic": None, "avg_launch_ms": r["ms"] / max(r["launches"], 1)}
    elif args.row == "anova":
        nbytes = float(n) * work.spec["img_c"] * work.spec["img_hw"] ** 2 * 4
        gbps = nbytes * args.steps / dt / 1e9
        out_j["roofline"] = {"kernel": "anova (whole call, including the synchronising copy back)", "bound": "hbm", "achieved": gbps,
                             "peak": PEAK["hbm"], "unit": "GB/s", "frac": gbps / PEAK["hbm"], "traffic": None}
    gan.close()
    print(json.dumps(out_j))


def build_workload(args, config, torch, binding, synth, prec_name, single_pair=None, spec_name=None):
    """Context, resident inputs and description of one workload (spec_name: config's label models with other networks)."""
    work = synth.Workload(config, spec=spec_name)
    prec = binding.BF16 if prec_name == "bf16" else binding.FP32
    n = work.n
    lab = work.labels(single_label=3) if work.n_models == 1 else work.labels()
    spec, n_models, n_labels, descr = work.spec, work.n_models, work.n_labels, DESCR[config]
    if spec_name:
        descr += ", networks '%s'" % spec_name
    img_lab = lab                              # the classes the real images are drawn from
    if single_pair:
        spec, n_models = dict(work.spec), 1
        if single_pair == "cgan":
            n_labels = max(work.n_labels, 2)
            spec["cond_g"] = spec["cond_d"] = n_labels
            # one model owns the whole batch, and the library addresses one model's slice of any tensor with 32-bit
            # byte offsets; the largest slice is the patch matrix of D's first layer
            kc = -(-(16 * spec["img_c"] + 9 * n_labels + 1) // 64) * 64
            row_bytes = kc * (2 if prec_name == "bf16" else 4) * (spec["img_hw"] // 2) ** 2
            n = min(n, ((1 << 31) - 1) // row_bytes // 64 * 64)
            descr = "one conditional pair (all %d labels) of config %d's widths, batch %d" % (n_labels, config, n)
        else:
            n_labels = 1
            spec["cond_g"] = spec["cond_d"] = 0
            descr = "one unconditional pair of config %d's widths, batch %d" % (config, n)
            lab = np.zeros_like(lab)
        lab, img_lab = lab[:n], img_lab[:n]
    cfg = binding.make_config(spec, n_models, n_labels, n, prec, seed=work.seed)
    gan = binding.Gan(cfg, torch.cuda.current_stream().cuda_stream)
    d_lab = torch.from_numpy(lab).cuda()
    d_real = torch.from_numpy(work.images(img_lab)).cuda()
    d_noise = [torch.from_numpy(work.noise()[:n].copy()).cuda() for _ in range(2)]
    torch.cuda.synchronize()
    return dict(work=work, gan=gan, prec=prec, n=n, n_models=n_models, descr=descr, d_lab=d_lab, d_real=d_real, d_noise=d_noise)


def time_steps(torch, w, steps, warmup):
    """W warm-up steps, then K steps between two synchronisations: milliseconds per step (no per-kernel timing on)."""
    gan, n = w["gan"], w["n"]

    def step(i):
        gan.train_step(w["d_lab"].data_ptr(), w["d_noise"][i % 2].data_ptr(), w["d_real"].data_ptr(), n)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    jd, jg, cnt = gan.get_losses()
    assert np.all(np.isfinite(jd)) and np.all(np.isfinite(jg)) and int(cnt.sum()) == n
    return 1e3 * dt / steps


def kernel_timings(torch, w, steps, detail=False, gemm_only=False):
    """`steps` more steps with HIP events around the launches on the library's stream: per kernel family the launches
    per step, milliseconds, and the algorithmic flops and bytes those launches stood for."""
    gan, n = w["gan"], w["n"]
    gan.profile_enable(True, detail=detail, gemm_only=gemm_only)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        gan.train_step(w["d_lab"].data_ptr(), w["d_noise"][i % 2].data_ptr(), w["d_real"].data_ptr(), n)
    torch.cuda.synchronize()
    ms_instr = 1e3 * (time.perf_counter() - t0) / steps
    prof = gan.profile_read()
    gan.profile_enable(False)
    kern = {}
    for name, r in prof.items():
        kern[name] = {"launches_per_step": r["launches"] / steps, "ms_per_step": r["ms"] / steps,
                      "avg_launch_ms": r["ms"] / max(r["launches"], 1),
                      "tflops": r["flops"] / (r["ms"] * 1e9) if r["ms"] > 0 else 0.0,
                      "gbps": r["bytes"] / (r["ms"] * 1e6) if r["ms"] > 0 else 0.0,
                      "flops_per_launch": r["flops"] / max(r["launches"], 1), "bytes_per_launch": r["bytes"] / max(r["launches"], 1)}
    return kern, ms_instr


MFMA_BUSY = "(mfma busy)"


def is_mfma(name):
    return name.startswith("gemm_") or name.startswith("wgrad")


def mfma_summary(kern, peak):
    """All GEMM and weight-gradient launches together: their algorithmic flops over the time during which at least one
    of them ran (the library runs weight gradients beside the data-gradient chain on a second stream, so the launches'
    own durations, which the per-kernel table shows, add up to more than that)."""
    gemm = [k for k in kern if is_mfma(k)]
    fl = sum(kern[k]["flops_per_launch"] * kern[k]["launches_per_step"] for k in gemm)
    busy = kern[MFMA_BUSY]["ms_per_step"] if MFMA_BUSY in kern else sum(kern[k]["ms_per_step"] for k in gemm)
    return {"tflops": fl / (busy * 1e9), "frac_of_peak": fl / (busy * 1e9) / peak, "ms_per_step": busy,
            "sum_of_launch_ms_per_step": sum(kern[k]["ms_per_step"] for k in gemm)}


# the bandwidth-bound kernel families reported against the HBM peak (algorithmic bytes: every input read once, every
# output written once, in the storage type; Adam: 28 B per parameter plus the storage-type copies)
ELEMENTWISE = ("adam", "bn_apply", "bn_bwd_reduce", "bn_bwd_apply", "im2col", "up_img", "head_fwd", "head_bwd_data", "head_bwd_w",
               "stage", "transpose_w")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="workload 0-4 (default: 2, the largest)")
    ap.add_argument("--precision", choices=["fp32", "bf16"], default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="no per-kernel timing pass (no roofline object)")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the short runs of the other workloads (`configs` object)")
    ap.add_argument("--detail", action="store_true", help="per-kernel pass with one line per layer shape (analysis runs)")
    ap.add_argument("--row", choices=["train", "sample", "anova"], default="train",
                    help="train (default): the training step; sample: mixture sampling (Eq. 5) of images_per_step images per "
                         "call; anova: the per-channel F-statistic of one batch")
    ap.add_argument("--single-pair", choices=["cgan", "gan"], default=None,
                    help="train row on the paper's comparison systems instead of the label models: ONE pair of the same widths over "
                         "the same flat batch -- cgan: conditioned on the label of every sample (Tables 3 and 4); gan: unconditional "
                         "(Tables 1 and 2)")
    ap.add_argument("--networks", choices=["paper32"], default=None,
                    help="train row with the config's labels and batches but other networks: paper32 = the generator and "
                         "discriminator exactly as the paper's Tables 1 and 2 print them (32x32x3)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="before the timed region, run one elementwise kernel over 1 GiB (reads 1 GiB, writes 1 GiB: known traffic for scaling "
                         "hardware byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the library runs on one GPU (the label models shard across GPUs with no per-step traffic, "
                 "each GPU running this same step on its labels); run with --gpus 1")

    import torch
    from paper_2102_10485_amd import binding, synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP library has no CPU fallback")
    torch.cuda.set_device(0)
    if args.single_pair and args.row != "train":
        sys.exit("bench.py: --single-pair goes with the train row")
    prec_name = args.precision or synth.Workload(args.config).precision
    w = build_workload(args, args.config, torch, binding, synth, prec_name, args.single_pair, args.networks)
    work, gan, n = w["work"], w["gan"], w["n"]

    if args.row != "train":
        return other_rows(args, torch, binding, work, gan, w["prec"], prec_name, w["d_lab"], w["d_real"], w["d_noise"], n)

    if args.copy_probe:
        time_steps(torch, w, 1, 1)
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)      # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    # the timed region: K steps with nothing but the step's own launches in the stream
    ms_per_step = time_steps(torch, w, args.steps, args.warmup)
    out = {
        "metric": "training images/sec (G+D step, all labels)", "value": n * 1e3 / ms_per_step, "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": prec_name, "data": "synthetic",
        "config": {"workload": w["descr"] + (", %s" % prec_name), "n_models": w["n_models"], "images_per_step": n,
                   "batch_sizes": "min %d / median %d / max %d" % (work.batch_sizes.min(), np.median(work.batch_sizes),
                                                                  work.batch_sizes.max()) if not args.single_pair else str(n)},
    }
    peak = PEAK["mfma_bf16"] if prec_name == "bf16" else PEAK["mfma_fp32"]
    if not args.no_profile:
        # the same K steps again with HIP events on the library's stream around the MFMA launches (the roofline's
        # launch durations), then a few with events around every launch (the bandwidth-bound families)
        kern, ms_instr = kernel_timings(torch, w, args.steps, detail=args.detail, gemm_only=not args.detail)
        if args.detail:
            for k, v in sorted(kern.items(), key=lambda kv: -kv[1]["ms_per_step"]):
                print("%-44s %5.1f launches %8.3f ms/step %8.1f TFLOP/s %8.1f GB/s" % (k, v["launches_per_step"], v["ms_per_step"], v["tflops"], v["gbps"]), file=sys.stderr)
        gemm = [k for k in kern if is_mfma(k)]
        dom = max(gemm, key=lambda k: kern[k]["ms_per_step"])
        traffic = measured_traffic(dom, "config %d %s" % (args.config, prec_name))
        out["roofline"] = {"kernel": dom, "bound": "mfma", "achieved": kern[dom]["tflops"], "peak": peak,
                           "unit": "TFLOP/s", "frac": kern[dom]["tflops"] / peak, "traffic": traffic,
                           "traffic_unit": "HBM bytes per launch",
                           "traffic_source": ("stored hardware counters (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this "
                                              "command with these kernel sources, profiles/hbm_traffic_config2_bf16.md), not measured by "
                                              "this run") if traffic is not None else
                                             "none: the kernel sources changed since the counters were taken",
                           "algorithmic_flops_per_launch": kern[dom]["flops_per_launch"],
                           "algorithmic_bytes": kern[dom]["bytes_per_launch"],
                           "avg_launch_ms": kern[dom]["avg_launch_ms"],
                           "timing": "HIP events around every launch of this kernel, on the stream it is launched on, in %d steps "
                                     "that repeat the timed region (%.3f ms/step with the events in the streams); launches that "
                                     "run beside another stream's kernels are timed as they ran" % (args.steps, ms_instr)}
        out["conv_mfma"] = mfma_summary(kern, peak)
        allk, ms_all = kernel_timings(torch, w, min(args.steps, 5))
        out["elementwise"] = {k: {"launches_per_step": round(v["launches_per_step"], 2), "ms_per_step": round(v["ms_per_step"], 4),
                                  "gbps": round(v["gbps"], 1), "frac_of_hbm_peak": round(v["gbps"] / PEAK["hbm"], 4)}
                              for k, v in sorted(allk.items(), key=lambda kv: -kv[1]["ms_per_step"]) if k in ELEMENTWISE}
        out["elementwise_note"] = ("algorithmic bytes (inputs read once, outputs written once, storage type; Adam 28 B per parameter + "
                                   "storage copies) / HIP-event time, against 8 TB/s; %d steps with events around every launch" % min(args.steps, 5))
        # the same figures against what the simplest kernels reach on this chip (register-only MFMA loop, plain copy)
        mfma_meas = binding.probe_mfma(w["prec"], torch.cuda.current_stream().cuda_stream)
        copy_meas = binding.probe_copy(1 << 30, torch.cuda.current_stream().cuda_stream)
        out["measured_ceilings"] = {"mfma_loop_tflops": mfma_meas, "device_copy_gbps": copy_meas,
                                    "roofline_frac_of_mfma_loop": kern[dom]["tflops"] / mfma_meas,
                                    "conv_mfma_frac_of_mfma_loop": out["conv_mfma"]["tflops"] / mfma_meas}
        out["kernels"] = {k: {kk: round(vv, 4) for kk, vv in v.items() if not kk.endswith("_per_launch")}
                          for k, v in sorted(kern.items(), key=lambda kv: -kv[1]["ms_per_step"]) if k != MFMA_BUSY}
    gan.close()
    del w
    if not args.no_profile and not args.no_other_configs and not args.single_pair and not args.networks and args.config == 2:
        # the other workloads and the comparison systems, a few steps each (parity-test cases, not the headline)
        others = {}
        runs = [("config 0 fp32", 0, "fp32", None, None), ("config 1 fp32", 1, "fp32", None, None), ("config 1 bf16", 1, "bf16", None, None),
                ("config 2 fp32", 2, "fp32", None, None),
                ("config 3 bf16", 3, "bf16", None, None), ("config 4 bf16", 4, "bf16", None, None),
                ("single pair gan (config 2 widths) bf16", 2, "bf16", "gan", None),
                ("single pair cgan (config 2 widths) bf16", 2, "bf16", "cgan", None),
                # config 2's label models with the networks exactly as the paper's Tables 1 and 2 print them
                ("paper networks (Tables 1-2), config 2 labels and batch, bf16", 2, "bf16", None, "paper32"),
                ("paper networks (Tables 1-2), config 2 labels and batch, fp32", 2, "fp32", None, "paper32")]
        for name, cfg_id, pn, sp, spec_name in runs:
            torch.cuda.empty_cache()
            ww = build_workload(args, cfg_id, torch, binding, synth, pn, sp, spec_name)
            ms = time_steps(torch, ww, 10, 3)
            kk, _ = kernel_timings(torch, ww, 5, gemm_only=True)
            pk = PEAK["mfma_bf16"] if pn == "bf16" else PEAK["mfma_fp32"]
            mm = mfma_summary(kk, pk)
            others[name] = {"workload": ww["descr"], "ms_per_step": round(ms, 4), "images_per_s": round(ww["n"] * 1e3 / ms, 1),
                            "conv_mfma_tflops": round(mm["tflops"], 2), "conv_mfma_frac_of_peak": round(mm["frac_of_peak"], 4),
                            "mfma_peak_tflops": pk}
            ww["gan"].close()
            del ww
        out["configs"] = others
    if not args.no_cpu_baseline and not args.single_pair and not args.networks:
        out["cpu_baseline"] = cpu_baseline(synth.Workload(args.config))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
