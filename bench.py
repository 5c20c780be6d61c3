#!/usr/bin/env python3
"""Benchmark of the packed training step on one MI355X.

A "step" is one pass of the whole hot path over one synthetic batch: shared-input forward of all
K members, softmax cross-entropy, backward, and the per-member-learning-rate SGD update, inputs
resident in HBM before timing starts.  The default run measures all five configurations (c1 .. c5)
and prints ONE JSON line: the headline fields are those of the largest one, c5 (K = 4 ResNet-style
CNNs on 64 x 64 images, bf16 operands, batch 64), and `configs` carries one record per configuration.
`--workload cN` measures that configuration alone (and is what the profiler runs use).

Protocol (the paper's Section 4.1): inputs resident on the device, warm-up steps dropped, then
5 repeats of exactly --steps steps each, every repeat between two device synchronisations; the
median repeat gives `ms_per_step` and `value`, the mean is reported beside it.

Per configuration it reports
  - the unpacked baseline of the paper's Eq. 1-3: T_s(Seq) = sum of the step times of K packs of
    one member each (same library, same stream), speed-up T_s(Seq)/T_s(Pack) and IMPV;
  - `roofline`: the dominant kernel of the step (chosen by measured time), its algorithmic bytes
    or flops per launch divided by its average duration from HIP events on the pack's stream;
  - `cpu_baseline`: the CPU oracle (float64, members trained separately) timed on this host on a
    bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
REPEATS = 5                    # timed repeats per configuration (Section 4.1: mean of 5 runs)
HEADLINE = "c5"                # the largest configuration that fits one GPU

# HBM bytes per launch of a dominant kernel from hardware counters (FETCH_SIZE and WRITE_SIZE, each
# scaled by a copy kernel of known size; the summary under profiles/ named here), valid only for the
# kernel source it was measured on (hash of the kernel's text): {workload: {...}}.
COUNTER_TRAFFIC = {
    "c2": {"kernel": "gemm_lin_dw+sgd", "bytes": 373.4e6, "kernel_sha": "4df60122164a5d1a", "sources": "staged",
           "profile": "profiles/c2_weight_gradient_update_hbm_counters.txt"},
    "c5": {"kernel": "gemm_conv_dw+sgd", "bytes": 1108.6e6, "kernel_sha": "e8dbb0d29c1761f9", "sources": "conv_dw_halo",
           "profile": "profiles/c5_convolution_weight_gradient_hbm_counters.txt"},
}


def _kernel_sha(sources):
    """Hash of the code that decides a launch's memory traffic (comments and layout removed): the kernel and the
    order in which the planner deals its tiles to the XCDs.  Counter figures are only reported while it matches."""
    import hashlib
    import re
    csrc = os.path.join(ROOT, "paper_2002_02885_amd", "csrc")
    api = open(os.path.join(csrc, "pack_api.cpp")).read()
    c, d = api.index("struct TileOrder"), api.index("void set_row_space(")
    e, f = api.index("void emit_gemm_launch("), api.index("    Launch L;\n    L.kind = L_GEMM;")
    code = api[c:d] + api[e:f]
    if sources == "staged":
        src = open(os.path.join(csrc, "pack_kernels.hip")).read()
        a, b = src.index("namespace packk {"), src.index("template <int MODE, typename T, int WM, int WN, int TN>\n__global__")
        code += open(os.path.join(csrc, "gemm_fetch.h")).read() + src[a:b]
    else:
        code += open(os.path.join(csrc, "pack_conv_dw.hip")).read() + open(os.path.join(csrc, "conv_dw_halo.h")).read()
    code = re.sub(r"/\*.*?\*/", "", code, flags=re.S)
    code = re.sub(r"//[^\n]*", "", code)
    return hashlib.sha256("".join(code.split()).encode()).hexdigest()[:16]


def _time_steps(pk, x, y, lr, steps, torch):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        pk.step(x.data_ptr(), y.data_ptr(), lr)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def _search(args, np, torch, wl):
    """Hyperband and its pack-aware variants (paper Section 5.3, Table 4) with the library's tuner."""
    from paper_2002_02885_amd import tuner
    in_shape, n, dtype = (1, 1, 3072), 50000, wl.BF16          # CIFAR-10's training set shape, flattened
    X, Y = wl.labelled_dataset(5, n, in_shape, dtype)
    data = torch.from_numpy(X).to(torch.bfloat16).cuda().contiguous()
    labels = torch.from_numpy(Y).cuda().contiguous()
    family = tuner.mlp_family([512], 10)

    def init(cfg, layers):
        seed = 7919 + ((cfg[0] * 4 + cfg[1]) * 6 + cfg[2]) * 4 + cfg[3]
        return wl.draw_weights(np.random.default_rng(np.random.PCG64(seed)), layers, in_shape, dtype)

    space = tuner.all_configurations()
    rng = np.random.default_rng(17)
    from paper_2002_02885_amd import binding
    sampled = [[space[i] for i in rng.choice(len(space), size=rungs[0][0], replace=False)]
               for rungs in binding.hyperband_plan(81, 3)]
    res = {}
    # the similarity threshold is the user's knob (Section 5.2): 4 packs near neighbours only, 17 (the
    # diameter of the space) lets memory alone bound a group
    for name, policy, threshold in (("none", "none", 0), ("knn", "knn", 4), ("knn_threshold_17", "knn", 17),
                                    ("random", "random", 0), ("batchsize", "batchsize", 0)):
        t = tuner.Tuner(data.data_ptr(), labels.data_ptr(), n, in_shape, dtype, family, init,
                        steps_per_unit=args.search_units, policy=policy, capacity_bytes=16 << 30, threshold=threshold,
                        random_m=8, seed=3, sync=torch.cuda.synchronize)
        t0 = time.perf_counter()
        best, loss = t.run(81, 3, sampled)
        wall = time.perf_counter() - t0
        res[name] = {"wall_s": wall, "train_s": t.train_seconds, "packs": t.packs_built, "best": list(best), "best_loss": loss,
                       "largest_group": max(len(g) for e in t.log for g in e["groups"])}
    assert len(set((tuple(r["best"]), r["best_loss"]) for r in res.values())) == 1, "policies must agree on the winner"
    out = {"metric": "hyperband training time", "unit": "s", "higher_is_better": False, "n_gpus": 1,
           "config": {"workload": "Hyperband R=81 eta=3 over the 1056 configurations of Table 3, MLP 3072-512-10 bf16, "
                                  f"50000 synthetic samples, {args.search_units} steps per resource unit"},
           "value": res["knn"]["train_s"], "policies": res,
           "time_saved_vs_plain": {p: 1.0 - res[p]["train_s"] / res["none"]["train_s"] for p in res if p != "none"},
           "data": "synthetic", "dtype": "bf16"}
    print(json.dumps(out))


def _cpu_baseline(w, args, np, wl, lr, budget_s):
    """The oracle as it stands, timed on this host on a bounded sample of workload `w`: whole steps of
    single members, members in turn, until `budget_s` seconds have passed.  A member whose step would
    take longer than the budget by itself (the convolution configurations) is trained on the leading
    rows of the shared batch only, as many as fit the budget; the rate is rows x models per second
    either way."""
    from oracle import pack_oracle as po
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    mode = "weights" if w.dtype == wl.BF16 else "exact"
    opts = [{"kind": args.optimizer}] * w.K if args.optimizer != "sgd" else None
    blobs = [b.astype(np.float64) for b in w.weights]
    x64 = w.x.astype(np.float64)
    lr64 = lr.astype(np.float64)

    def member_step(k, rows):
        t0 = time.perf_counter()
        po.train_pack([w.models[k]], w.in_shape, [blobs[k]], [rows], lr64[k:k + 1], x64, w.labels, 1, mode=mode,
                      optimizers=opts[k:k + 1] if opts else None)
        return time.perf_counter() - t0

    # grow the slice (2, 8, 32, ... rows) while four times the last time still fits the budget
    full = int(w.batch[0])
    rows = min(2, full)
    t_rows = member_step(0, rows)
    while rows < full and 4.0 * t_rows <= budget_s:
        rows = min(full, 4 * rows)
        t_rows = member_step(0, rows)
    if rows < full:
        more = min(full, int(rows * budget_s / t_rows))
        if more > rows:
            print(f"cpu_baseline {w.name}: one member on {more} of {full} rows ...", file=sys.stderr, flush=True)
            rows, t_rows = more, member_step(0, more)
        return {"value": rows / t_rows, "unit": "samples*models/s", "cores": int(threads), "kind": "oracle",
                "sample": f"one step of member 0 of {w.name} on the leading {rows} of its {full} rows "
                          f"({t_rows:.1f} s; numpy float64)"}
    n_member_steps, samples_done, t_cpu = 0, 0, 0.0
    print(f"cpu_baseline {w.name}: single-member steps for about {budget_s:.0f} s ...", file=sys.stderr, flush=True)
    while t_cpu < budget_s and n_member_steps < 50 * w.K:
        k = n_member_steps % w.K
        t_cpu += member_step(k, int(w.batch[k]))
        samples_done += int(w.batch[k])
        n_member_steps += 1
    return {"value": samples_done / t_cpu, "unit": "samples*models/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n_member_steps} single-member steps of {w.name} ({n_member_steps / w.K:.2f} steps of the pack, "
                      f"{t_cpu:.1f} s; numpy float64, members trained one after another)"}


def bench_config(name, args, np, torch, wl, binding, extras, cpu_budget_s):
    """Measures one configuration; returns its record (the fields of the JSON line that depend on it)."""
    w = wl.CONFIGS[name]()
    stream = torch.cuda.current_stream().cuda_stream
    x = torch.from_numpy(w.x)
    x = (x.to(torch.bfloat16) if w.dtype == wl.BF16 else x).cuda().contiguous()
    y = torch.from_numpy(w.labels).cuda().contiguous()

    if args.different_inputs:
        # K independent seeded batches, stacked [K][B, ...]; single-member packs read block 0
        g = torch.Generator().manual_seed(1234)
        xs = torch.rand((w.K,) + tuple(w.x.shape), generator=g, dtype=torch.float32)
        x = (xs.to(torch.bfloat16) if w.dtype == wl.BF16 else xs).cuda().contiguous()
        y = torch.randint(0, w.n_classes, (w.K, w.B), generator=g, dtype=torch.int32).cuda().contiguous()

    def make(models, batch, weights, on_stream=None):
        pk = binding.Pack(w.B, w.in_shape, w.dtype, models, batch, stream=stream if on_stream is None else on_stream)
        if args.different_inputs and len(models) > 1:
            pk.set_input_mode(True)
        for k, blob in enumerate(weights):
            pk.write_weights(k, blob)
            if args.optimizer != "sgd":
                pk.set_optimizer(k, {"kind": args.optimizer})
        return pk

    # a tiny learning rate keeps hundreds of timed steps finite; arithmetic and traffic per step
    # do not depend on its value
    lr = np.full(w.K, 1e-6, dtype=np.float32)

    pk = make(w.models, w.batch, w.weights)
    n_params = sum(pk.num_params(k) for k in range(w.K))
    flops = sum(wl.step_flops(m, w.in_shape, b) for m, b in zip(w.models, w.batch))
    samples_models = float(sum(w.batch))

    # warm-up, with every launch timed once to find the dominant kernel
    for _ in range(max(args.warmup - 5, 1)):
        pk.step(x.data_ptr(), y.data_ptr(), lr)
    pk.profile_start(-1)
    for _ in range(5):
        pk.step(x.data_ptr(), y.data_ptr(), lr)
    ms, cnt = pk.profile_stop()
    names = [pk.launch_name(i) for i in range(pk.num_launches())]
    per_launch = ms / np.maximum(cnt, 1)
    dom = int(np.argmax(per_launch))
    breakdown = {}
    for nm, t in zip(names, per_launch):
        breakdown[nm] = breakdown.get(nm, 0.0) + float(t) * 1e3
    # timed region: REPEATS repeats of EXACTLY --steps steps; the dominant launch of every 4th step is
    # bracketed by events (an event pair costs about 10 us of stream time, so not every step carries one)
    pk.profile_start(dom, every=4)
    repeats = [_time_steps(pk, x, y, lr, args.steps, torch) for _ in range(REPEATS)]
    ms, cnt = pk.profile_stop()
    t_pack = float(np.median(repeats))
    dom_ms = float(ms[dom] / max(cnt[dom], 1))
    loss = pk.read_loss()
    assert np.all(np.isfinite(loss)), loss
    launches = pk.num_launches()
    dev_bytes = pk.device_bytes()
    dom_flops = pk.launch_flops(dom)
    dom_bytes = pk.launch_bytes(dom)
    pk.destroy()

    dom_name = names[dom]
    if dom_name in ("sgd_update", "optimizer_update"):
        # master r+w, gradient r, each state array r+w, (+ bf16 copy w)
        bpp = 12.0 + 8.0 * {"sgd": 0, "momentum": 1, "adagrad": 1, "adam": 2}[args.optimizer] + (2.0 if w.dtype == wl.BF16 else 0.0)
        achieved = n_params * bpp / (dom_ms * 1e-3) / 1e9
        roofline = {"kernel": dom_name, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": None, "avg_ms": dom_ms,
                    "algorithmic_bytes": n_params * bpp}
    else:
        # a matrix-product launch (with the SGD update fused into it when the name says so): the
        # roofline that bounds it is the slower of its algorithmic bytes at the HBM peak and its
        # flops at the MFMA peak
        peak = MFMA_PEAK_TFLOPS[w.dtype]
        t_hbm, t_mfma = dom_bytes / (HBM_PEAK_GBS * 1e9), dom_flops / (peak * 1e12)
        traffic = None
        try:
            known = COUNTER_TRAFFIC.get(w.name)
            if (known and args.optimizer == "sgd" and not args.different_inputs and dom_name == known["kernel"]
                    and _kernel_sha(known["sources"]) == known["kernel_sha"]):
                traffic = known["bytes"]
        except (OSError, ValueError):
            pass
        if t_hbm >= t_mfma:
            achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
            roofline = {"kernel": dom_name, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "avg_ms": dom_ms,
                        "algorithmic_bytes": dom_bytes, "algorithmic_flops": dom_flops}
        else:
            achieved = dom_flops / (dom_ms * 1e-3) / 1e12
            roofline = {"kernel": dom_name, "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                        "frac": achieved / peak, "traffic": traffic, "avg_ms": dom_ms,
                        "algorithmic_bytes": dom_bytes, "algorithmic_flops": dom_flops}

    rec = {
        "workload": f"{w.name}: K={w.K} packed models, batch {w.B}, input {list(w.in_shape)}, "
                    f"{n_params} parameters, optimiser {args.optimizer}"
                    + (", every member on its own batch" if args.different_inputs else ""),
        "K": w.K, "batch": w.B, "launches_per_step": launches, "device_bytes": dev_bytes,
        "dtype": "bf16" if w.dtype == wl.BF16 else "f32",
        "value": samples_models / t_pack, "unit": "samples*models/s",
        "ms_per_step": t_pack * 1e3, "ms_per_step_mean": float(np.mean(repeats)) * 1e3,
        "ms_per_step_repeats": [round(r * 1e3, 5) for r in repeats],
        "tflops": flops / t_pack / 1e12,
        "tflops_frac_of_mfma_peak": flops / t_pack / 1e12 / MFMA_PEAK_TFLOPS[w.dtype],
        "kernel_us": {k: round(v, 2) for k, v in breakdown.items()},
        "launch_us": [[nm, round(float(t) * 1e3, 2)] for nm, t in zip(names, per_launch)],
        "roofline": roofline,
    }

    if extras and not args.no_ceilings:
        # what this GPU delivers on the simplest code of each kind, beside the published peaks used above
        ceil = {"hbm_copy_GBps": binding.measure_ceiling("hbm_copy", stream),
                "mfma_bf16_TFLOPs": binding.measure_ceiling("mfma_bf16", stream),
                "mfma_fp32_TFLOPs": binding.measure_ceiling("mfma_fp32", stream)}
        rec["measured_ceilings"] = {k: round(v, 1) for k, v in ceil.items()}
        own = ceil["hbm_copy_GBps"] if roofline["bound"] == "hbm" else ceil["mfma_bf16_TFLOPs" if w.dtype == wl.BF16 else "mfma_fp32_TFLOPs"]
        roofline["frac_of_measured_ceiling"] = roofline["achieved"] / own

    if args.calibrate_copy and extras:
        a = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        for _ in range(5):
            torch.add(a, 0.0, out=b)
        torch.cuda.synchronize()
        del a, b

    if args.optimizer == "sgd" and not args.no_unpacked and n_params > 1_000_000:
        # the same step with the update as a launch of its own (the library's measuring aid): how the
        # stand-alone update kernel fares against its own HBM roofline, and what fusing it buys
        os.environ["PACK_NO_FUSED_UPDATE"] = "1"
        try:
            ref = make(w.models, w.batch, w.weights)
        finally:
            del os.environ["PACK_NO_FUSED_UPDATE"]
        for _ in range(5):
            ref.step(x.data_ptr(), y.data_ptr(), lr)
        i_sgd = [ref.launch_name(i) for i in range(ref.num_launches())].index("sgd_update")
        ref.profile_start(i_sgd, every=4)
        t_ref = _time_steps(ref, x, y, lr, max(args.steps, 8), torch)
        ms_r, cnt_r = ref.profile_stop()
        ref.destroy()
        sgd_ms = float(ms_r[i_sgd] / max(cnt_r[i_sgd], 1))
        bpp = 12.0 + (2.0 if w.dtype == wl.BF16 else 0.0)
        rec["separate_update"] = {"ms_per_step": t_ref * 1e3, "sgd_kernel_avg_ms": sgd_ms,
                                  "sgd_kernel_algorithmic_bytes": n_params * bpp,
                                  "sgd_kernel_frac_of_hbm_peak": n_params * bpp / (sgd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

    if args.swap_cost and extras:
        pk2 = make(w.models, w.batch, w.weights)
        pk2.step(x.data_ptr(), y.data_ptr(), lr)
        torch.cuda.synchronize()
        k = w.K - 1
        t0 = time.perf_counter()
        blob = pk2.read_weights(k)
        t1 = time.perf_counter()
        pk2.free(k)
        t2 = time.perf_counter()
        kk = pk2.load(w.models[k], w.batch[k], seed=1)
        t3 = time.perf_counter()
        pk2.write_weights(kk, blob)
        t4 = time.perf_counter()
        pk2.step(x.data_ptr(), y.data_ptr(), lr)
        assert kk == k and np.all(np.isfinite(pk2.read_loss()))
        pk2.destroy()
        rec["swap_ms"] = {"checkpoint_read": (t1 - t0) * 1e3, "free": (t2 - t1) * 1e3, "load": (t3 - t2) * 1e3,
                          "checkpoint_write": (t4 - t3) * 1e3, "member_params": int(blob.size),
                          "in_steps": (t4 - t0) / t_pack}

    if not args.no_unpacked:
        # T_s(Seq): K packs of one member each, stepped one after the other on the same stream, every
        # one reading x itself; members with the same layer list and batch take the same time, so one
        # of each kind is measured (REPEATS repeats, median) and counted as often as it occurs
        kinds = {}
        for k in range(w.K):
            kinds.setdefault((tuple(map(tuple, w.models[k])), int(w.batch[k])), []).append(k)
        t_seq = 0.0
        for members in kinds.values():
            k = members[0]
            solo = make([w.models[k]], [w.batch[k]], [w.weights[k]])
            l1 = lr[k:k + 1]
            for _ in range(max(args.warmup // 2, 2)):
                solo.step(x.data_ptr(), y.data_ptr(), l1)
            t_seq += len(members) * float(np.median([_time_steps(solo, x, y, l1, max(args.steps // 2, 5), torch)
                                                     for _ in range(REPEATS)]))
            solo.destroy()
        rec["unpacked_ms_per_step"] = t_seq * 1e3
        rec["speedup_vs_unpacked"] = t_seq / t_pack
        rec["impv"] = (t_seq - t_pack) / t_seq

    if args.two_streams and extras and w.K >= 2 and not args.different_inputs:
        # packing against concurrency on the device (Section 4.6 compares pack with running the models side
        # by side): the same members as two packs of K/2 on two streams of default priority, their steps
        # enqueued alternately and left to the hardware to overlap
        h = w.K // 2
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        pa = make(w.models[:h], w.batch[:h], w.weights[:h], sa.cuda_stream)
        pb = make(w.models[h:], w.batch[h:], w.weights[h:], sb.cuda_stream)
        torch.cuda.synchronize()

        def both(n):
            for _ in range(n):
                pa.step(x.data_ptr(), y.data_ptr(), lr[:h])
                pb.step(x.data_ptr(), y.data_ptr(), lr[h:])
        both(max(args.warmup, 2))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        both(args.steps)
        torch.cuda.synchronize()
        rec["two_half_packs_on_two_streams_ms_per_step"] = (time.perf_counter() - t0) / args.steps * 1e3
        pa.destroy()
        pb.destroy()

    del x, y
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = _cpu_baseline(w, args, np, wl, lr, cpu_budget_s)
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20, help="steps per timed repeat (5 repeats per configuration)")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="all", choices=["all", "c1", "c2", "c3", "c4", "c5"],
                    help="all (default): every configuration, headline c5; cN: that configuration alone")
    ap.add_argument("--optimizer", default="sgd", choices=["sgd", "momentum", "adagrad", "adam"],
                    help="optimiser of every member (the configurations use plain SGD)")
    ap.add_argument("--different-inputs", action="store_true",
                    help="every member trains on its own batch (the 'Training Data: Different' rows of the paper's "
                         "Table 2) instead of the shared one")
    ap.add_argument("--search", action="store_true",
                    help="instead of the step benchmark: run Hyperband (R=81, eta=3) over the paper's Table 3 space with "
                         "every grouping policy (none / kNN pack_opt / Random Pack / Batch-size Pack) on a CIFAR-shaped "
                         "synthetic dataset and print the training time of each (the paper's Table 4)")
    ap.add_argument("--search-units", type=int, default=10, help="training steps per Hyperband resource unit")
    ap.add_argument("--swap-cost", action="store_true",
                    help="also time a member leaving a live pack (checkpoint read + pack_free) and a member joining "
                         "(pack_load + checkpoint write): the switching overhead of Section 3.3, outside the timed steps")
    ap.add_argument("--two-streams", action="store_true",
                    help="also time the same members as two packs of K/2 on two streams (pack against device concurrency)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-unpacked", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip measuring what this GPU sustains on a plain copy and on a register-resident MFMA loop")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise copy of 256 MiB (reads 256 MiB, writes 256 MiB) five times, "
                         "so that a hardware-counter run has a kernel of known traffic to scale by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU (the packed step has no cross-GPU part); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as wl
    from paper_2002_02885_amd import binding

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.search:
        return _search(args, np, torch, wl)

    names = ["c1", "c2", "c3", "c4", "c5"] if args.workload == "all" else [args.workload]
    head_name = HEADLINE if args.workload == "all" else args.workload
    records = {}
    for name in names:
        print(f"bench: {name} ...", file=sys.stderr, flush=True)
        # the oracle sample: about 12 s on the headline configuration, about 3 s on each of the others
        records[name] = bench_config(name, args, np, torch, wl, binding, extras=(name == head_name),
                                     cpu_budget_s=12.0 if name == head_name else 3.0)
    head = records[head_name]
    out = {
        "metric": "packed train samples x models / s",
        "value": head["value"],
        "unit": "samples*models/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"], "K": head["K"], "batch": head["batch"],
                   "launches_per_step": head["launches_per_step"], "device_bytes": head["device_bytes"],
                   "timing": f"median of {REPEATS} repeats of {args.steps} steps after {args.warmup} warm-up steps"},
    }
    for key, val in head.items():
        if key not in ("workload", "K", "batch", "launches_per_step", "device_bytes", "value", "unit", "ms_per_step", "dtype"):
            out[key] = val
    if len(records) > 1:
        out["configs"] = records
    print(json.dumps(out))


if __name__ == "__main__":
    main()
