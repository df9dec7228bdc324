#!/usr/bin/env python3
"""Benchmark of the RAD train step on one MI355X.

A step is one rad_train_step: sampling plan + pack, forward GEMMs with fused
ReLU-bit / sample epilogues, softmax cross-entropy, dW from the compressed
stores and the exact dX chain.  Default workload: the wide bf16 MLP
(4096-4096-4096-1000, batch 4096) with per-example fixed-k sampling at p=0.1.

Prints ONE JSON line: whole-job samples/s with inputs resident in HBM, the
roofline of the dominant kernel (the GEMM variant with the largest share of
the step, found in two warm-up steps) timed with HIP events on the library's
stream inside the timed region, and the CPU oracle
timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"bf16": 2500.0, "f32": 157.3}      # dense MFMA TFLOP/s, MI355X published
# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a plain copy kernel): read
# from the `traffic_bytes <workload> <scheme> <p> <kernel label> <bytes>` lines of this counter summary
TRAFFIC_FILE = os.path.join("profiles", "train_step_mlp4096_bf16_hbm_traffic.txt")


def measured_traffic(workload, scheme, p, kernel):
    """HBM bytes per launch of `kernel` from the committed counter summary, or None if it has no line for it."""
    try:
        with open(os.path.join(ROOT, TRAFFIC_FILE)) as f:
            for ln in f:
                w = ln.split()
                if len(w) == 6 and w[0] == "traffic_bytes" and w[1:5] == [workload, scheme, "%g" % p, kernel]:
                    return float(w[5])
    except OSError:
        pass
    return None


HBM_PEAK = 8000.0                          # GB/s
TIMED_EVERY = 4                            # steps between two in which the dominant kernel is event-timed

WORKLOADS = {
    # name: (dtype, batch, dims, pixels, has_bias)
    "mlp4096_bf16": ("bf16", 4096, (4096, 4096, 4096, 1000), False, False),
    "mlp784_f32": ("f32", 150, (784, 300, 300, 10), True, True),
}
SCHEMES = {"per_example": 3, "shared": 2, "bernoulli": 1, "exact": 0,
           "replace_per_example": 5, "replace_shared": 4,      # draws with replacement
           "project": 6,                                       # Rademacher projection, one R per layer and step
           "project_per_example": 7}                           # a Rademacher matrix per example


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="mlp4096_bf16", choices=sorted(WORKLOADS) + ["pde32", "other", "pack_stream", "ceilings", "library_gemm"],
                    help="pde32: the reaction-diffusion study instead of a train step (a step = one gradient of each "
                         "of 256 problems); other: only the small configurations 1, 2, 3 and 5 (ms per train step)")
    ap.add_argument("--scheme", default="per_example", choices=sorted(SCHEMES))
    ap.add_argument("--p", type=float, default=0.1)
    ap.add_argument("--index-free", action="store_true",
                    help="stores keep values only; columns are drawn again in the backward pass")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the kernel breakdown and the pack stream")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives are built); use --gpus 1")

    import numpy as np
    import torch
    from paper_2007_10412_amd import binding as B, synth

    if args.workload == "other":
        ctx = B.rad_ctx_create()
        print(json.dumps({"metric": "ms_per_train_step", "data": "synthetic", "n_gpus": 1,
                          "other_configs": other_configs(B, ctx, torch, synth)}))
        B.rad_ctx_destroy(ctx)
        return
    if args.workload == "ceilings":        # what plain kernels reach on this device (HBM, MFMA, integer multiply)
        ctx = B.rad_ctx_create()
        print(json.dumps({"metric": "measured_ceilings", "data": "synthetic", "n_gpus": 1,
                          "ceilings": ceilings(B, ctx, torch)}))
        B.rad_ctx_destroy(ctx)
        return
    if args.workload == "library_gemm":    # the 4096^3 dX GEMM alone, next to the vendor library's GEMM of that shape
        ctx = B.rad_ctx_create()
        print(json.dumps({"metric": "gemm_4096_us", "data": "synthetic", "n_gpus": 1,
                          "library_gemm": library_gemm(B, ctx, torch)}))
        B.rad_ctx_destroy(ctx)
        return
    if args.workload == "pack_stream":     # the stand-alone sampler on a 1 GiB stream, alone
        ctx = B.rad_ctx_create()
        print(json.dumps({"metric": "sampler_stream_GBps", "data": "synthetic", "n_gpus": 1,
                          "pack_stream": pack_stream(B, ctx, torch, "f32")}))
        B.rad_ctx_destroy(ctx)
        return
    if args.workload == "pde32":
        ctx = B.rad_ctx_create()
        out = pde_study(B, ctx, torch, steps=args.steps, warmup=args.warmup, p=args.p if args.p < 1 else 0.01)
        B.rad_ctx_destroy(ctx)
        print(json.dumps(out))
        return

    dtype_name, batch, dims, pixels, has_bias = WORKLOADS[args.workload]
    dtype = B.RAD_BF16 if dtype_name == "bf16" else B.RAD_F32
    tdt = torch.bfloat16 if dtype == B.RAD_BF16 else torch.float32
    scheme = SCHEMES[args.scheme]
    p = 1.0 if scheme == 0 else args.p
    L = len(dims) - 1
    data = synth.mlp(seed=1234, batch=batch, dims=dims, pixels=pixels, bf16=(dtype == B.RAD_BF16))

    ctx = B.rad_ctx_create()
    model = B.rad_model_create_mlp(ctx, dtype, batch, list(dims), has_bias, scheme, p)
    if args.index_free:
        B.rad_model_set_index_free(ctx, model, True)
    params, grads = [], []
    for l in range(L):
        params.append(torch.from_numpy(data["Ws"][l]).cuda().to(tdt).contiguous())
        grads.append(torch.empty(data["Ws"][l].shape, device="cuda", dtype=torch.float32))
        if has_bias:
            params.append(torch.from_numpy(data["bs"][l]).cuda())
            grads.append(torch.empty(data["bs"][l].shape, device="cuda", dtype=torch.float32))
    x = torch.from_numpy(data["x"]).cuda().to(tdt).contiguous()
    labels = torch.from_numpy(data["labels"]).cuda()

    def step(i, want_loss=True):
        return B.rad_train_step(ctx, model, B.make_sampling(scheme, p, 1000 + i, 0, 0), x, labels, params, grads,
                                want_loss)

    for i in range(args.warmup):
        step(i)
    # Which kernel dominates the step: two untimed steps with every launch bracketed by events.  The timed
    # region then brackets only that kernel (events around every launch would add gaps between all of them).
    B.rad_ctx_timing(ctx, None)
    B.rad_ctx_timing_reset(ctx)
    for i in range(2):
        step(500 + i)
    labels_ms = {}
    for fam in ("fwd", "fwd_dma", "fwd_partial", "fwd_partial_dma", "dx", "dx_dma", "dw_sparse", "dw_sparse_splitk", "dw_dense", "dw_dense_dma"):
        for tile in ("64", "128", "256", "256x64", "256x128", "256x256"):
            nm = "gemm_%s_%s_%s" % (dtype_name, fam, tile)
            n, ms = B.rad_ctx_timing_read(ctx, nm)
            # a name may be a prefix of another (…_256 of …_256x64): keep exact matches only
            longer = sum(B.rad_ctx_timing_read(ctx, nm + "x" + t)[1] for t in ("64", "128", "256")) if "x" not in tile else 0.0
            if n and ms - longer > 0:
                labels_ms[nm] = ms - longer
    big = max(labels_ms, key=labels_ms.get)
    # the dW kernel of the widest layers, from the same two steps
    dw_labels = [k_ for k_ in labels_ms if "_dw_" in k_]
    dw_kernel = None
    if dw_labels:
        dwl = max(dw_labels, key=labels_ms.get)
        n_, ms_ = B.rad_ctx_timing_read(ctx, dwl)
        a_, x_ = B.rad_ctx_timing_read_flops(ctx, dwl)
        if "x" not in dwl.rsplit("_", 1)[1]:
            for t in ("64", "128", "256"):
                n2, ms2 = B.rad_ctx_timing_read(ctx, dwl + "x" + t)
                a2, x2 = B.rad_ctx_timing_read_flops(ctx, dwl + "x" + t)
                n_ -= n2; ms_ -= ms2; a_ -= a2; x_ -= x2
        if n_ and ms_ > 0:
            dw_kernel = {"kernel": dwl, "avg_launch_ms": ms_ / n_, "launches_per_step": n_ / 2,
                         "executed_tflops": x_ / (ms_ * 1e-3) / 1e12, "algorithmic_tflops": a_ / (ms_ * 1e-3) / 1e12,
                         "executed_frac_of_peak": x_ / (ms_ * 1e-3) / 1e12 / PEAK[dtype_name],
                         "note": "executed = 2 B D N on zero-filled tiles (MFMA utilisation); algorithmic = 2 N per kept entry"}
    B.rad_ctx_timing(ctx, "")
    B.rad_ctx_timing_reset(ctx)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # the steps are enqueued back to back, as a training loop would; only the last one reads its loss back.
    # The dominant kernel carries timing events in every fourth step of the timed region: an event-carrying
    # launch costs about 6 us of stream time, which timing all of them would put into every step.
    loss = 0.0
    for i in range(args.steps):
        B.rad_ctx_timing(ctx, big if i % TIMED_EVERY == 0 else "")
        loss = step(args.warmup + i, want_loss=(i == args.steps - 1))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    ms_per_step = 1e3 * elapsed / args.steps
    value = batch * args.steps / elapsed

    # roofline of that kernel from the events of the timed region; flops as the library counted them per launch
    n_all, ms_all = B.rad_ctx_timing_read(ctx, big)
    alg_all, exe_all = B.rad_ctx_timing_read_flops(ctx, big)
    n_long = ms_long = alg_long = exe_long = 0
    if "x" not in big.rsplit("_", 1)[1]:
        for t in ("64", "128", "256"):
            n_, ms_ = B.rad_ctx_timing_read(ctx, big + "x" + t)
            a_, x_ = B.rad_ctx_timing_read_flops(ctx, big + "x" + t)
            n_long += n_; ms_long += ms_; alg_long += a_; exe_long += x_
    n_launch, tot_ms = n_all - n_long, ms_all - ms_long
    alg_flops, exe_flops = (alg_all - alg_long) / max(1, n_launch), (exe_all - exe_long) / max(1, n_launch)
    B.rad_ctx_timing(ctx, "")
    per_step = n_launch / max(1, (args.steps + TIMED_EVERY - 1) // TIMED_EVERY)
    avg_ms = tot_ms / max(1, n_launch)
    peak = PEAK[dtype_name]
    roofline = {
        "kernel": big, "bound": "mfma", "unit": "TFLOP/s",
        "achieved": alg_flops / (avg_ms * 1e-3) / 1e12 if avg_ms > 0 else None,
        "peak": peak,
        "frac": alg_flops / (avg_ms * 1e-3) / 1e12 / peak if avg_ms > 0 else None,
        "executed": exe_flops / (avg_ms * 1e-3) / 1e12 if avg_ms > 0 else None,
        "executed_frac": exe_flops / (avg_ms * 1e-3) / 1e12 / peak if avg_ms > 0 else None,
        "avg_launch_ms": avg_ms, "launches": n_launch, "launches_per_step": per_step, "timed_every_steps": TIMED_EVERY,
        "share_of_step": avg_ms * per_step / ms_per_step if ms_per_step > 0 else None,
        "algorithmic_flops_per_launch": alg_flops, "executed_flops_per_launch": exe_flops,
        "traffic": measured_traffic(args.workload, args.scheme, p, big), "traffic_source": TRAFFIC_FILE,
        "step_share_by_kernel_ms": {k_: v_ / 2 for k_, v_ in sorted(labels_ms.items())},
    }

    out = {
        "metric": "rad_train_step_samples_per_sec", "value": value, "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype_name, "data": "synthetic",
        "config": {"workload": "%s: MLP %s, batch %d, %s sampling p=%g, softmax-CE, full fwd+bwd train step"
                   % (args.workload, "-".join(str(d) for d in dims), batch, args.scheme, p),
                   "batch": batch, "dims": list(dims), "scheme": args.scheme, "p": p,
                   "index_free": bool(args.index_free)},
        "loss": loss,
        "roofline": roofline,
        "dw_kernel": dw_kernel,
    }

    # stored activation bytes (values / indices+tables / ReLU bits) vs the dense baseline
    sb = {"value_bytes": 0, "index_bytes": 0, "bit_bytes": 0, "dense_bytes": 0}
    for l in range(L):
        st = B.rad_store_get_stats(ctx, B.rad_model_store(model, l))
        for k_ in sb:
            sb[k_] += st[k_]
    sb["stored_total"] = sb["value_bytes"] + sb["index_bytes"] + sb["bit_bytes"]
    sb["paper_convention"] = sb["value_bytes"] + sb["bit_bytes"]
    out["stored_activation_bytes"] = sb

    if not args.no_extras:
        # per-kernel breakdown of one step (separate pass: every launch bracketed by events)
        B.rad_ctx_timing(ctx, None)
        B.rad_ctx_timing_reset(ctx)
        reps = 3
        for i in range(reps):
            step(10_000 + i)
        kern = {}
        names = ["plan", "row_scan", "pack", "reindex", "sign_matrix", "scale_cast", "unpack", "project_rows_fwd",
                 "project_rows_bwd", "fwd", "dx", "dw_sparse", "dw_dense", "dw_overflow", "splitk_fwd", "splitk_bias",
                 "splitk_reduce", "softmax_ce", "colsum", "fill"]
        # labels are matched as substrings: the GEMM families by "_fwd_" / "_dx_", which the finishing and projection
        # kernels (…_fwd at the end of their names) do not contain
        pattern = {"fwd": "_fwd_", "dx": "_dx_"}
        for nm in names:
            n, ms = B.rad_ctx_timing_read(ctx, pattern.get(nm, nm))
            if n:
                kern[nm] = {"launches_per_step": n / reps, "ms_per_step": ms / reps}
        if "pack" in kern and "unpack" in kern:        # "pack" also matched the unpack launches
            kern["pack"] = {k_: kern["pack"][k_] - kern["unpack"][k_] for k_ in kern["pack"]}
            if kern["pack"]["launches_per_step"] <= 0:
                del kern["pack"]
        B.rad_ctx_timing(ctx, "")
        B.rad_ctx_timing_reset(ctx)
        fl = {"fwd": sum(2.0 * batch * dims[l] * dims[l + 1] for l in range(L)),
              "dx": sum(2.0 * batch * dims[l] * dims[l + 1] for l in range(1, L)),
              "dw_sparse": sum(2.0 * batch * dims[l] * dims[l + 1] for l in range(L) if dims[l + 1] % 256 or "dw_dense" not in kern),
              "dw_dense": sum(2.0 * batch * dims[l] * dims[l + 1] for l in range(L) if dims[l + 1] % 256 == 0)}
        for nm, f in fl.items():
            if nm in kern and kern[nm]["ms_per_step"] > 0:
                kern[nm]["executed_tflops"] = f / (kern[nm]["ms_per_step"] * 1e-3) / 1e12
        out["kernels"] = kern
        # the published peaks are what every `frac` above is against; beside them, what plain kernels reach on
        # this very device, and the same fractions against those
        ceil = ceilings(B, ctx, torch)
        out["ceilings"] = ceil
        if dtype_name == "bf16":
            out["library_gemm"] = library_gemm(B, ctx, torch)
        mf = ceil["mfma_bf16_32x32x16_random_TFLOPs"] if dtype_name == "bf16" else ceil["mfma_f32_32x32x2_random_TFLOPs"]
        if roofline["executed"]:
            roofline["frac_of_measured_mfma_loop"] = roofline["executed"] / mf
        if dw_kernel:
            dw_kernel["executed_frac_of_measured_mfma_loop"] = dw_kernel["executed_tflops"] / mf
        out["pack_stream"] = pack_stream(B, ctx, torch, dtype_name)
        for rule in ("bernoulli", "fixed_k_per_example"):
            ps = out["pack_stream"][rule]
            ps["pack"]["frac_of_measured_read"] = ps["pack"]["achieved"] / ceil["hbm_read_GBps"]
            ps["whole"]["frac_of_measured_read"] = ps["whole"]["achieved"] / ceil["hbm_read_GBps"]
            ps["plan"]["philox_mad_share_of_measured_int_rate"] = ps["plan"]["keys_per_s"] * 5 / (ceil["int_mad64_Tops"] * 1e12)
        out["optimizer"] = optimizer_stream(B, ctx, torch, dtype, params, grads)
        out["pde"] = pde_study(B, ctx, torch, steps=2, warmup=1, p=0.01)
        out["other_configs"] = other_configs(B, ctx, torch, synth)
        if args.workload == "mlp4096_bf16":
            out["config4_variants"] = config4_variants(B, ctx, torch, data, dims, batch)

    B.rad_model_destroy(model)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(data, dims, scheme, p, dtype, batch, has_bias)

    B.rad_ctx_destroy(ctx)
    print(json.dumps(out))


def config4_variants(B, ctx, torch, data, dims, batch):
    """ms/step of the wide bf16 MLP at the other fractions and sampling schemes (steps enqueued back to back)."""
    res = {}
    params = [torch.from_numpy(w).cuda().to(torch.bfloat16).contiguous() for w in data["Ws"]]
    grads = [torch.empty(w.shape, device="cuda", dtype=torch.float32) for w in data["Ws"]]
    x = torch.from_numpy(data["x"]).cuda().to(torch.bfloat16).contiguous()
    labels = torch.from_numpy(data["labels"]).cuda()
    for name, scheme in (("per_example", 3), ("shared", 2), ("replace_per_example", 5), ("replace_shared", 4),
                         ("project", 6), ("per_example_index_free", 3)):
        for p in ((0.5, 0.1, 0.02) if name in ("per_example", "shared") else
                  (0.5, 0.1) if name.endswith("index_free") else (0.1,)):
            model = B.rad_model_create_mlp(ctx, B.RAD_BF16, batch, list(dims), False, scheme, p)
            if name.endswith("index_free"):
                B.rad_model_set_index_free(ctx, model, True)
            for i in range(3):
                B.rad_train_step(ctx, model, B.make_sampling(scheme, p, 50 + i, 0, 0), x, labels, params, grads, False)
            torch.cuda.synchronize()
            steps = 10
            t0 = time.perf_counter()
            for i in range(steps):
                B.rad_train_step(ctx, model, B.make_sampling(scheme, p, 60 + i, 0, 0), x, labels, params, grads, False)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / steps
            stored = 0
            for l in range(len(dims) - 1):
                st_ = B.rad_store_get_stats(ctx, B.rad_model_store(model, l))
                stored += st_["value_bytes"] + st_["index_bytes"] + st_["bit_bytes"]
            res["%s_p%g" % (name, p)] = {"ms_per_step": 1e3 * dt, "samples_per_s": batch / dt,
                                         "stored_activation_bytes": stored}
            B.rad_model_destroy(model)
    return res


def other_configs(B, ctx, torch, synth):
    """samples/s of the train step on the remaining configurations (small, latency bound), a few steps each."""
    import numpy as np
    res = {}

    def timed(fn, steps, batch):
        fn(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fn(1 + i)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        return {"ms_per_step": 1e3 * dt, "samples_per_s": batch / dt}

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    # config 1: single layer 784 -> 300, batch 150, Bernoulli p = 0.1: forward+sample, dW, dX
    d = synth.single_layer()
    L = B.make_layer(150, 784, 300)
    st = B.rad_store_create(ctx, L, B.RAD_BERNOULLI, 0.1)
    x, W, dy = dev(d["x"]), dev(d["W"]), dev(d["dy"])
    y = torch.empty(150, 300, device="cuda"); dW = torch.empty(784, 300, device="cuda"); dX = torch.empty(150, 784, device="cuda")

    def c1(i):
        B.rad_forward_sample(ctx, L, B.make_sampling(B.RAD_BERNOULLI, 0.1, i), x, W, None, y, st)
        B.rad_backward_dW(ctx, L, st, dy, dW, None, 0.0)
        B.rad_backward_dX(ctx, L, st, dy, W, dX)
        B.rad_ctx_synchronize(ctx)
    res["config1_layer_784x300_f32_bernoulli"] = timed(c1, 50, 150)
    B.rad_store_destroy(st)

    # config 2: MLP 784-300-300-10, batch 150, per-example fixed-k
    dims = (784, 300, 300, 10)
    d = synth.mlp(seed=1234, batch=150, dims=dims)
    m = B.rad_model_create_mlp(ctx, B.RAD_F32, 150, list(dims), True, B.RAD_FIXEDK_PER_EXAMPLE, 0.1)
    params, grads = [], []
    for Wl, bl in zip(d["Ws"], d["bs"]):
        params += [dev(Wl), dev(bl)]; grads += [torch.empty(Wl.shape, device="cuda"), torch.empty(bl.shape, device="cuda")]
    x, lab = dev(d["x"]), dev(d["labels"])
    res["config2_mlp_784_300_300_10_f32_per_example"] = timed(
        lambda i: B.rad_train_step(ctx, m, B.make_sampling(B.RAD_FIXEDK_PER_EXAMPLE, 0.1, i), x, lab, params, grads), 50, 150)
    B.rad_model_destroy(m)

    # config 3: CNN 3-16-32-64 @32x32, batch 150, Bernoulli
    ch, pool = (3, 16, 32, 64), (0, 1, 1)
    d = synth.cnn(seed=1234, batch=150, channels=ch, pool=pool)
    m = B.rad_model_create_cnn(ctx, 150, list(ch), list(pool), 3, 32, 32, 10, B.RAD_BERNOULLI, 0.1)
    params, grads = [], []
    for cv in d["convs"]:
        params += [dev(cv["W"]), dev(cv["b"])]; grads += [torch.empty(cv["W"].shape, device="cuda"), torch.empty(cv["b"].shape, device="cuda")]
    params += [dev(d["fc"][0]), dev(d["fc"][1])]; grads += [torch.empty(d["fc"][0].shape, device="cuda"), torch.empty(10, device="cuda")]
    x, lab = dev(d["x"]), dev(d["labels"])
    res["config3_cnn_f32_bernoulli"] = timed(
        lambda i: B.rad_train_step(ctx, m, B.make_sampling(B.RAD_BERNOULLI, 0.1, i), x, lab, params, grads), 10, 150)
    B.rad_model_destroy(m)

    # config 5: ReLU RNN hidden 1024, T 784, batch 128, Bernoulli per step
    d = synth.rnn(seed=1234)
    m = B.rad_model_create_rnn(ctx, 128, 784, 1, 1024, 10, B.RAD_BERNOULLI, 0.1)
    names = ["W_ih", "W_hh", "b", "W_ho", "b_o"]
    params = [dev(d[n]) for n in names]; grads = [torch.empty(d[n].shape, device="cuda") for n in names]
    x, lab = dev(d["x"]), dev(d["labels"])
    res["config5_rnn_h1024_T784_f32_bernoulli"] = timed(
        lambda i: B.rad_train_step(ctx, m, B.make_sampling(B.RAD_BERNOULLI, 0.1, i), x, lab, params, grads), 3, 128)
    B.rad_model_destroy(m)
    return res


def ceilings(B, ctx, torch):
    """Measured ceilings of this device (rad_probe_ceiling): HBM streaming read and copy of 1 GiB, register-resident
    loops of the matrix instructions on random and on zero operands, independent integer multiply-adds."""
    n = 1 << 28                                        # 1 GiB of fp32
    gen = torch.Generator(device="cuda").manual_seed(3)
    a = torch.randn(n, device="cuda", dtype=torch.float32, generator=gen)
    b = torch.empty(n, device="cuda", dtype=torch.float32)
    ab = a[: 1 << 23].to(torch.bfloat16).contiguous()  # 16 MiB of random bf16 operands
    zeros = torch.zeros(1 << 23, device="cuda", dtype=torch.bfloat16)
    res = {"hbm_read_GBps": B.rad_probe_ceiling(ctx, 0, a, b, n * 4, 10) / 1e9,
           "hbm_copy_GBps": B.rad_probe_ceiling(ctx, 1, a, b, n * 4, 10) / 1e9}
    for name, kind in (("mfma_bf16_32x32x16", 2), ("mfma_bf16_16x16x32", 3)):
        # alternate random and zero operands a few times: the clock follows the power drawn, with some lag
        r, z = [], []
        for _ in range(3):
            r.append(B.rad_probe_ceiling(ctx, kind, ab, b, ab.numel() * 2, 100))
            z.append(B.rad_probe_ceiling(ctx, kind, zeros, b, zeros.numel() * 2, 100))
        res[name + "_random_TFLOPs"] = sum(r) / len(r) / 1e12
        res[name + "_zeros_TFLOPs"] = sum(z) / len(z) / 1e12
    res["mfma_f32_32x32x2_random_TFLOPs"] = B.rad_probe_ceiling(ctx, 4, a, b, 1 << 24, 100) / 1e12
    res["int_mad64_Tops"] = B.rad_probe_ceiling(ctx, 5, a, b, 1 << 25, 100) / 1e12
    res["published"] = {"hbm_GBps": HBM_PEAK, "mfma_bf16_TFLOPs": PEAK["bf16"], "mfma_f32_TFLOPs": PEAK["f32"]}
    return res


def library_gemm(B, ctx, torch):
    """Context for the GEMM kernels, not a target: rad_backward_dX on a 4096 x 4096 x 4096 bf16 layer (no ReLU mask)
    called alone in a loop, next to the vendor library's GEMM of the same shape and layout (torch.matmul), each on
    the same buffers every call ("warm": operands stay in the last-level cache) and on ten rotating sets ("cold":
    every call reads its operands from HBM, as a kernel inside a train step does)."""
    n, sets = 4096, []
    gen = torch.Generator(device="cuda").manual_seed(5)
    for _ in range(10):
        dy = torch.randn(n, n, device="cuda", generator=gen).to(torch.bfloat16)
        W = (torch.randn(n, n, device="cuda", generator=gen) / 64.0).to(torch.bfloat16)
        sets.append((dy, W, torch.empty(n, n, device="cuda", dtype=torch.bfloat16)))
    L = B.make_layer(n, n, n, dtype=B.RAD_BF16, relu=False)
    st = B.rad_store_create(ctx, L, B.RAD_FIXEDK_PER_EXAMPLE, 0.1)

    def us_per_call(f, reps=1000):
        for i in range(20):
            f(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            f(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    res = {"shape": "dX[4096,4096] = dy[4096,4096] W[4096,4096]^T, bf16 in, fp32 accumulate, bf16 out",
           "rad_backward_dX_warm_us": us_per_call(lambda i: B.rad_backward_dX(ctx, L, st, *sets[0])),
           "rad_backward_dX_cold_us": us_per_call(lambda i: B.rad_backward_dX(ctx, L, st, *sets[i % 10])),
           "library_warm_us": us_per_call(lambda i: torch.matmul(sets[0][0], sets[0][1].t(), out=sets[0][2])),
           "library_cold_us": us_per_call(lambda i: torch.matmul(sets[i % 10][0], sets[i % 10][1].t(),
                                                                 out=sets[i % 10][2]))}
    B.rad_store_destroy(st)
    flop = 2.0 * n ** 3
    for k in list(res):
        if k.endswith("_us"):
            res[k.replace("_us", "_TFLOPs")] = flop / res[k] / 1e6
    return res


def pack_stream(B, ctx, torch, dtype_name):
    """The stand-alone sampler (key generation, selection, scale + pack: rad_sample_pack) on a 1 GiB stream of
    4096-wide fp32 rows, fraction 0.1, under the Bernoulli and the per-example fixed-k rule.  Two kernels: the plan
    kernel reads nothing and is bound by the integer arithmetic of the Philox keys (plus the k-select for fixed-k)
    and writes a keep bitmap; the pack kernel is an HBM stream (x and the bitmap in, values and indices out).
    `whole` is both kernels (and the row scan) against the algorithmic bytes: read 4 B per element, write 6 B per
    kept entry."""
    rows, cols, p = 65536, 4096, 0.1
    n = rows * cols
    x = torch.randn(rows, cols, device="cuda", dtype=torch.float32)
    res = {"rows": rows, "cols": cols, "p": p, "dtype": "f32"}
    reps = 5
    for name, scheme in (("bernoulli", B.RAD_BERNOULLI), ("fixed_k_per_example", B.RAD_FIXEDK_PER_EXAMPLE)):
        L = B.make_layer(rows, cols, 8, dtype=B.RAD_F32, relu=False)
        st = B.rad_store_create(ctx, L, scheme, p)
        B.rad_ctx_timing(ctx, None)
        for i in range(2):
            B.rad_sample_pack(ctx, B.make_sampling(scheme, p, i), x, st)
        B.rad_ctx_timing_reset(ctx)
        for i in range(reps):
            B.rad_sample_pack(ctx, B.make_sampling(scheme, p, 10 + i), x, st)
        n_plan, ms_plan = B.rad_ctx_timing_read(ctx, "plan")
        n_pack, ms_pack = B.rad_ctx_timing_read(ctx, "pack_f32")
        n_scan, ms_scan = B.rad_ctx_timing_read(ctx, "row_scan")
        B.rad_ctx_timing(ctx, "")
        B.rad_ctx_timing_reset(ctx)
        nnz = B.rad_store_get_stats(ctx, st)["nnz"]
        B.rad_store_destroy(st)
        t_plan, t_pack, t_scan = ms_plan / n_plan * 1e-3, ms_pack / n_pack * 1e-3, (ms_scan / n_scan * 1e-3 if n_scan else 0.0)
        alg = n * 4 + nnz * 6                         # read s per element, write (s + 2) per kept entry
        pack_bytes = alg + n / 8                      # the pack kernel also reads the keep bitmap
        t_whole = t_plan + t_pack + t_scan
        res[name] = {
            "whole": {"bound": "hbm", "ms": t_whole * 1e3, "achieved": alg / t_whole / 1e9, "peak": HBM_PEAK,
                      "unit": "GB/s", "frac": alg / t_whole / 1e9 / HBM_PEAK, "keys_per_s": n / t_whole},
            "plan": {"bound": "alu", "ms": t_plan * 1e3, "keys_per_s": n / t_plan, "write_GBps": n / 8 / t_plan / 1e9},
            "row_scan_ms": t_scan * 1e3,
            "pack": {"bound": "hbm", "ms": t_pack * 1e3, "achieved": pack_bytes / t_pack / 1e9, "peak": HBM_PEAK,
                     "unit": "GB/s", "frac": pack_bytes / t_pack / 1e9 / HBM_PEAK,
                     "frac_algorithmic_bytes": alg / t_pack / 1e9 / HBM_PEAK}}
    return res


def pde_study(B, ctx, torch, steps, warmup, p, problems=256):
    """The reaction-diffusion study at the paper's size (32 x 32 intervals, 40960 time steps, fraction p of every
    state kept): one call = loss and sampled gradient of `problems` control vectors, one workgroup (CU) each.
    The time steps of a problem depend on each other, so the kernels are bound by the latency of one step
    (instruction issue of the workgroup's 16 waves plus a barrier), not by a memory or arithmetic roofline:
    what is reported is the time per step of the chain."""
    grid = B.make_pde_grid(32, 40960)
    ws = torch.empty(B.rad_pde_workspace_bytes(ctx, grid, p, problems), dtype=torch.uint8, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(7)
    theta = torch.rand(problems, 7, dtype=torch.float64, device="cuda", generator=gen) * 2 - 1
    loss = torch.empty(problems, dtype=torch.float64, device="cuda")
    grad = torch.empty(problems, 7, dtype=torch.float64, device="cuda")
    stored = torch.empty(problems, dtype=torch.int64, device="cuda")
    for i in range(warmup):
        B.rad_pde_gradient(ctx, grid, theta, p, i, 0, ws, loss, grad, stored)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        B.rad_pde_gradient(ctx, grid, theta, p, 100 + i, 0, ws, loss, grad, stored)   # synchronises
    dt = (time.perf_counter() - t0) / max(steps, 1)
    kept = float(stored.double().mean())
    return {"metric": "pde_gradients_per_sec", "value": problems / dt, "unit": "gradients/s", "n_gpus": 1,
            "steps": steps, "warmup": warmup, "ms_per_step": dt * 1e3, "higher_is_better": True, "dtype": "f64",
            "data": "synthetic", "config": {"workload": "reaction-diffusion 32x32, 40960 time steps, p=%g" % p,
                                            "problems": problems},
            "us_per_time_step_and_pass": dt / (2 * 40960) * 1e6,
            "stored_fraction": kept / (40961 * 961), "stored_bytes_per_problem": kept * 8,
            "dense_bytes_per_problem": 40961 * 961 * 8}


def optimizer_stream(B, ctx, torch, dtype, params, grads):
    """One Adam step over the workload's parameters after the step's gradients (outside the timed step: the
    metric is the forward + backward step).  An HBM stream: per parameter 16 bytes read (fp32 master or
    parameter, gradient, two moments), 12 written, and 2 more for the bf16 copy."""
    bf16 = dtype == B.RAD_BF16
    master = [p_.to(torch.float32) for p_ in params] if bf16 else None
    m = [torch.zeros_like(g) for g in grads]
    v = [torch.zeros_like(g) for g in grads]
    opt = B.make_optimizer(B.RAD_ADAM, 1e-4, 1e-5)
    keep = [p_.clone() for p_ in params]
    B.rad_ctx_timing(ctx, None)
    for t in (1, 2):
        B.rad_optimizer_step(ctx, opt, t, dtype, params, grads, m, v, master)
    B.rad_ctx_timing_reset(ctx)
    reps = 10
    for t in range(3, 3 + reps):
        B.rad_optimizer_step(ctx, opt, t, dtype, params, grads, m, v, master)
    n_l, ms = B.rad_ctx_timing_read(ctx, "optim_adam")
    B.rad_ctx_timing(ctx, "")
    B.rad_ctx_timing_reset(ctx)
    for p_, k_ in zip(params, keep):      # the parameters the rest of the run uses stay as they were
        p_.copy_(k_)
    n = sum(int(p_.numel()) for p_ in params)
    bytes_ = n * (30 if bf16 else 28)
    t_step = ms / reps * 1e-3
    return {"kind": "adam", "parameters": n, "ms_per_step": t_step * 1e3, "bound": "hbm",
            "achieved": bytes_ / t_step / 1e9, "peak": HBM_PEAK, "unit": "GB/s", "frac": bytes_ / t_step / 1e9 / HBM_PEAK}


def cpu_baseline(data, dims, scheme, p, dtype, batch, has_bias):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    import numpy as np
    from oracle import rad_oracle as R
    rows = batch
    reps = 2
    bs = data["bs"] if has_bias else None
    t0 = time.perf_counter()
    for _ in range(reps):
        R.mlp_train_step(data["x"][:rows], data["labels"][:rows], data["Ws"], bs, scheme, p, seed=1,
                         dtype=(R.BF16 if dtype == 1 else R.F32))
    dt = (time.perf_counter() - t0) / reps
    cores = os.cpu_count()
    try:
        from threadpoolctl import threadpool_info
        th = [i.get("num_threads") for i in threadpool_info() if i.get("user_api") == "blas"]
        if th:
            cores = max(th)
    except Exception:
        pass
    return {"value": rows / dt, "unit": "samples/s", "cores": cores, "kind": "oracle",
            "seconds": dt * reps,
            "sample": "%d oracle train steps (numpy fp64) on all %d rows of the batch, full layer widths" % (reps, rows)}


if __name__ == "__main__":
    main()
