"""Benchmark of the policy-worker step (paper, Sec. 3.1) on one MI355X.

One "step" = one sf_policy_step over a batch of synthetic observations already
resident in HBM (the standard configuration: B=1024 frames of 3x72x128 bytes,
conv encoder, FC-512, GRU-512, one 7-way head + value, fp32).  Prints one JSON
line: env-frames/s, the roofline of the dominant kernel (live HIP-event timing of
every launch) and the CPU oracle timed on the host cores on a bounded sample.
"""
import argparse
import json
import sys
import time

import numpy as np

MI355X_PEAK_TFLOPS = {"fp32": 157.3, "bf16": 2500.0}

# HBM bytes per launch of the standard workload (B=1024), from the two rocprofv3 --pmc runs
# recorded in profiles/policy_step_standard_hbm_traffic.md: (FETCH_SIZE x 2.000 + WRITE_SIZE
# x 1.000) KiB, the factors being what the same counters read for a 256 MiB plain copy.
MEASURED_HBM_KIB = {"standard": {"conv1": 30902 + 67456, "conv2": 76932 + 25088, "conv3": 25710 + 9216,
                                 "fc": 46216 + 2048, "gru": 54646 + 2048, "heads": 2293 + 24},
                    # profiles/policy_step_bf16_kernel_trace_and_hbm_traffic.md (FETCH_SIZE x 2 + WRITE_SIZE)
                    "standard_bf16": {"conv1": 2 * 56104 + 134920, "conv2": 2 * 67967 + 50252,
                                      "conv3": 2 * 25731 + 18432, "fc": 2 * 18550 + 4096,
                                      "gru": 2 * 18638 + 8426, "heads": 2 * 4219 + 96},
                    # profiles/policy_step_resnet_counters.md (FETCH_SIZE x 2 + WRITE_SIZE)
                    "resnet_bf16": {"stage1.conv_pool": 2 * 110600 + 589820, "stage1.block1": 2 * 295000 + 589820,
                                    "stage1.block2": 2 * 295000 + 589820, "stage2.conv_pool": 2 * 295100 + 294900,
                                    "stage2.block1": 2 * 147800 + 294900, "stage2.block2": 2 * 147800 + 294900}}


def measure_pipeline(torch, binding, wl, pol, net, rounds):
    """Host-resident observations: env-frames/s of submit/wait through the pipeline with one
    slot (copy, step, copy back, in sequence) and with two slots in alternation."""
    B, dev = net["B"], pol.device
    n_env = 2 * B
    table = torch.zeros((n_env, wl.state_dim(net)), dtype=torch.float32, device=dev)
    meas = wl.measurements(net)
    obs, done = torch.from_numpy(wl.observations(net)), torch.from_numpy(wl.done_mask(net))
    res = {}
    for n_slots in (1, 2):
        pipe = binding.Pipeline(pol, B, n_slots)
        hbs = [pipe.host_buffers() for _ in range(n_slots)]
        for s, hb in enumerate(hbs):
            hb["obs"].copy_(obs)
            hb["done"].copy_(done)
            if meas is not None:
                hb["meas"].copy_(torch.from_numpy(meas))
            hb["env_ids"].copy_(torch.arange(s * B, (s + 1) * B, dtype=torch.int32))
        t = 0

        def go(n):
            nonlocal t
            for _ in range(n):
                for s in range(n_slots):
                    pipe.wait(s)
                    pipe.submit(s, hbs[s], table, wl.PHILOX_SEED, t)
                t += 1
            for s in range(n_slots):
                pipe.wait(s)

        go(max(3, rounds // 10))
        tic = time.perf_counter()
        go(rounds)
        dt = time.perf_counter() - tic
        res[n_slots] = B * n_slots * rounds / dt
        pipe.close()
    obs_bytes = int(np.prod(net["obs"]))
    return {"slot_batch": B, "rounds": rounds, "one_slot_fps": round(res[1], 1), "two_slot_fps": round(res[2], 1),
            "two_slot_h2d_GBps": round(res[2] * obs_bytes / 1e9, 2),
            "note": "host-to-device copy of the observations included; never the headline value"}


def measure_loss(torch, binding, wl, reps):
    """Learner-side loss kernels on the paper's batch (T=32, 2048 samples) and on a 32x larger one."""
    res = {}
    for name, hp in (("paper_batch_T32_N64", wl.loss_config((7,), 32, 64)),
                     ("T32_N2048", wl.loss_config((7,), 32, 2048)),
                     ("full_heads_T32_N2048", wl.loss_config((3, 3, 2, 2, 2, 8, 21), 32, 2048))):
        tr = {k: torch.from_numpy(v).cuda() for k, v in wl.trajectories(hp).items()}
        out = binding.appo_loss(hp, tr)
        for _ in range(5):
            binding.appo_loss(hp, tr, out=out)
        torch.cuda.synchronize()
        tic = time.perf_counter()
        for _ in range(reps):
            binding.appo_loss(hp, tr, out=out)
        torch.cuda.synchronize()
        us = 1e6 * (time.perf_counter() - tic) / reps
        M, sumA, nh = hp["T"] * hp["N"], sum(hp["heads"]), len(hp["heads"])
        # logits and actions are read for the forward pass and again for the gradient; the rest once
        nbytes = M * (2 * (4 * sumA + 4 * nh) + 4 * 4 + 1 + 4 * 4 + 4 * sumA)
        res[name] = {"us_per_call": round(us, 2), "samples_per_s": round(M / us * 1e6, 1),
                     "algorithmic_GBps": round(nbytes / us / 1e3, 2)}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="workload index (1 = the headline one)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (experiments)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pipeline", action="store_true",
                    help="also measure the double-buffered pipeline with host-resident observations")
    ap.add_argument("--loss", action="store_true", help="also time the learner-side loss kernels")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (the step is data-parallel over rows "
                 "with no exchange between GPUs); run with --gpus 1")

    import torch
    from paper_2006_11751_amd import binding, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    net = wl.network(args.config, **({"B": args.batch} if args.batch > 0 else {}))
    B = net["B"]
    w = wl.weights(net)
    pol = binding.Policy(net, w)
    dev = pol.device
    obs = torch.from_numpy(wl.observations(net)).to(dev)
    done = torch.from_numpy(wl.done_mask(net)).to(dev)
    h = [torch.from_numpy(wl.initial_state(net)).to(dev), torch.empty((B, wl.state_dim(net)), device=dev)]
    meas = wl.measurements(net)
    meas = None if meas is None else torch.from_numpy(meas).to(dev)
    out = [pol.alloc_outputs(B, logits=False) for _ in range(2)]
    out[0]["h_out"], out[1]["h_out"] = h[1], h[0]
    stream = torch.cuda.current_stream(dev)

    def run(n, t0):
        for t in range(t0, t0 + n):
            pol.step(obs, h[t & 1], done, wl.PHILOX_SEED, t, out=out[t & 1], stream=stream, meas=meas)

    if args.calibrate_copy:
        n = 256 << 20
        src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 256)
        dst = torch.empty(n, dtype=torch.uint8, device=dev)
        for _ in range(3):
            binding.sf_copy_bytes(src.data_ptr(), dst.data_ptr(), n, stream.cuda_stream)
        torch.cuda.synchronize()
        assert torch.equal(src, dst)
        del src, dst

    run(args.warmup, 0)
    torch.cuda.synchronize()
    tic = time.perf_counter()
    run(args.steps, args.warmup)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - tic
    ms_per_step = 1e3 * elapsed / args.steps
    fps = B * args.steps / elapsed

    # per-launch durations: the same steps again with a HIP event after every launch
    ops = pol.ops()
    pol.set_op_timing(True)
    acc = np.zeros(len(ops))
    n_timed = min(args.steps, 100)
    for t in range(n_timed):
        run(1, args.warmup + args.steps + t)
        acc += np.array(pol.last_op_times_ms())
    pol.set_op_timing(False)
    op_ms = acc / n_timed
    dtype = net["dtype"]
    peak = MI355X_PEAK_TFLOPS[dtype]
    i_dom = int(np.argmax(op_ms))
    per_op = {name: {"ms": round(float(ms), 5),
                     "tflops": round(fl * B / (ms * 1e-3) / 1e12, 3) if ms > 0 else None}
              for (name, fl), ms in zip(ops, op_ms)}
    dom_tflops = ops[i_dom][1] * B / (op_ms[i_dom] * 1e-3) / 1e12
    whole_tflops = pol.flops_per_row() * B / (ms_per_step * 1e-3) / 1e12
    kib = MEASURED_HBM_KIB.get(net["name"], {}).get(ops[i_dom][0]) if B == wl.CONFIGS[args.config]["B"] else None
    kib_all = MEASURED_HBM_KIB.get(net["name"]) if B == wl.CONFIGS[args.config]["B"] else None
    whole = {"achieved": round(whole_tflops, 3), "frac": round(whole_tflops / peak, 5)}
    if kib_all and set(kib_all) >= {name for name, _ in ops}:
        # second roof: measured HBM bytes of all launches of the step over the step's time
        hbm = sum(kib_all[name] for name, _ in ops) * 1024 / (ms_per_step * 1e-3) / 1e9
        whole.update({"hbm_GBps": round(hbm, 1), "hbm_frac": round(hbm / 8000.0, 4)})
    roofline = {"bound": "mfma", "kernel": ops[i_dom][0], "achieved": round(dom_tflops, 3), "peak": peak,
                "unit": "TFLOP/s", "frac": round(dom_tflops / peak, 5),
                "traffic": kib * 1024 if kib is not None else None,
                "avg_launch_ms": round(float(op_ms[i_dom]), 5),
                "whole_step": whole,
                "per_kernel": per_op}
    if kib is not None and op_ms[i_dom] > 0:
        # the dominant launch against the other roof; it is reported against the one it is nearer to
        gbps = kib * 1024 / (float(op_ms[i_dom]) * 1e-3) / 1e9
        if gbps / 8000.0 > roofline["frac"]:
            roofline.update({"bound": "hbm", "achieved": round(gbps, 1), "peak": 8000.0, "unit": "GB/s",
                             "frac": round(gbps / 8000.0, 5), "mfma_frac": round(dom_tflops / peak, 5)})
        else:
            roofline["hbm_frac"] = round(gbps / 8000.0, 5)

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ref
        n_rows = min(B, 1024)
        o_obs, o_h, o_done = wl.observations(net, B=n_rows), wl.initial_state(net, B=n_rows), wl.done_mask(net, B=n_rows)
        reps, spent = 0, 0.0
        while spent < 10.0 and reps < 50:
            tic = time.perf_counter()
            ref.policy_step(net, w, o_obs, o_h, o_done, wl.PHILOX_SEED, reps, want_logits=False, want_margin=False,
                            meas=wl.measurements(net, B=n_rows))
            spent += time.perf_counter() - tic
            reps += 1
        cpu = {"value": round(n_rows * reps / spent, 2), "unit": "env-frames/s", "cores": ref.num_threads(),
               "kind": "oracle", "sample": "%d rows of the same workload x %d repeats (%.1f s)" % (n_rows, reps, spent)}

    pipeline = measure_pipeline(torch, binding, wl, pol, net, min(args.steps, 100)) if args.pipeline else None

    line = {
        "metric": "policy-step env-frames/sec at B=1024 3x72x128 GRU-512; % MFMA/HBM roofline",
        "value": round(fps, 1), "unit": "env-frames/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if dtype == "fp32" else "bf16",
        "data": "synthetic",
        "config": {"workload": "%s: B=%d obs u8 %dx%dx%d, %s encoder, FC%d, %s%d, heads %s%s" % (
            net["name"], B, *net["obs"], net["encoder"], net["fc"], net["rnn_type"].upper(), net["rnn"],
            net["heads"], ", %d measurements -> FC%s" % (net["meas_dim"], net["meas_hidden"]) if net["meas_dim"] else ""),
            "paper_accounting_x4_frameskip_fps": round(4 * fps, 1),
            "inputs": "device-resident; host-to-device transfer excluded"},
        "roofline": roofline, "cpu_baseline": cpu}
    if pipeline is not None:
        line["pipeline"] = pipeline
    if args.loss:
        line["loss_kernels"] = measure_loss(torch, binding, wl, 200)
    print(json.dumps(line))
    pol.close()


if __name__ == "__main__":
    main()
