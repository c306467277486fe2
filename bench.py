"""Benchmark of the policy-worker step (paper, Sec. 3.1) on one MI355X.

One "step" = one sf_policy_step over a batch of synthetic observations already
resident in HBM (the standard configuration: B=1024 frames of 3x72x128 bytes,
conv encoder, FC-512, GRU-512, one 7-way head + value, fp32).  Prints one JSON
line: env-frames/s, the roofline of the dominant kernel (live HIP-event timing of
every launch, each launch scored against the peak of the arithmetic it runs on)
and the CPU oracle timed on the host cores on a bounded sample.

Timing protocol: an uncounted, time-based pre-warm-up (the clocks of an idle GPU
need a few hundred milliseconds of work to settle), then --warmup counted untimed
steps, then BLOCKS blocks of exactly --steps steps, each bracketed by a device
synchronisation; ms_per_step is the median block (min and max beside it).
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))

# MI355X dense peaks per arithmetic ("pipe") of a launch, in Tera-operations/s: fp32 MFMA (also
# the fp32 vector rate), 16-bit MFMA, int8 MFMA.  An int8 digit-plane launch executes 2 or 3
# integer multiply-adds per algorithmic one; its figure below is algorithmic work over the
# int8 peak, i.e. a lower bound of how busy the int8 pipe is.
PEAK_TOPS = {"f32": 157.3, "valu": 157.3, "bf16": 2500.0, "f16": 2500.0, "i8x2": 5000.0, "i8x3": 5000.0}
HBM_PEAK_GBPS = 8000.0


def peak_of(pipe):
    """Peak for a launch; a launch that runs two layers on two pipes ("i8x2+bf16") is held
    against the slower pipe's peak (a lower bound of its fraction)."""
    return min(PEAK_TOPS[p] for p in pipe.split("+"))

BLOCKS = 5
PREWARM_SECONDS = 0.3
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_table.txt")


def source_hash():
    """Identifies the kernels that run: sha256 over the library's sources."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2006_11751_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    h.update(open(os.path.join(ROOT, "include", "sf_policy.h"), "rb").read())
    return h.hexdigest()[:16]


def load_traffic(workload, B, ops, pipes):
    """HBM bytes per launch from the tracked table of rocprofv3 counter runs, or None when the
    table has no entry measured on these sources for this workload, batch and launch sequence."""
    try:
        text = "".join(l for l in open(TRAFFIC_TABLE) if not l.startswith("#"))
        table = json.loads(text)
    except (OSError, ValueError):
        return None, "no traffic table"
    src = source_hash()
    for e in table:
        if (e["workload"] == workload and e["B"] == B and e["source_hash"] == src and
                [o["op"] for o in e["ops"]] == [n for n, _ in ops] and [o["pipe"] for o in e["ops"]] == pipes):
            return {o["op"]: o for o in e["ops"]}, "profiles/hbm_traffic_table.txt (%s)" % e.get("profile", "")
    return None, "no table entry for these kernels (sources %s)" % src


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
        # the raw entry point with everything marshalled once: the loop below measures the two
        # launches, not the construction of their arguments
        cfg = binding.make_loss_config(hp)
        st = torch.cuda.current_stream().cuda_stream
        ptrs = [tr[k].data_ptr() for k in ("logits", "actions", "logp_mu", "values", "rewards", "dones")] + \
               [out[k].data_ptr() for k in ("vs", "adv", "loss", "dlogits", "dvalues", "workspace")]
        for _ in range(20):
            binding.sf_appo_loss(cfg, *ptrs, st)
        torch.cuda.synchronize()
        tic = time.perf_counter()
        for _ in range(reps):
            binding.sf_appo_loss(cfg, *ptrs, st)
        torch.cuda.synchronize()
        us = 1e6 * (time.perf_counter() - tic) / reps
        # the same calls recorded into a HIP graph (eight per graph) and replayed: what a learner
        # loop that captures its step pays, without the host's cost of enqueueing two launches
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(8):
                binding.sf_appo_loss(cfg, *ptrs, torch.cuda.current_stream().cuda_stream)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        tic = time.perf_counter()
        for _ in range(max(1, reps // 8)):
            graph.replay()
        torch.cuda.synchronize()
        gus = 1e6 * (time.perf_counter() - tic) / (8 * max(1, reps // 8))
        M, sumA, nh = hp["T"] * hp["N"], sum(hp["heads"]), len(hp["heads"])
        # logits and actions are read for the forward pass and again for the gradient; the rest once
        nbytes = M * (2 * (4 * sumA + 4 * nh) + 4 * 4 + 1 + 4 * 4 + 4 * sumA)
        res[name] = {"us_per_call": round(us, 2), "samples_per_s": round(M / us * 1e6, 1),
                     "algorithmic_GBps": round(nbytes / us / 1e3, 2),
                     "graph_replay_us_per_call": round(gus, 2),
                     "graph_replay_algorithmic_GBps": round(nbytes / gus / 1e3, 2)}
    return res


def measure_learner_forward(torch, binding, wl, net, w, reps):
    """The learner's forward pass on the paper's batch (64 trajectories of 32 steps = 2048 samples):
    one call of the unrolled pass, and the same work as 32 single steps of 64 rows, for comparison."""
    T, N = 32, 64
    pol = binding.Policy(net, w, max_batch=T * N)
    d = pol.device
    obs, h0, done, meas = wl.trajectory_inputs(net, T, N)
    obs, h0, done = (torch.from_numpy(a).to(d) for a in (obs, h0, done))
    meas = None if meas is None else torch.from_numpy(meas).to(d)
    out = pol.unroll(obs, h0, done, meas=meas)
    st = torch.cuda.current_stream().cuda_stream
    args = (pol.handle, T, N, obs.data_ptr(), None if meas is None else meas.data_ptr(), h0.data_ptr(), done.data_ptr(),
            out["logits"].data_ptr(), out["value"].data_ptr(), out["h_seq"].data_ptr(), st)
    for _ in range(5):
        binding.sf_policy_unroll(*args)
    torch.cuda.synchronize()
    tic = time.perf_counter()
    for _ in range(reps):
        binding.sf_policy_unroll(*args)
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - tic) / reps
    step_out = pol.alloc_outputs(N)
    hs = [h0] + [torch.empty_like(h0) for _ in range(2)]

    def steps():
        for t in range(T):
            step_out["h_out"] = hs[1 + t % 2]
            pol.step(obs[t], hs[0] if t == 0 else hs[1 + (t - 1) % 2], done[t], 1, t, out=step_out,
                     meas=None if meas is None else meas[t])
    steps()
    torch.cuda.synchronize()
    tic = time.perf_counter()
    for _ in range(max(1, reps // 4)):
        steps()
    torch.cuda.synchronize()
    ms_steps = 1e3 * (time.perf_counter() - tic) / max(1, reps // 4)
    flops = pol.flops_per_row() * T * N
    pol.close()
    return {"T": T, "N": N, "ms_per_pass": round(ms, 4), "samples_per_s": round(T * N / ms * 1e3, 1),
            "algorithmic_tflops": round(flops / ms / 1e9, 2), "as_32_single_steps_ms": round(ms_steps, 4),
            "launches": "encoder and FC once on 2048 frames, the core 32 times on 64 rows, the heads once on 2048 states"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="workload index (1 = the headline one)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (experiments)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay figure")
    ap.add_argument("--pipeline", action="store_true",
                    help="also measure the double-buffered pipeline with host-resident observations")
    ap.add_argument("--loss", action="store_true", help="also time the learner-side loss kernels and forward pass")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for HBM byte counters)")
    ap.add_argument("--profile-run", action="store_true",
                    help="for runs under rocprofv3: no pre-warm-up, one block, no per-launch event pass, "
                         "no graph, no CPU baseline; the last launches of the trace are one whole step")
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

    profile_run = args.profile_run
    t_next = 0
    prewarm_steps = 0
    if not profile_run:
        tic = time.perf_counter()
        while time.perf_counter() - tic < PREWARM_SECONDS:
            run(20, t_next)
            torch.cuda.synchronize()
            t_next += 20
        prewarm_steps = t_next
    run(args.warmup, t_next)
    t_next += args.warmup
    torch.cuda.synchronize()
    block_ms = []
    for _ in range(1 if profile_run else BLOCKS):
        tic = time.perf_counter()
        run(args.steps, t_next)
        torch.cuda.synchronize()
        block_ms.append(1e3 * (time.perf_counter() - tic) / args.steps)
        t_next += args.steps
    ms_per_step = float(np.median(block_ms))
    fps = B / (ms_per_step * 1e-3)

    ops = pol.ops()
    pipes = pol.op_pipes()
    dtype = net["dtype"]
    roofline = None
    graph = None
    if not profile_run:
        # per-launch durations: the same steps again with a HIP event after every launch, on the
        # stream the launches go to
        pol.set_op_timing(True)
        n_timed = min(args.steps, 100)
        samples = np.zeros((n_timed, len(ops)))
        for t in range(n_timed):
            run(1, t_next + t)
            samples[t] = pol.last_op_times_ms()
        t_next += n_timed
        pol.set_op_timing(False)
        event_ms = samples.mean(axis=0)
        # An event between two launches costs time of its own (the first launch must have drained
        # and its time stamp be written before the next one starts), which the untimed steps do
        # not pay: there the launches follow one another without a gap (the kernel trace's
        # durations add up to the step).  That cost, (sum of the intervals - untimed step) / number
        # of launches, is taken off every interval; the raw intervals are kept as "event_ms".
        event_cost = float(np.clip((event_ms.sum() - ms_per_step) / len(ops), 0.0, 0.5 * event_ms.min()))
        op_ms = event_ms - event_cost
        i_dom = int(np.argmax(op_ms))
        traffic, traffic_src = load_traffic(net["name"], B, ops, pipes)
        per_op = {}
        for (name, fl), pipe, ms, ems in zip(ops, pipes, op_ms, event_ms):
            tops = fl * B / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
            e = {"ms": round(float(ms), 5), "event_ms": round(float(ems), 5), "pipe": pipe, "tops": round(tops, 3),
                 "frac_of_pipe_peak": round(tops / peak_of(pipe), 5)}
            if traffic is not None:
                byts = 1024.0 * traffic[name]["hbm_kib"]
                e["hbm_bytes"] = int(byts)
                e["hbm_frac"] = round(byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 5) if ms > 0 else None
            per_op[name] = e
        dom = per_op[ops[i_dom][0]]
        whole_tops = pol.flops_per_row() * B / (ms_per_step * 1e-3) / 1e12
        # the step against a roof of its own: every launch at the peak of its pipe
        t_roof_ms = sum(fl * B / (peak_of(p) * 1e12) * 1e3 for (_, fl), p in zip(ops, pipes))
        whole = {"algorithmic_tops": round(whole_tops, 3), "ms_at_pipe_peaks": round(t_roof_ms, 5),
                 "frac": round(t_roof_ms / ms_per_step, 5)}
        f32 = [(fl, ms) for (_, fl), p, ms in zip(ops, pipes, op_ms) if p == "f32"]
        if f32:
            tf = sum(fl for fl, _ in f32) * B / (sum(ms for _, ms in f32) * 1e-3) / 1e12
            whole["fp32_mfma_launches"] = {"tflops": round(tf, 3), "frac": round(tf / PEAK_TOPS["f32"], 5),
                                           "ms": round(float(sum(ms for _, ms in f32)), 5)}
        if traffic is not None:
            hbm = sum(1024.0 * traffic[name]["hbm_kib"] for name, _ in ops) / (ms_per_step * 1e-3) / 1e9
            whole.update({"hbm_GBps": round(hbm, 1), "hbm_frac": round(hbm / HBM_PEAK_GBPS, 4)})
        roofline = {"bound": "mfma", "kernel": ops[i_dom][0], "pipe": dom["pipe"], "achieved": dom["tops"],
                    "peak": peak_of(dom["pipe"]), "unit": "TFLOP/s" if not dom["pipe"].startswith("i8") else "TOP/s",
                    "frac": dom["frac_of_pipe_peak"],
                    "traffic": dom.get("hbm_bytes"), "traffic_source": traffic_src,
                    "avg_launch_ms": dom["ms"], "event_cost_ms_per_launch": round(event_cost, 5),
                    "whole_step": whole, "per_kernel": per_op}
        if dom.get("hbm_frac") is not None:
            # the dominant launch against the other roof; it is reported against the one it is nearer to
            if dom["hbm_frac"] > roofline["frac"]:
                roofline.update({"bound": "hbm", "achieved": round(dom["hbm_bytes"] / (dom["ms"] * 1e-3) / 1e9, 1),
                                 "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": dom["hbm_frac"],
                                 "mfma_frac": dom["frac_of_pipe_peak"]})
            else:
                roofline["hbm_frac"] = dom["hbm_frac"]

        if not args.no_graph:
            # second, labelled figure: two steps (one ping-pong of the state buffers) recorded
            # into a HIP graph and replayed; launch overhead and inter-launch gaps shrink
            side = torch.cuda.Stream(device=dev)
            with torch.cuda.stream(side):
                pol.step(obs, h[0], done, wl.PHILOX_SEED, 0, out=out[0], stream=side, meas=meas)
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                s = torch.cuda.current_stream(dev)
                pol.step(obs, h[0], done, wl.PHILOX_SEED, 0, out=out[0], stream=s, meas=meas)
                pol.step(obs, h[1], done, wl.PHILOX_SEED, 1, out=out[1], stream=s, meas=meas)
            reps = max(1, args.steps // 2)
            for _ in range(5):
                g.replay()
            torch.cuda.synchronize()
            gms = []
            for _ in range(BLOCKS):
                tic = time.perf_counter()
                for _ in range(reps):
                    g.replay()
                torch.cuda.synchronize()
                gms.append(1e3 * (time.perf_counter() - tic) / (2 * reps))
            gm = float(np.median(gms))
            graph = {"ms_per_step": round(gm, 5), "value": round(B / (gm * 1e-3), 1), "unit": "env-frames/s",
                     "note": "the same step replayed from a HIP graph (seed/step arguments frozen); "
                             "not the headline value"}

    cpu = None
    if not args.no_cpu_baseline and not profile_run:
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

    p0 = pipes[0].split("+")[0]
    conv1 = {"i8x3": "int8 MFMA, 3 fixed-point digit planes (error-bound ratio %.3f)",
             "i8x2": "int8 MFMA, 2 fixed-point digit planes (admitted: error-bound ratio %.3f <= 1)",
             "f32": "fp32 MFMA (fixed-point bank not admitted: ratio %.3f)"}.get(p0)
    if conv1:
        conv1 = conv1 % pol.conv1_fixed_point_ratio(2 if p0 == "i8x2" else 3)
    line = {
        "metric": "policy-step env-frames/sec at B=1024 3x72x128 GRU-512; % MFMA/HBM roofline",
        "value": round(fps, 1), "unit": "env-frames/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if dtype == "fp32" else "bf16",
        "data": "synthetic",
        "config": {"workload": "%s: B=%d obs u8 %dx%dx%d, %s encoder, FC%d, %s%d, heads %s%s" % (
            net["name"], B, *net["obs"], net["encoder"], net["fc"], net["rnn_type"].upper(), net["rnn"],
            net["heads"], ", %d measurements -> FC%s" % (net["meas_dim"], net["meas_hidden"]) if net["meas_dim"] else ""),
            "name": net["name"], "B": B, "conv1": conv1 or pipes[0],
            "launch_pipes": dict(zip((n for n, _ in ops), pipes)),
            "launch_kernels": dict(zip((n for n, _ in ops), pol.op_kernels())),
            "paper_accounting_x4_frameskip_fps": round(4 * fps, 1),
            "inputs": "device-resident; host-to-device transfer excluded",
            "timing": "median of %d blocks of %d steps after %d uncounted pre-warm-up steps (>= %.1f s) and %d "
                      "warm-up steps" % (len(block_ms), args.steps, prewarm_steps, PREWARM_SECONDS, args.warmup),
            "ms_per_step_min": round(min(block_ms), 5), "ms_per_step_max": round(max(block_ms), 5),
            "source_hash": source_hash()},
        "roofline": roofline, "cpu_baseline": cpu}
    if graph is not None:
        line["graph_replay"] = graph
    if pipeline is not None:
        line["pipeline"] = pipeline
    if args.loss:
        line["loss_kernels"] = measure_loss(torch, binding, wl, 200)
        line["learner_forward"] = measure_learner_forward(torch, binding, wl, net, w, 40)
    print(json.dumps(line))
    pol.close()


if __name__ == "__main__":
    main()
