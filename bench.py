#!/usr/bin/env python3
"""Benchmark of the packed-iteration hot path on one MI355X.

Workload = the inference-packing configuration: 64 resident 3-layer MLPs
(1024 -> 4096 -> 1024 -> 1024, GELU, bf16 weights ~ N(0, 0.02), float
accumulation), Poisson request arrivals with per-model rates lognormal(0, 1)
req/s sampled every 4 s tick, requests batched to 1..32 per model and round.
One step = one scheduling round: pending flags -> salus_schedule_iteration ->
salus_grouped_forward (one grouped launch per layer depth).  All inputs are in
HBM before the timed region.

The weights are stored in the library's 128-column strips (--row-major for the
plain layout); values and results are the same either way.

Prints ONE JSON line; `value` is TFLOP/s with flops = 2*M*K*N of the true batch
sizes.  Extra objects: roofline (HBM-bound weight streaming; traffic = profiler
byte counters from the committed summary of this command), saturated (all 64
models at batch 32), cpu_baseline (the CPU oracle on a bounded sample of the same
rounds), switch (evict / restore / compaction bandwidth, and the same switch
overlapped with running lanes), training (packed training step of 8 jobs),
small_case_latency (the 4-job correctness configuration, per round) and
batch_sweep (supplemental: the same 64 models at 32 .. 4096 rows each).
"""
import argparse
import ctypes
import json
import os
import sys
import time
import types

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

DIMS = (1024, 4096, 1024, 1024)
MODELS = 64
MAX_BATCH = 32
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
MiB = 1 << 20
W_OFFS = (0, DIMS[0] * DIMS[1] * 2, DIMS[0] * DIMS[1] * 2 + DIMS[1] * DIMS[2] * 2)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def packing(torch, np, salus, synth, stream, K_steps, W_steps, fused):
    """Workload 2 resident in a pool of its own: returns the handles and a
    `run(plans, batches, label)` that times K_steps rounds after W_steps."""
    dev = torch.device("cuda:0")
    rounds = W_steps + K_steps
    # ---------------------------------------------------------------- set-up (untimed)
    up = lambda v: (v + 255) // 256 * 256
    w_sizes = [k * n * 2 for k, n in zip(DIMS[:-1], DIMS[1:])]
    w_offs = [0, w_sizes[0], w_sizes[0] + w_sizes[1]]
    P = sum(w_sizes)
    x_off, y_off = 0, up(MAX_BATCH * DIMS[0] * 2)
    h_off = y_off + up(MAX_BATCH * DIMS[-1] * 4)
    E = up(h_off + salus.forward_work_bytes(
        MAX_BATCH, [(k, n, 0, 0) for k, n in zip(DIMS[:-1], DIMS[1:])], salus.BF16))
    cap = MODELS * (P + E)
    buf = torch.empty(cap, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    pool = salus.Pool(buf.data_ptr(), cap, policy=salus.POLICY_PACK, stream=stream, fuse_depths=fused)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    lane_off = []
    for m in range(MODELS):
        st, j = pool.lane_alloc(P, E, 0, 0)
        assert st == salus.OK and j == m
        q = pool.job_query(m)
        lane_off.append(q.lane_off)
        for (k, n), off in zip(zip(DIMS[:-1], DIMS[1:]), w_offs):
            w = (torch.randn(k, n, generator=gen, device=dev) * 0.02).to(torch.bfloat16)
            buf[q.persist_off + off:q.persist_off + off + k * n * 2].copy_(stored(w))
        x = torch.randn(MAX_BATCH, DIMS[0], generator=gen, device=dev).to(torch.bfloat16)
        buf[q.lane_off + x_off:q.lane_off + x_off + x.numel() * 2].copy_(x.view(torch.uint8).reshape(-1))
    torch.cuda.synchronize()

    rates, arrivals = synth.workload2_arrivals(seed=1, models=MODELS, rounds=rounds)
    layers = layer_list(salus)

    def plan(batches_per_round):
        """Per round: pending flags and job descriptors, marshalled before the clock starts."""
        out = []
        for b in batches_per_round:
            act = [m for m in range(MODELS) if b[m] > 0]
            flags = (ctypes.c_uint64 * MODELS)(*[1 if b[m] > 0 else 0 for m in range(MODELS)])
            descs, keep = salus.Pool.make_descs(
                dict(job=m, M=int(b[m]), dtype=salus.BF16, layers=layers, x_off=x_off, y_off=y_off,
                     h_off=h_off) for m in act)
            out.append((flags, descs, keep, len(act)))
        return out

    waiting = np.zeros(MODELS, np.int64)
    batches = []
    for r in range(rounds):
        waiting += arrivals[r]
        b = np.minimum(waiting, MAX_BATCH)
        waiting -= b
        batches.append(b)
    poisson = plan(batches)
    saturated = plan([np.full(MODELS, MAX_BATCH)] * rounds)
    job_ids = (ctypes.c_int32 * MODELS)(*range(MODELS))
    slots = (salus.Slot * MODELS)()
    mac_per_row = sum(k * n for k, n in zip(DIMS[:-1], DIMS[1:]))
    act_bytes_per_row = 2 * DIMS[0] + sum(2 * n for n in DIMS[1:-1]) * 2 + 4 * DIMS[-1]

    def run(plans, batches_per_round, label):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(K_steps)]

        def step(r, timed_idx=None):
            flags, descs, keep, n_act = plans[r]
            pool.set_pending_many(job_ids, flags, MODELS)
            n = pool.schedule_into(slots, MODELS)
            assert n == n_act
            if timed_idx is not None:
                ev[timed_idx][0].record()
            rc = pool.grouped_forward(descs, n_act, stream)
            assert rc == salus.OK, pool.last_error()
            if timed_idx is not None:
                ev[timed_idx][1].record()

        for r in range(W_steps):
            step(r)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(K_steps):
            step(W_steps + i, i)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        kernel_ms = sum(a.elapsed_time(b) for a, b in ev)
        rows = sum(int(b.sum()) for b in batches_per_round[W_steps:])
        active = sum(int((b > 0).sum()) for b in batches_per_round[W_steps:])
        flops = 2.0 * mac_per_row * rows
        alg_bytes = active * P + rows * act_bytes_per_row
        assert pool.fused_check() == salus.OK, pool.last_error()
        launches = (1 if fused else 3) * K_steps
        res = dict(tflops=flops / wall / 1e12, ms_per_step=wall / K_steps * 1e3,
                   kernel_ms_per_launch=kernel_ms / launches,
                   gbs=alg_bytes / (kernel_ms * 1e-3) / 1e9,
                   bytes_per_launch=alg_bytes / launches,
                   mean_active=active / K_steps, mean_batch=rows / max(active, 1))
        log(f"[{label}] {res}")
        return res


    return types.SimpleNamespace(pool=pool, buf=buf, cap=cap, P=P, w_offs=w_offs, w_sizes=w_sizes, batches=batches,
                                 poisson=poisson, saturated=saturated, run=run, mac_per_row=mac_per_row)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-switch", action="store_true", help="skip the evict/restore/compaction figures")
    ap.add_argument("--no-training", action="store_true", help="skip the packed training-step figures")
    ap.add_argument("--hot-only", action="store_true", help="only the timed packed-iteration loop (for profiling)")
    ap.add_argument("--poisson-only", action="store_true",
                    help="with --hot-only: leave out the saturated rounds (for the traffic counters)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the supplemental batch-size sweep")
    ap.add_argument("--sweep-only", action="store_true", help="only the supplemental batch-size sweep")
    ap.add_argument("--overlap-only", action="store_true", help="only the overlapped-switching figures")
    ap.add_argument("--row-major", action="store_true",
                    help="store the weights row-major instead of in 128-column strips")
    ap.add_argument("--fused", action="store_true",
                    help="time the depth-fused forward (one launch per round) as the main path, for profiling")
    ap.add_argument("--switch-only", action="store_true",
                    help="only evict / restore / compaction (for profiling)")
    ap.add_argument("--latency-only", action="store_true", help="only the small-case latency, both launch modes")
    ap.add_argument("--train-only", action="store_true", help="only the packed training step (for profiling)")
    ap.add_argument("--calibrate", action="store_true",
                    help="only the calibration: one 2048 x 2048 bf16 layer of J jobs per launch, J = 2 .. 64, at 32 "
                         "and 64 rows (how the streaming rate depends on the number of workgroups), and a plain copy")
    args = ap.parse_args()
    global STRIP
    STRIP = not args.row_major
    fused = args.fused
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (jobs are packed inside one device); "
                 "--gpus must be 1")

    import numpy as np
    import torch
    from paper_1902_04610_amd import salus, synth

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.calibrate:
        torch.cuda.set_device(0)
        print(json.dumps(calibration_figures(torch, salus, torch.cuda.current_stream().cuda_stream)))
        return
    if args.train_only:
        torch.cuda.set_device(0)
        print(json.dumps(training_figures(torch, salus, torch.cuda.current_stream().cuda_stream,
                                          with_cpu=not args.no_cpu_baseline)))
        return
    if args.switch_only:
        torch.cuda.set_device(0)
        print(json.dumps(switch_figures(torch, salus, torch.cuda.current_stream().cuda_stream,
                                        with_cpu=not args.no_cpu_baseline)))
        return
    if args.latency_only:
        torch.cuda.set_device(0)
        st = torch.cuda.current_stream().cuda_stream
        print(json.dumps([latency_figures(torch, salus, synth, st, fused=f) for f in (False, True)]))
        return
    if args.overlap_only:
        torch.cuda.set_device(0)
        print(json.dumps(overlap_figures(torch, salus, torch.cuda.current_stream().cuda_stream)))
        return
    if args.sweep_only:
        torch.cuda.set_device(0)
        print(json.dumps(sweep_figures(torch, salus, torch.cuda.current_stream().cuda_stream)))
        return
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K_steps, W_steps = args.steps, args.warmup
    rounds = W_steps + K_steps

    S = packing(torch, np, salus, synth, torch.cuda.current_stream().cuda_stream, K_steps, W_steps, fused)
    pool, buf, cap, P, w_offs, w_sizes, batches = S.pool, S.buf, S.cap, S.P, S.w_offs, S.w_sizes, S.batches
    poisson, saturated, run, mac_per_row = S.poisson, S.saturated, S.run, S.mac_per_row
    stream = torch.cuda.current_stream().cuda_stream
    log(f"pool {cap / 1e9:.2f} GB, {MODELS} models resident, {rounds} rounds planned")
    main_res = run(poisson, batches, "poisson")
    if args.hot_only:
        sat = None if args.poisson_only else run(saturated, [np.full(MODELS, MAX_BATCH)] * rounds, "saturated")
        # a plain copy of known size in the same process: scale for profiler byte counters
        cal = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
        for _ in range(3):
            salus.copy(cal.data_ptr(), cal.data_ptr() + (1 << 30), 1 << 30, stream)
        torch.cuda.synchronize()
        del cal
    else:
        sat = run(saturated, [np.full(MODELS, MAX_BATCH)] * rounds, "saturated")

    out = {
        "metric": "packed grouped-GEMM TFLOP/s (% MFMA peak) + job-switch ms/GB (% HBM BW)",
        "value": round(main_res["tflops"], 3), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": K_steps, "warmup": W_steps,
        "ms_per_step": round(main_res["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "inference packing: 64 resident 3-layer MLPs 1024-4096-1024-1024 GELU, "
                               "bf16 weights, Poisson arrivals (rates lognormal(0,1) req/s, 4 s tick), "
                               "batch 1-32, PACK policy, one grouped launch per layer depth; weights stored "
                               + ("in 128-column strips" if STRIP else "row-major"),
                   "mean_active_models": round(main_res["mean_active"], 2),
                   "mean_batch": round(main_res["mean_batch"], 2),
                   "pct_of_bf16_mfma_peak": round(100 * main_res["tflops"] / MFMA_BF16_PEAK_TFLOPS, 3)},
        "roofline": {"bound": "hbm", "achieved": round(main_res["gbs"], 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(main_res["gbs"] / HBM_PEAK_GBS, 4),
                     "traffic": profiled_traffic(K_steps, W_steps, main_res["bytes_per_launch"]),
                     "kernel": "chained_dense" if fused else "grouped_dense_bf16",
                     "avg_launch_ms": round(main_res["kernel_ms_per_launch"], 5),
                     "algorithmic_bytes_per_launch": int(main_res["bytes_per_launch"])},
    }
    if sat:
        out["saturated"] = {"workload": "same 64 models, every model at batch 32 every round",
                            "tflops": round(sat["tflops"], 2), "ms_per_step": round(sat["ms_per_step"], 4),
                            "hbm_gbs": round(sat["gbs"], 1), "hbm_frac": round(sat["gbs"] / HBM_PEAK_GBS, 4),
                            "pct_of_bf16_mfma_peak": round(100 * sat["tflops"] / MFMA_BF16_PEAK_TFLOPS, 3),
                            "avg_launch_ms": round(sat["kernel_ms_per_launch"], 5)}

    # ---------------------------------------------------------------- CPU oracle on a sample
    if not args.no_cpu_baseline and not args.hot_only:
        from concurrent.futures import ThreadPoolExecutor
        from oracle import dense
        dense.lib()
        cores = min(16, os.cpu_count() or 1)
        sample_rounds = min(4, K_steps)
        work = []
        for r in range(W_steps, W_steps + sample_rounds):
            for m in range(MODELS):
                if batches[r][m] > 0:
                    work.append((m, int(batches[r][m])))
        host_w = {}
        for m in sorted({m for m, _ in work}):
            q = pool.job_query(m)
            blob = buf[q.persist_off:q.persist_off + P].cpu().numpy()
            unstrip = lambda a, k, n: (np.ascontiguousarray(a.reshape(n // 128, k, 128).transpose(1, 0, 2))
                                       .reshape(k, n) if STRIP else a.reshape(k, n))
            host_w[m] = [unstrip(blob[o:o + s].view(np.uint16), k, n)
                         for o, s, (k, n) in zip(w_offs, w_sizes, zip(DIMS[:-1], DIMS[1:]))]
            host_w[m].append(buf[q.lane_off:q.lane_off + MAX_BATCH * DIMS[0] * 2].cpu().numpy()
                             .view(np.uint16).reshape(MAX_BATCH, DIMS[0]))
        acts = [dense.ACT_GELU, dense.ACT_GELU, dense.ACT_NONE]

        def one(item):
            m, b = item
            return dense.mlp_forward_bf16(host_w[m][3][:b], host_w[m][:3], acts)[-1]

        t0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            list(ex.map(one, work))
        cpu_s = time.perf_counter() - t0
        cpu_flops = 2.0 * mac_per_row * sum(b for _, b in work)
        out["cpu_baseline"] = {"value": round(cpu_flops / cpu_s / 1e12, 6), "unit": "TFLOP/s",
                               "cores": cores, "kind": "oracle",
                               "sample": f"the first {sample_rounds} timed rounds of the same workload "
                                         f"({len(work)} model forwards, {cpu_flops / 2e9:.2f} GMAC), "
                                         f"{cpu_s:.1f} s wall on {cores} threads"}
        log(f"[cpu] {out['cpu_baseline']}")
        # the same oracle on one thread: the first timed round (about a quarter of the work above)
        single, rows_1 = [], 0
        for item in work:
            if rows_1 >= sum(b for _, b in work) // 4:
                break
            single.append(item)
            rows_1 += item[1]
        t0 = time.perf_counter()
        for item in single:
            one(item)
        one_s = time.perf_counter() - t0
        out["cpu_baseline_single_thread"] = {
            "value": round(2.0 * mac_per_row * rows_1 / one_s / 1e12, 6), "unit": "TFLOP/s", "cores": 1,
            "kind": "oracle", "sample": f"the first {len(single)} model forwards of the same rounds "
                                        f"({mac_per_row * rows_1 / 1e9:.2f} GMAC), {one_s:.1f} s wall on 1 thread"}
        log(f"[cpu 1 thread] {out['cpu_baseline_single_thread']}")
    pool.close()
    del buf
    torch.cuda.empty_cache()

    # ---------------------------------------------------------------- switch path
    if not args.no_switch and not args.hot_only:
        out["switch"] = switch_figures(torch, salus, stream, with_cpu=not args.no_cpu_baseline)
        out["switch"]["overlapped"] = overlap_figures(torch, salus, stream)
    if not args.no_training and not args.hot_only:
        out["training"] = training_figures(torch, salus, stream, with_cpu=not args.no_cpu_baseline)
    if not args.hot_only:
        out["small_case_latency"] = latency_figures(torch, salus, synth, stream)
    if not args.no_sweep and not args.hot_only:
        out["batch_sweep"] = sweep_figures(torch, salus, stream)
    if not args.hot_only and not fused:
        # the same rounds as one depth-fused launch each (SALUS_FLAG_FUSE_DEPTHS), for comparison
        F = packing(torch, np, salus, synth, stream, K_steps, W_steps, True)
        fp = F.run(F.poisson, F.batches, "fused poisson")
        fs = F.run(F.saturated, [np.full(MODELS, MAX_BATCH)] * len(F.batches), "fused saturated")
        out["fused_depths"] = {"what": "the same workload with one launch per round: tiles of layer l+1 wait on "
                                       "device counters for their job's layer l (bit-identical outputs)",
                               "ms_per_step": round(fp["ms_per_step"], 4), "hbm_gbs": round(fp["gbs"], 1),
                               "saturated_ms_per_step": round(fs["ms_per_step"], 4),
                               "saturated_hbm_gbs": round(fs["gbs"], 1),
                               "per_depth_ms_per_step": round(main_res["ms_per_step"], 4)}
        F.pool.close()
    print(json.dumps(out), flush=True)


def training_figures(torch, salus, stream, jobs=8, dims=(2048, 2048, 2048, 2048, 1000), M=64,
                     steps=50, warmup=5, with_cpu=True):
    """Hyper-parameter-tuning packing: 8 training jobs of one architecture, one
    packed step = schedule + forward + loss + backward + SGD for all of them."""
    up = lambda v: (v + 255) // 256 * 256
    layers, off = [], 0
    for k, n in zip(dims[:-1], dims[1:]):
        layers.append((k, n, off, off + up(k * n * 2)))
        off += up(k * n * 2) + up(k * n * 4)
    P = off
    x_off, labels_off = 0, up(M * dims[0] * 2)
    logits_off = labels_off + up(M * 4)
    loss_off = logits_off + up(M * dims[-1] * 4)
    work_off = loss_off + 256
    E = up(work_off + salus.train_work_bytes(M, layers))
    cap = jobs * (P + E)
    buf = torch.empty(cap, dtype=torch.uint8, device="cuda:0")
    pool = salus.Pool(buf.data_ptr(), cap, policy=salus.POLICY_PACK, stream=stream)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(2)
    items = []
    for j in range(jobs):
        st, jid = pool.lane_alloc(P, E, 0, 10 ** 9)
        assert st == salus.OK
        q = pool.job_query(jid)
        for k, n, wb, wm in layers:
            w = torch.randn(k, n, generator=gen, device="cuda:0") * (1.0 / k ** 0.5)
            buf[q.persist_off + wm:q.persist_off + wm + k * n * 4].copy_(w.view(torch.uint8).reshape(-1))
            buf[q.persist_off + wb:q.persist_off + wb + k * n * 2].copy_(
                w.to(torch.bfloat16).view(torch.uint8).reshape(-1))
        x = torch.randn(M, dims[0], generator=gen, device="cuda:0").to(torch.bfloat16)
        y = torch.randint(0, dims[-1], (M,), generator=gen, device="cuda:0", dtype=torch.int32)
        buf[q.lane_off + x_off:q.lane_off + x_off + M * dims[0] * 2].copy_(x.view(torch.uint8).reshape(-1))
        buf[q.lane_off + labels_off:q.lane_off + labels_off + M * 4].copy_(y.view(torch.uint8).reshape(-1))
        lr = 10.0 ** (-4.0 + 3.0 * j / max(jobs - 1, 1))          # log-spaced in [1e-4, 1e-1]
        items.append(dict(job=jid, M=M, lr=lr, layers=layers, x_off=x_off, labels_off=labels_off,
                          logits_off=logits_off, loss_off=loss_off, work_off=work_off))
    descs, keep = salus.Pool.make_train_descs(items)
    slots = (salus.Slot * jobs)()

    def step():
        assert pool.schedule_into(slots, jobs) == jobs
        assert pool.grouped_train_step(descs, jobs, stream) == salus.OK

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    params = sum(k * n for k, n, _, _ in layers)
    flops = jobs * 2.0 * M * (3 * params - layers[0][0] * layers[0][1])
    # bf16 weights read by forward and by the input gradient (not layer 1), master read + written,
    # bf16 copy rewritten; activations are a few MB and left out
    alg_bytes = jobs * (2 * params + 2 * (params - layers[0][0] * layers[0][1]) + 8 * params + 2 * params)
    loss = buf[pool.job_query(0).lane_off + loss_off:][:4].view(torch.float32).item()
    res = {"workload": f"{jobs} training jobs, MLP {'-'.join(map(str, dims))}, batch {M}, bf16 + float master, SGD",
           "ms_per_step": round(wall * 1e3, 4), "tflops": round(flops / wall / 1e12, 2),
           "hbm_gbs": round(alg_bytes / wall / 1e9, 1), "hbm_frac": round(alg_bytes / wall / 1e9 / HBM_PEAK_GBS, 4),
           "launches_per_step": 9, "loss_job0_after": round(loss, 4)}
    log(f"[training] {res}")
    pool.close()
    del buf
    if with_cpu:
        res.update(training_cpu_baseline(dims, M, jobs))
    return res


def training_cpu_baseline(dims, M, jobs):
    """The oracle's training step (oracle/train.py as it stands) on the host: one
    job-step on one thread, then one step of all jobs on a thread per job."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import dense, train
    from paper_1902_04610_amd import synth
    dense.lib()
    rng = np.random.Generator(np.random.PCG64(2))
    params = sum(k * n for k, n in zip(dims[:-1], dims[1:]))
    flops = 2.0 * M * (3 * params - dims[0] * dims[1])

    def make():
        Wm = [(rng.standard_normal((k, n), dtype=np.float32) * np.float32(1 / np.sqrt(k)))
              for k, n in zip(dims[:-1], dims[1:])]
        Wb = [synth.f32_to_bf16_bits(w) for w in Wm]
        X = synth.f32_to_bf16_bits(rng.standard_normal((M, dims[0]), dtype=np.float32))
        y = rng.integers(0, dims[-1], M).astype(np.int32)
        return X, y, Wm, Wb

    state = [make() for _ in range(jobs)]
    t0 = time.perf_counter()
    train.train_step(*state[0], 1e-3)
    one_s = time.perf_counter() - t0
    cores = min(jobs, os.cpu_count() or 1)
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        list(ex.map(lambda st: train.train_step(*st, 1e-3), state))
    all_s = time.perf_counter() - t0
    out = {"cpu_baseline_single_thread": {"value": round(flops / one_s / 1e12, 6), "unit": "TFLOP/s", "cores": 1,
                                          "kind": "oracle", "sample": f"one job-step ({flops / 1e9:.2f} GFLOP), "
                                                                      f"{one_s:.1f} s wall"},
           "cpu_baseline": {"value": round(jobs * flops / all_s / 1e12, 6), "unit": "TFLOP/s", "cores": cores,
                            "kind": "oracle", "sample": f"one packed step of all {jobs} jobs, a thread per job, "
                                                        f"{all_s:.1f} s wall"}}
    log(f"[training cpu] {out}")
    return out


def calibration_figures(torch, salus, stream, K=2048, N=2048, max_jobs=64, sets=3):
    """What one launch of the weight-streaming kernel reaches as a function of its
    size: J jobs, each one K x N bf16 layer, J = 2 .. 64, at 32 rows (128-column
    tiles) and at 64 rows.  Weight sets rotate so that every launch reads HBM.
    Context for the small launches of the training step; not a workload."""
    up = lambda v: (v + 255) // 256 * 256
    P = sets * K * N * 2
    x_off, y_off = 0, up(64 * K * 2)
    E = up(y_off + 64 * N * 4)
    cap = max_jobs * (P + E)
    buf = torch.empty(cap, dtype=torch.uint8, device="cuda:0")
    buf.view(torch.bfloat16).normal_(0, 0.02)
    pool = salus.Pool(buf.data_ptr(), cap, policy=salus.POLICY_PACK, stream=stream)
    for m in range(max_jobs):
        st, j = pool.lane_alloc(P, E, 0, 10 ** 9)
        assert st == salus.OK and j == m
    rows = []
    for M in (32, 64):
        for J in (2, 4, 8, 16, 32, 64):
            descs = [salus.Pool.make_descs(dict(job=m, M=M, dtype=salus.BF16, x_off=x_off, y_off=y_off, h_off=0,
                                                layers=[(K, N, s * K * N * 2, salus.ACT_RELU)]) for m in range(J))
                     for s in range(sets)]
            reps = 30
            for s in range(sets):
                assert pool.grouped_forward(descs[s][0], J, stream) == salus.OK, pool.last_error()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for r in range(reps):
                assert pool.grouped_forward(descs[r % sets][0], J, stream) == salus.OK
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) * 1e3 / reps
            tile_cols = 128 if M <= 32 or J * (N // 128) >= 256 else 64
            wgs = J * (N // tile_cols) * (2 if M > 32 and tile_cols == 128 else 1)
            rows.append({"rows": M, "jobs": J, "workgroups": wgs, "us_per_launch": round(us, 2),
                         "weight_MB": round(J * K * N * 2 / 1e6, 1), "hbm_gbs": round(J * K * N * 2 / us / 1e3, 1)})
            log(f"[calibrate] {rows[-1]}")
    pool.close()
    del buf
    torch.cuda.empty_cache()
    n = 8 << 30
    cal = torch.empty(2 * n, dtype=torch.uint8, device="cuda:0")
    best = None
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        salus.copy(cal.data_ptr(), cal.data_ptr() + n, n, stream)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    out = {"workload": f"calibration: one {K} x {N} bf16 layer of J jobs per launch; 8 GiB plain copy; "
                       "the LDS-tiled kernel's multiply without its memory traffic",
           "launches": rows, "copy_GBs_read_plus_write": round(2 * n / best / 1e9, 1)}
    log(f"[calibrate] copy {out['copy_GBs_read_plus_write']} GB/s read + write")
    # a kernel that only loads: what the read path delivers to a pure stream
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    salus.calibrate_read(cal.data_ptr(), n, sink.data_ptr(), stream)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(5):
        salus.calibrate_read(cal.data_ptr(), n, sink.data_ptr(), stream)
    b.record()
    torch.cuda.synchronize()
    out["read_only_GBs"] = round(5 * n / (a.elapsed_time(b) * 1e-3) / 1e9, 1)
    log(f"[calibrate] load-only kernel over 8 GiB: {out['read_only_GBs']} GB/s")
    del cal
    # what the matrix pipes sustain on nonzero operands, and at which clock
    clk = torch.zeros(3, dtype=torch.int64, device="cuda:0")
    out["mfma"] = []
    for from_lds in (False, True):
        salus.calibrate_mfma(clk.data_ptr(), 256, from_lds, stream)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        flop = salus.calibrate_mfma(clk.data_ptr(), 8192, from_lds, stream)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b)
        cycles, ticks = (int(v) for v in clk[:2].tolist())
        row = {"operands": "read from LDS every k-step, one barrier per slab" if from_lds else "held in registers",
               "ms": round(ms, 3), "tflops": round(flop / (ms * 1e-3) / 1e12, 1),
               "pct_of_bf16_mfma_peak": round(100 * flop / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 1),
               "shader_clock_MHz": round(100.0 * cycles / max(ticks, 1))}
        out["mfma"].append(row)
        log(f"[calibrate] mfma {row}")
    # the vendor library on the sweep's largest point: 64 independent products of the three layer
    # shapes at 4096 rows (torch.bmm, bf16 in, bf16 out, no activation) - a yardstick, not the product
    out["vendor_bmm"] = []
    rows_ = 4096
    for K, N in zip(DIMS[:-1], DIMS[1:]):
        xa = torch.randn(MODELS, rows_, K, device="cuda:0").to(torch.bfloat16)
        wa = (torch.randn(MODELS, K, N, device="cuda:0") * 0.02).to(torch.bfloat16)
        for _ in range(2):
            torch.bmm(xa, wa)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            torch.bmm(xa, wa)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / 5
        row = {"K": K, "N": N, "rows": rows_, "ms": round(ms, 3),
               "tflops": round(2.0 * MODELS * rows_ * K * N / (ms * 1e-3) / 1e12, 1)}
        out["vendor_bmm"].append(row)
        log(f"[calibrate] vendor bmm {row}")
        del xa, wa
    return out


def sweep_figures(torch, salus, stream, batches=(32, 48, 64, 80, 96, 112, 128, 256, 512, 1024, 2048, 4096)):
    """Supplemental, NOT the headline workload: the same 64 resident models with
    every model at M rows per round, M from the packing regime (weight stream
    bound) up to 4096 rows per model (compute bound), to show where the grouped
    kernel leaves the bandwidth roof and what share of the MFMA peak it reaches."""
    up = lambda v: (v + 255) // 256 * 256
    Mmax = max(batches)
    w_sizes = [k * n * 2 for k, n in zip(DIMS[:-1], DIMS[1:])]
    w_offs = [0, w_sizes[0], w_sizes[0] + w_sizes[1]]
    P = sum(w_sizes)
    x_off, y_off = 0, up(Mmax * DIMS[0] * 2)
    h_off = y_off + up(Mmax * DIMS[-1] * 4)
    E = up(h_off + salus.forward_work_bytes(
        Mmax, [(k, n, 0, 0) for k, n in zip(DIMS[:-1], DIMS[1:])], salus.BF16))
    cap = MODELS * (P + E)
    buf = torch.empty(cap, dtype=torch.uint8, device="cuda:0")
    pool = salus.Pool(buf.data_ptr(), cap, policy=salus.POLICY_PACK, stream=stream)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(11)
    for m in range(MODELS):
        st, j = pool.lane_alloc(P, E, 0, 10 ** 9)
        assert st == salus.OK and j == m
        q = pool.job_query(m)
        for (k, n), off in zip(zip(DIMS[:-1], DIMS[1:]), w_offs):
            w = (torch.randn(k, n, generator=gen, device="cuda:0") * 0.02).to(torch.bfloat16)
            buf[q.persist_off + off:q.persist_off + off + k * n * 2].copy_(stored(w))
        x = torch.randn(Mmax, DIMS[0], generator=gen, device="cuda:0").to(torch.bfloat16)
        buf[q.lane_off + x_off:q.lane_off + x_off + x.numel() * 2].copy_(x.view(torch.uint8).reshape(-1))
    layers = layer_list(salus)
    mac_per_row = sum(k * n for k, n in zip(DIMS[:-1], DIMS[1:]))
    act_bytes_per_row = 2 * DIMS[0] + sum(2 * n for n in DIMS[1:-1]) * 2 + 4 * DIMS[-1]
    rows = []
    for M in batches:
        descs, keep = salus.Pool.make_descs(
            dict(job=m, M=M, dtype=salus.BF16, layers=layers, x_off=x_off, y_off=y_off, h_off=h_off)
            for m in range(MODELS))
        reps = 20 if M <= 512 else 5
        for _ in range(2):
            assert pool.grouped_forward(descs, MODELS, stream) == salus.OK, pool.last_error()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            assert pool.grouped_forward(descs, MODELS, stream) == salus.OK
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        tf = 2.0 * mac_per_row * M * MODELS / (ms * 1e-3) / 1e12
        gbs = MODELS * (P + M * act_bytes_per_row) / (ms * 1e-3) / 1e9
        rows.append({"M": M, "ms": round(ms, 4), "tflops": round(tf, 1),
                     "pct_of_bf16_mfma_peak": round(100 * tf / MFMA_BF16_PEAK_TFLOPS, 2),
                     "hbm_gbs": round(gbs, 1)})
        log(f"[sweep] {rows[-1]}")
    pool.close()
    return {"workload": "supplemental: same 64 models, every model at M rows per round "
                        "(forward only, 3 grouped launches)", "points": rows}


STRIP = True      # weights stored in 128-column strips (set False by --row-major)


def stored(w):
    """The bytes of a K x N bf16 weight tensor in the layout the benchmark stores:
    the library's 128-column strips (same values, contiguous per column tile) or row-major."""
    if STRIP:
        k, n = w.shape
        w = w.view(k, n // 128, 128).permute(1, 0, 2).contiguous()
    return w.view(__import__("torch").uint8).reshape(-1)


def layer_list(salus):
    return [(k, n, off, act, salus.LAYOUT_STRIP128 if STRIP else salus.LAYOUT_ROWMAJOR)
            for (k, n), off, act in zip(zip(DIMS[:-1], DIMS[1:]), W_OFFS,
                                        (salus.ACT_GELU, salus.ACT_GELU, salus.ACT_NONE))]


def profiled_traffic(steps, warmup, algorithmic_bytes_per_launch):
    """HBM bytes per launch of the dominant kernel as the profiler's counters saw
    them (FETCH_SIZE + WRITE_SIZE, each scaled by a copy of known size), taken from
    the committed summary of the same workload.  The summary holds one line per
    profiled command (--steps / --warmup); a run with other values gets the
    summary's counted / algorithmic ratio applied to its own algorithmic bytes."""
    path = os.path.join(ROOT, "profiles", "grouped_dense_bf16_inference_packing.txt")
    ratio = None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                f = dict(kv.split("=") for kv in line.split()[1:])
                if int(f["steps"]) == steps and int(f["warmup"]) == warmup:
                    return int(f["bytes"])
                ratio = int(f["bytes"]) / float(f["algorithmic"]) if "algorithmic" in f else ratio
    except (OSError, KeyError, ValueError):
        pass
    return None if ratio is None else int(ratio * algorithmic_bytes_per_launch)


def latency_figures(torch, salus, synth, stream, rounds=2000, fused=False):
    """The small correctness configuration (4 jobs, two 256 x 256 float layers,
    batch 8, two lanes, round-robin): far too small for bandwidth or flops to
    mean anything, so it is reported as latency per scheduling round."""
    w = synth.workload1(seed=0)
    width, batch = w["width"], w["batch"]
    buf = torch.zeros(w["capacity"], dtype=torch.uint8, device="cuda:0")
    pool = salus.Pool(buf.data_ptr(), w["capacity"], granule=w["granule"], policy=salus.POLICY_FAIR,
                      stream=stream, fuse_depths=fused)
    wbytes, items = width * width * 4, []
    for j in range(w["jobs"]):
        st, jid = pool.lane_alloc(w["P"], w["E"], 0, 10 ** 9)
        assert st == salus.OK
        q = pool.job_query(jid)
        for l in range(2):
            t = torch.from_numpy(w["W"][j][l]).to("cuda:0")
            buf[q.persist_off + l * wbytes:q.persist_off + (l + 1) * wbytes].copy_(t.view(torch.uint8).reshape(-1))
        x = torch.from_numpy(w["X"][j][0]).to("cuda:0")
        buf[q.lane_off:q.lane_off + x.numel() * 4].copy_(x.view(torch.uint8).reshape(-1))
        items.append(dict(job=jid, M=batch, dtype=salus.F32, x_off=0, y_off=batch * width * 4,
                          h_off=2 * batch * width * 4,
                          layers=[(width, width, 0, salus.ACT_RELU), (width, width, wbytes, salus.ACT_NONE)]))
    by_job = {it["job"]: it for it in items}
    descs = {}
    slots = (salus.Slot * 8)()

    def one_round():
        n = pool.schedule_into(slots, 8)
        key = tuple(slots[i].job for i in range(n))
        if key not in descs:
            descs[key] = salus.Pool.make_descs([by_job[j] for j in key])
        assert pool.grouped_forward(descs[key][0], n, stream) == salus.OK
        return n

    for _ in range(50):
        one_round()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(rounds):
        one_round()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / rounds
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    lat = []
    for _ in range(200):                      # one round at a time: launch + execution latency
        a.record()
        one_round()
        b.record()
        b.synchronize()
        lat.append(a.elapsed_time(b))
    lat.sort()
    res = {"workload": "4 jobs, two 256 x 256 float layers, batch 8, two lanes, round-robin (2 jobs per round)",
           "us_per_round_back_to_back": round(wall * 1e6, 2),
           "us_per_round_gpu_median": round(lat[len(lat) // 2] * 1e3, 2), "launches_per_round": 1 if fused else 2}
    assert pool.fused_check() == salus.OK
    log(f"[latency] {res}")
    pool.close()
    return res


def overlap_figures(torch, salus, stream, blob_gb=8, batch=MAX_BATCH):
    """Overlapped switching: an 8 GB job leaves and comes back on a copy stream
    while the 64 inference models keep running packed rounds on the pool's stream.
    Reports the round time and the link rate, each alone and together."""
    up = lambda v: (v + 255) // 256 * 256
    w_sizes = [k * n * 2 for k, n in zip(DIMS[:-1], DIMS[1:])]
    w_offs = [0, w_sizes[0], w_sizes[0] + w_sizes[1]]
    P = sum(w_sizes)
    x_off, y_off = 0, up(batch * DIMS[0] * 2)
    h_off = y_off + up(batch * DIMS[-1] * 4)
    E = up(h_off + salus.forward_work_bytes(
        batch, [(k, n, 0, 0) for k, n in zip(DIMS[:-1], DIMS[1:])], salus.BF16))
    blob = blob_gb * 10 ** 9 // 256 * 256
    cap = MODELS * (P + E) + blob + 4096
    buf = torch.empty(cap, dtype=torch.uint8, device="cuda:0")
    buf[:MODELS * P].view(torch.bfloat16).normal_(0, 0.02)
    pool = salus.Pool(buf.data_ptr(), cap, policy=salus.POLICY_PACK, stream=stream)
    layers = layer_list(salus)
    for m in range(MODELS):
        st, j = pool.lane_alloc(P, E, 0, 10 ** 9)
        assert st == salus.OK and j == m
        q = pool.job_query(m)
        buf[q.lane_off:q.lane_off + batch * DIMS[0] * 2].view(torch.bfloat16).normal_(0, 1)
    st, bj = pool.lane_alloc(blob, 4096, 0, 0)
    assert st == salus.OK
    salus.fill_pattern(buf.data_ptr() + pool.job_query(bj).persist_off, blob, 77, stream)
    descs, keep = salus.Pool.make_descs(
        dict(job=m, M=batch, dtype=salus.BF16, layers=layers, x_off=x_off, y_off=y_off, h_off=h_off)
        for m in range(MODELS))
    slots = (salus.Slot * (MODELS + 1))()
    copy_stream = torch.cuda.Stream()
    cs = copy_stream.cuda_stream

    def one_round():
        assert pool.schedule_into(slots, MODELS + 1) == MODELS
        assert pool.grouped_forward(descs, MODELS, stream) == salus.OK

    def rounds_alone(n=200):
        for _ in range(20):
            one_round()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            one_round()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    def transfer(begin, end, with_rounds):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        assert begin() == salus.OK
        n = 0
        if with_rounds:
            while end(False) == salus.EBUSY:
                for _ in range(8):
                    one_round()
                n += 8
                torch.cuda.current_stream().synchronize()     # keep the host at most 8 rounds ahead
            dt = time.perf_counter() - t0
        else:
            assert end(True) == salus.OK
            dt = time.perf_counter() - t0
        torch.cuda.synchronize()
        return dt, n

    out_b = lambda: pool.switch_out_begin(bj, cs)
    out_e = lambda w: pool.switch_out_end(bj, w)
    in_b = lambda: pool.switch_in_begin(bj, cs)
    in_e = lambda w: pool.switch_in_end(bj, w)
    transfer(out_b, out_e, False)                  # first eviction allocates the pinned buffer: untimed
    transfer(in_b, in_e, False)
    alone = rounds_alone()
    t_out, _ = transfer(out_b, out_e, False)
    t_in, _ = transfer(in_b, in_e, False)
    t_out_ov, n_out = transfer(out_b, out_e, True)
    t_in_ov, n_in = transfer(in_b, in_e, True)
    scratch = torch.zeros(8, dtype=torch.uint8, device="cuda:0")
    bad = salus.check_pattern(buf.data_ptr() + pool.job_query(bj).persist_off, blob, 77,
                              scratch.data_ptr(), stream)
    res = {"workload": f"{blob_gb} GB job switched out and in on a copy stream; 64 models at batch {batch} "
                       "run packed rounds meanwhile",
           "round_ms_alone": round(alone * 1e3, 4),
           "round_ms_during_evict": round(t_out_ov / max(n_out, 1) * 1e3, 4),
           "round_ms_during_restore": round(t_in_ov / max(n_in, 1) * 1e3, 4),
           "evict_GBs_alone": round(blob / t_out / 1e9, 2), "evict_GBs_overlapped": round(blob / t_out_ov / 1e9, 2),
           "restore_GBs_alone": round(blob / t_in / 1e9, 2),
           "restore_GBs_overlapped": round(blob / t_in_ov / 1e9, 2),
           "rounds_during_evict": n_out, "rounds_during_restore": n_in,
           "bytes_wrong_after_round_trips": int(bad)}
    log(f"[overlap] {res}")
    pool.close()
    return res


def switch_figures(torch, salus, stream, with_cpu=True):
    """The job-switch path at the sizes of the priority-preemption and
    fragmentation workloads: evict / restore of a 20 GB job over the host link with
    both engines (best of 2 after the repetition that allocates the pinned buffer),
    and on-device compaction on four plans, each verified with the device pattern:
    three 8 GB blocks that move by their own length (independent segments), one
    8 GB block that moves by 256 bytes and one that moves by 40 MiB (both overlap
    their own destination: the in-place kernel), and the forced compaction of the
    fragmentation workload (about 200 GB of blocks drawn from its size distribution,
    a seeded random half freed).  ms/GB counts GB = 1e9 bytes of payload moved;
    HBM traffic = read + write = 2 x payload."""
    import numpy as np
    GB = 10 ** 9
    res = {}
    scratch = torch.zeros(8, dtype=torch.uint8, device="cuda:0")

    def verify(buf, off, nbytes, seed):
        return salus.check_pattern(buf.data_ptr() + off, nbytes // 8 * 8, seed, scratch.data_ptr(), stream)

    P = 20 * GB // 256 * 256
    for name, engine in (("kernel", salus.COPY_KERNEL), ("dma", salus.COPY_DMA)):
        torch.cuda.empty_cache()
        buf = torch.empty(P + 2 * MiB, dtype=torch.uint8, device="cuda:0")
        pool = salus.Pool(buf.data_ptr(), P + 2 * MiB, stream=stream, copy_engine=engine)
        st, j = pool.lane_alloc(P, MiB, 0, 1)
        salus.fill_pattern(buf.data_ptr(), P, 7, stream)
        out_ms, in_ms = [], []
        for rep in range(3):                      # the first repetition allocates the pinned buffer
            t0 = time.perf_counter()
            assert pool.switch_out(j) == salus.OK
            t1 = time.perf_counter()
            assert pool.switch_in(j) == salus.OK
            t2 = time.perf_counter()
            if rep:
                out_ms.append((t1 - t0) * 1e3)
                in_ms.append((t2 - t1) * 1e3)
        assert verify(buf, pool.job_query(j).persist_off, P, 7) == 0
        res[f"evict_{name}_ms_per_GB"] = round(min(out_ms) / (P / GB), 3)
        res[f"restore_{name}_ms_per_GB"] = round(min(in_ms) / (P / GB), 3)
        res[f"evict_{name}_GBs"] = round(P / GB / (min(out_ms) * 1e-3), 2)
        res[f"restore_{name}_GBs"] = round(P / GB / (min(in_ms) * 1e-3), 2)
        pool.close()
        del buf
    res["switch_bytes_per_call"] = P

    def timed_compaction(sizes, free, cap, reps, label):
        """Blocks of `sizes` bytes are placed in order, those listed in `free` leave, then compact()."""
        torch.cuda.empty_cache()
        buf = torch.empty(cap, dtype=torch.uint8, device="cuda:0")
        best, moved, launches = None, 0, 0
        for rep in range(reps):
            pool = salus.Pool(buf.data_ptr(), cap, stream=stream, max_lanes=1)
            ids = [pool.lane_alloc(sz, MiB, 0, 1)[1] for sz in sizes]
            keep = [k for k in range(len(sizes)) if k not in free]
            for k in keep:
                salus.fill_pattern(buf.data_ptr() + pool.job_query(ids[k]).persist_off, sizes[k] // 8 * 8, 100 + k, stream)
            for k in free:
                pool.lane_free(ids[k])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            plan = pool.compact()
            dt = time.perf_counter() - t0
            moved = sum(m[2] for m in plan)
            for k in keep:
                assert verify(buf, pool.job_query(ids[k]).persist_off, sizes[k], 100 + k) == 0, (label, k)
            best = dt if best is None else min(best, dt)
            pool.close()
        del buf
        out = {"ms_per_GB_moved": round(best * 1e3 / (moved / GB), 4),
               "hbm_GBs_read_plus_write": round(2 * moved / best / 1e9, 1),
               "hbm_frac": round(2 * moved / best / 1e9 / HBM_PEAK_GBS, 4),
               "bytes_moved": moved, "moves": len(plan)}
        log(f"[compact {label}] {out}")
        return out

    blk = 8 * GB // 256 * 256
    indep = timed_compaction([blk] * 4, {0}, 4 * blk + 2 * MiB, 3, "independent 3 x 8 GB")
    res["compact_ms_per_GB_moved"] = indep["ms_per_GB_moved"]
    res["compact_hbm_GBs_read_plus_write"] = indep["hbm_GBs_read_plus_write"]
    res["compact_hbm_frac"] = indep["hbm_frac"]
    res["compact_bytes_moved"] = indep["bytes_moved"]
    res["compact_shift_256B"] = timed_compaction([256, blk], {0}, blk + 256 + 2 * MiB, 3, "8 GB by 256 B (in place)")
    res["compact_shift_40MiB"] = timed_compaction([40 * MiB, blk], {0}, blk + 42 * MiB, 3, "8 GB by 40 MiB (in place)")
    # forced compaction of the fragmentation workload
    rng = np.random.Generator(np.random.PCG64(44))
    sizes, total = [], 0
    while True:
        sz = int(rng.lognormal(np.log(1e9), 0.8)) // 256 * 256 + 256
        if total + sz > 200 * GB:
            break
        sizes.append(sz)
        total += sz
    free = set(int(k) for k in rng.permutation(len(sizes))[:len(sizes) // 2])
    forced = timed_compaction(sizes, free, 204 * GB // 256 * 256, 1, f"forced, {len(sizes)} blocks, {total / 1e9:.0f} GB")
    forced["blocks"] = len(sizes)
    res["compact_forced_200GB"] = forced
    torch.cuda.empty_cache()

    if with_cpu:
        # the oracle's switch is a memcpy out of and into its byte array: timed on a 2 GB job
        from oracle import pool as op
        n = 2 * GB // 256 * 256
        mem = np.zeros(n + MiB, np.uint8)
        o = op.Pool(n + MiB, mem=mem)
        o.job_arrive(n, MiB // 2)
        mem[:n:4096] = 1                              # touch the pages
        t0 = time.perf_counter()
        assert o.switch_out(0) == op.OK
        t1 = time.perf_counter()
        assert o.switch_in(0) == op.OK
        t2 = time.perf_counter()
        res["cpu_baseline"] = {"evict_ms_per_GB": round((t1 - t0) * 1e3 / (n / GB), 2),
                               "restore_ms_per_GB": round((t2 - t1) * 1e3 / (n / GB), 2),
                               "unit": "ms/GB", "cores": 1, "kind": "oracle",
                               "sample": "switch_out + switch_in of a 2 GB job in the oracle's host byte array "
                                         "(a tenth of the 20 GB job)"}
        # and its compaction plan for the forced case (metadata only: no host mirror of 200 GB exists)
        o = op.Pool(204 * GB // 256 * 256, max_lanes=1)
        for sz in sizes:
            o.job_arrive(sz, MiB)
        for k in sorted(free):
            o.job_finish(k)
        t0 = time.perf_counter()
        plan = o.compact()
        res["cpu_baseline"]["forced_plan_ms"] = round((time.perf_counter() - t0) * 1e3, 3)
        res["cpu_baseline"]["forced_plan_moves"] = len(plan)
        assert sum(m[2] for m in plan) == forced["bytes_moved"]
        log(f"[switch cpu] {res['cpu_baseline']}")
    log(f"[switch] { {k: v for k, v in res.items() if not isinstance(v, dict)} }")
    return res


if __name__ == "__main__":
    main()
