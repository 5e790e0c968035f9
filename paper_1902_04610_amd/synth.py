"""Seeded synthetic inputs for the five workloads.

This module only draws random numbers and packs them into arrays.  It holds
none of the method's arithmetic (no allocator, no scheduler, no GEMM) and is
the one piece of code that both the HIP path's tests and the CPU oracle's tests
feed from; neither of them is imported here.

The paper's own workloads (its 15 models, its 100-job trace, its 42 inference
models) need datasets and trained weights; the generators below keep their
structure instead: many small co-resident jobs whose persistent memory is much
smaller than their per-iteration peak, low-rate inference models, identical
architecture hyper-parameter jobs, a short urgent job preempting a long one.

All draws come from numpy's PCG64 in the order written in each function.
"""
import numpy as np

MiB = 1 << 20


def f32_to_bf16_bits(x):
    """Storage conversion for generated data: float32 -> bf16 bit patterns,
    round to nearest, ties to even (pure integer arithmetic on the bits)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(h):
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------
# workload 1: four small fp32 MLP jobs time-sharing two lanes
# --------------------------------------------------------------------------
def workload1(seed=0, jobs=4, width=256, batch=8, rounds=16):
    """Weights ~ N(0, variance 1/width), job-major then layer-major; then the
    inputs X[job][iteration] ~ U(-1, 1), job-major.  Each job runs in every
    second round, so it sees rounds/2 iterations."""
    rng = np.random.Generator(np.random.PCG64(seed))
    sigma = 1.0 / np.sqrt(width)
    W = [[(rng.standard_normal((width, width)) * sigma).astype(np.float32) for _ in range(2)]
         for _ in range(jobs)]
    iters = rounds // 2
    X = [[rng.uniform(-1.0, 1.0, (batch, width)).astype(np.float32) for _ in range(iters)]
         for _ in range(jobs)]
    return dict(W=W, X=X, width=width, batch=batch, rounds=rounds, jobs=jobs,
                capacity=4 * MiB, granule=256,
                P=2 * width * width * 4, E=1 * MiB)


# --------------------------------------------------------------------------
# workload 2: inference packing
# --------------------------------------------------------------------------
def workload2_weights(seed=1, models=64, dims=(1024, 4096, 1024, 1024), sigma=0.02):
    """Per model, per layer: W ~ N(0, sigma) stored as bf16, shape (K, N)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for _ in range(models):
        layers = []
        for K, N in zip(dims[:-1], dims[1:]):
            w = rng.standard_normal((K, N), dtype=np.float32)
            w *= np.float32(sigma)
            layers.append(f32_to_bf16_bits(w))
        out.append(layers)
    return out


def workload2_arrivals(seed=1, models=64, rounds=220, tick_s=4.0, max_batch=32):
    """Request rates lambda_m = exp(N(0,1)) req/s; arrivals per round
    ~ Poisson(lambda_m * tick).  Returns (rates, arrivals[rounds][models]).
    Drawn from a generator of its own (seed + 1000) so that the traffic does
    not depend on the model sizes."""
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    rates = np.exp(rng.standard_normal(models))
    arrivals = rng.poisson(rates * tick_s, size=(rounds, models)).astype(np.int64)
    return rates, arrivals


def workload2_inputs(seed, model, round_, batch, width):
    """Requests of one model in one round: X ~ N(0,1) as bf16, shape (batch, width).
    Keyed by (seed, model, round) so any sample can be regenerated alone."""
    rng = np.random.Generator(np.random.PCG64([seed, 2000 + model, round_]))
    return f32_to_bf16_bits(rng.standard_normal((batch, width), dtype=np.float32))


# --------------------------------------------------------------------------
# workload 3: hyper-parameter tuning (training) jobs
# --------------------------------------------------------------------------
def workload3(seed=2, jobs=8, dims=(2048, 2048, 2048, 2048, 1000), batch=64, steps=4):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = dict(dims=dims, batch=batch, jobs=jobs, steps=steps, Wm=[], lr=[], X=[], labels=[])
    for _ in range(jobs):
        out['Wm'].append([(rng.standard_normal((K, N), dtype=np.float32)
                           * np.float32(1.0 / np.sqrt(K))).astype(np.float32)
                          for K, N in zip(dims[:-1], dims[1:])])
    out['lr'] = (10.0 ** rng.uniform(-4.0, -1.0, jobs)).astype(np.float32)
    for _ in range(jobs):
        out['X'].append([f32_to_bf16_bits(rng.standard_normal((batch, dims[0]), dtype=np.float32))
                         for _ in range(steps)])
        out['labels'].append([rng.integers(0, dims[-1], batch).astype(np.int32)
                              for _ in range(steps)])
    return out


# --------------------------------------------------------------------------
# workloads 4 and 5: byte patterns and job traces
# --------------------------------------------------------------------------
def pattern_bytes(seed, nbytes):
    """Random persistent state (weights + optimizer moments are just bytes here)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, 256, nbytes, dtype=np.uint8)


def workload5_trace(seed=4, rounds=2000, arrival_rate=0.08, mean_life=200,
                    p_median=1e9, p_sigma=0.8, e_median=2e9, e_sigma=0.5, scale=1.0,
                    initial_jobs=16):
    """Job trace: ``initial_jobs`` present at round 0, then Poisson arrivals per
    round; each job lives a geometric number of rounds after admission.  Sizes
    are lognormal, multiplied by ``scale`` (1/1024 gives the MB-sized replica).
    Returns a list of dicts sorted by arrival round."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n_new = rng.poisson(arrival_rate, rounds)
    n_new[0] += initial_jobs
    trace = []
    for r in range(rounds):
        for _ in range(int(n_new[r])):
            P = int(rng.lognormal(np.log(p_median), p_sigma) * scale)
            E = int(rng.lognormal(np.log(e_median), e_sigma) * scale)
            life = int(rng.geometric(1.0 / mean_life))
            trace.append(dict(arrive=r, P=max(P, 1), E=max(E, 1), life=life))
    return trace


def workload_trace100(seed=6, jobs=100, load=0.9):
    """Stand-in for the 100-job training trace of Section 5.1.1 (the trace itself is
    not available): most jobs are short and a few are long, as in the production
    cluster the paper refers to.  All times are integer milliseconds.

    Per job: arrival, persistent bytes P (lognormal, median 0.5 GB), ephemeral peak E
    (lognormal, median 2 GB), iterations, cost = duration of one scheduling
    quantum of the job when it has the GPU to itself, util = share of the GPU it
    keeps busy while it runs (per mille).  Arrivals are Poisson with a rate that
    makes the offered load `load` of one GPU used by one job at a time."""
    rng = np.random.Generator(np.random.PCG64(seed))
    dur_ms = np.clip(rng.lognormal(np.log(8 * 60e3), 1.3, jobs), 60e3, 4 * 3600e3)
    cost_ms = np.clip(rng.lognormal(np.log(10e3), 0.6, jobs), 2e3, 60e3).astype(np.int64)
    iters = np.maximum(1, np.round(dur_ms / cost_ms)).astype(np.int64)
    P = (np.clip(rng.lognormal(np.log(0.5e9), 0.8, jobs), 5e7, 4e9) // 256 * 256).astype(np.int64)
    E = (np.clip(rng.lognormal(np.log(2e9), 0.5, jobs), 2e8, 8e9) // 256 * 256).astype(np.int64)
    util = rng.integers(200, 901, jobs)
    work = int((iters * cost_ms).sum())
    gaps = rng.exponential(work / load / jobs, jobs)
    arrival = np.floor(np.cumsum(gaps) - gaps[0]).astype(np.int64)
    return [dict(arrival=int(arrival[i]), P=int(P[i]), E=int(E[i]), iters=int(iters[i]),
                 cost=int(cost_ms[i]), util=int(util[i])) for i in range(jobs)]
